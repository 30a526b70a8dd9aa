"""Full-size parity of the MoE, backward and MLA configurations in the launch
configuration `bench.py` times: the oracle computes sampled rows / columns of
the outputs one by one on the very codes and scales the GPU quantizers wrote
(those are bit-checked against the oracle at full size in test_gpu_quant.py and
at reduced sizes for every layout).  BF16 outputs are held to the normwise bar
and, element by element, to "the rounded reference or its neighbour"."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from synth import workloads as wl
from tests._gpu_util import announce, bf16_elementwise, dev, host, magnitude_sum, normwise

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL_F32 = 1e-4
BF16_IDENTICAL = 0.96


def _check_bf16(what, got, a, sa, b, sb, identical=BF16_IDENTICAL):
    """Normwise bar, and element by element: half a BF16 ulp of output rounding plus the
    accumulation bound, with nearly all outputs equal to the rounded reference."""
    ref = orc.gemm_fp8_bs(a, sa, b, sb)
    e = normwise(got, ref)
    excess, same = bf16_elementwise(got, ref, magnitude_sum(a, sa, b, sb))
    print(f"{what}: normwise {e:.3e}; worst (|err| - accumulation bound) = {excess:.3f} BF16 ulp; {100 * same:.2f}% equal the rounded reference")
    assert e <= TOL_BF16, what
    assert excess <= 0.5 and same >= identical, what


def _expert_weights(g, shape, tensor_index, sampled, expert_fn, ids=None):
    """Device BF16 [g][shape]: the sampled experts from the config's seeded numpy generator, the
    rest drawn on the device (same distribution) to keep the set-up short."""
    gen = torch.Generator(device="cuda:0").manual_seed(wl.seed_for(3, tensor_index))
    w = (torch.randn((g,) + shape, generator=gen, device="cuda:0") * 0.02).to(torch.bfloat16)
    for e in sampled:
        w[e] = dev(expert_fn(e if ids is None else ids[e]), bf16=True)
    return w


def _moe_pipeline(ds3, sizes, off, sampled, ids=None, tag="cfg3"):
    """quantize -> grouped gate|up -> fused SwiGLU + quantize -> grouped down at full width, every
    stage checked on the inputs it actually received."""
    G, H, I = len(sizes), wl.HIDDEN, wl.MOE_INTER
    rows = int(off[-1])
    x = wl.cfg3_tokens(rows)
    qx, sx = ds3.ds3_quant_act_1x128(dev(x, bf16=True))
    del x
    w13 = _expert_weights(G, (2 * I, H), 2, sampled, wl.cfg3_w13_expert, ids)
    q13, s13 = ds3.ds3_quant_w_128x128(w13.view(G * 2 * I, H))
    q13v, s13v = q13.view(G, 2 * I, H), s13.view(G, 2 * I // 128, H // 128)
    # the weight quantizer on the generator's own data, one expert bit for bit
    e0 = sampled[0]
    q_ref, s_ref = orc.quant_w_128x128(host(w13[e0]))
    assert np.array_equal(host(q13v[e0]), q_ref) and np.array_equal(host(s13v[e0]), s_ref)
    del w13
    h = ds3.ds3_grouped_gemm_fp8_bs(qx, sx, dev(off), q13v, s13v)
    h_h, qx_h, sx_h = host(h), host(qx), host(sx)
    rng = np.random.default_rng(46)
    picks = {}
    for e in sampled:
        lo, hi = int(off[e]), int(off[e + 1])
        if hi == lo:
            continue
        picks[e] = np.unique(np.concatenate([[lo, hi - 1, min(lo + 255, hi - 1), min(lo + 256, hi - 1)], rng.integers(lo, hi, 4)]))
        _check_bf16(f"{tag} gate|up expert {e} ({hi - lo} rows)", h_h[picks[e]], qx_h[picks[e]], sx_h[picks[e]], host(q13v[e]), host(s13v[e]))
    # the same projection with SwiGLU and the cast in its epilogue (gate|up rows interleaved in
    # blocks of 128): compared below with the codes the two separate kernels give
    q13i = q13v.view(G, 2, I // 128, 128, H).transpose(1, 2).contiguous().view(G, 2 * I, H)
    s13i = s13v.view(G, 2, I // 128, H // 128).transpose(1, 2).contiguous().view(G, 2 * I // 128, H // 128)
    qh_e, sh_e = ds3.ds3_grouped_gemm_swiglu_quant_fp8_bs(qx, sx, dev(off), q13i, s13i)
    del q13, s13, q13v, s13v, q13i, s13i
    # SwiGLU fused with the 1x128 quantizer, on the GPU's own H.  Staged parity: the activation
    # ds3_swiglu writes is within one BF16 ulp of the FP64 SwiGLU of H, and the fused kernel's codes
    # and scales equal, bit for bit, the oracle's quantization of that BF16 activation (the codes
    # are decided from BF16 values; against the all-FP64 composition a one-ulp difference in an
    # activation may move a code, so there the agreement is statistical).
    qh, sh = ds3.ds3_swiglu_quant_1x128(h)
    act = host(ds3.ds3_swiglu(h))
    ref_act = orc.swiglu(h_h)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref_act), 2.0 ** -120))) - 7)
    assert np.all(np.abs(act - ref_act) <= ulp), f"{tag}: SwiGLU beyond one BF16 ulp"
    qh_ref, sh_ref = orc.quant_act_1x128(act)
    assert np.array_equal(host(qh), qh_ref), f"{tag}: fused SwiGLU->quant codes"
    assert np.array_equal(host(sh), sh_ref), f"{tag}: fused SwiGLU->quant scales"
    assert np.array_equal(host(qh_e)[:rows], qh_ref), f"{tag}: SwiGLU->quant in the GEMM epilogue, codes"
    assert np.array_equal(host(sh_e)[:rows], sh_ref), f"{tag}: SwiGLU->quant in the GEMM epilogue, scales"
    del qh_e, sh_e
    q_all, s_all = orc.swiglu_quant_1x128(h_h)
    assert np.mean(qh_ref == q_all) > 0.98 and np.mean(sh_ref == s_all) > 0.9
    del act, ref_act, ulp, q_all, s_all
    del h, h_h
    # down projection [n_e x 2048] . [7168 x 2048]^T
    w2 = _expert_weights(G, (H, I), 3, sampled, wl.cfg3_w2_expert, ids)
    q2, s2 = ds3.ds3_quant_w_128x128(w2.view(G * H, I))
    del w2
    q2v, s2v = q2.view(G, H, I), s2.view(G, H // 128, I // 128)
    y = host(ds3.ds3_grouped_gemm_fp8_bs(qh, sh, dev(off), q2v, s2v))
    for e, pick in picks.items():
        _check_bf16(f"{tag} down expert {e}", y[pick], qh_ref[pick], sh_ref[pick], host(q2v[e]), host(s2v[e]))
    return y


def test_cfg3_moe_full_size_sampled(ds3):
    """32 local experts, the real routing (120 .. 440 rows per expert), full width: gate|up
    [n_e x 7168] x [4096 x 7168]^T, SwiGLU + quantizer, down [n_e x 2048] x [7168 x 2048]^T."""
    announce("cfg3 full size sampled")
    sizes, off, _ = wl.cfg3_routing()
    sampled = sorted({0, 1, 7, 16, 31, int(np.argmin(sizes)), int(np.argmax(sizes))})
    _moe_pipeline(ds3, sizes, off, sampled)


def test_cfg3_stress_routing_full_width(ds3):
    """The stress variant: per-expert bias of sigma 0.05, the 16 least and the 16 most loaded of
    the 256 experts: empty groups, groups of a few rows and groups of about a thousand."""
    announce("cfg3 stress routing")
    ids = wl.cfg3_stress_experts()
    sizes, off, _ = wl.cfg3_routing(sigma_b=0.05, experts=ids)
    assert sizes.min() == 0 and sizes.max() > 1000
    order = np.argsort(sizes, kind="stable")
    nonempty = [int(e) for e in order if sizes[e] > 0]
    sampled = sorted({nonempty[0], nonempty[1], nonempty[len(nonempty) // 2], nonempty[-1], nonempty[-2],
                      int(order[0]) + 1 if int(order[0]) + 1 < len(sizes) else 0, len(sizes) - 1} & set(range(len(sizes))))
    y = _moe_pipeline(ds3, sizes, off, sampled, ids=ids, tag="cfg3 stress")
    assert y.shape[0] == int(off[-1])


def test_cfg4_wgrad_full_size_sampled(ds3):
    """dW[18432 x 7168] += dY^T X over 4096 tokens, both operands 128x1, FP32 accumulate; sampled output rows."""
    announce("cfg4 wgrad full size sampled")
    x, dy = wl.cfg2_x(), wl.cfg4_dy()
    qyt, syt = ds3.ds3_quant_act_128x1(dev(dy, bf16=True))
    qxt, sxt = ds3.ds3_quant_act_128x1(dev(x, bf16=True))
    del x, dy
    dw = torch.full((wl.DENSE_INTER, wl.HIDDEN), 0.25, dtype=torch.float32, device="cuda:0")
    ds3.ds3_gemm_fp8_bs(qyt, syt, qxt, sxt, sb_mode=ds3.DS3_BSCALE_PER_ROW, c=dw, accumulate=True)
    rng = np.random.default_rng(47)
    pick = np.unique(np.concatenate([[0, 255, 256, 18431], rng.integers(0, wl.DENSE_INTER, 12)]))
    ref = orc.gemm_fp8_bs(host(qyt)[pick], host(syt)[pick], host(qxt), host(sxt), sb_per_row=True,
                          c_in=np.full((len(pick), wl.HIDDEN), 0.25))
    e = normwise(host(dw[torch.from_numpy(pick).to("cuda:0")]), ref)
    print(f"cfg4 wgrad sampled: {e:.3e}")
    assert e <= TOL_F32


def test_cfg4_dgrad_full_size_sampled(ds3):
    """dX[4096 x 7168] = dY W with the weight codes taken from the dual-layout quantizer of W."""
    announce("cfg4 dgrad full size sampled")
    dy = wl.cfg4_dy()
    qdy, sdy = ds3.ds3_quant_act_1x128(dev(dy, bf16=True))
    del dy
    _, _, qwt, swt = ds3.ds3_quant_w_128x128_dual(dev(wl.cfg2_w(), bf16=True))
    dx = host(ds3.ds3_gemm_fp8_bs(qdy, sdy, qwt, swt))
    rng = np.random.default_rng(48)
    pick = np.unique(np.concatenate([[0, 4095], rng.integers(0, 4096, 10)]))
    _check_bf16("cfg4 dgrad sampled", dx[pick], host(qdy)[pick], host(sdy)[pick], host(qwt), host(swt))


def test_cfg5_mla_full_size_sampled(ds3):
    for idx, (name, m, n, k) in enumerate(wl.cfg5_shapes()):
        announce(f"cfg5 {name} full size sampled")
        x, w = wl.cfg5_act(m, k, idx), wl.cfg5_w(n, k, idx)
        qa, sa = ds3.ds3_quant_act_1x128(dev(x, bf16=True))
        qb, sb = ds3.ds3_quant_w_128x128(dev(w, bf16=True))
        del x, w
        c = ds3.ds3_gemm_fp8_bs(qa, sa, qb, sb)
        rng = np.random.default_rng(49 + idx)
        pick = np.unique(np.concatenate([[0, m - 1], rng.integers(0, m, 8)]))
        _check_bf16(f"cfg5 {name} {m}x{n}x{k}", host(c[torch.from_numpy(pick).to("cuda:0")]), host(qa)[pick], host(sa)[pick], host(qb), host(sb))


def test_cfg2_cfg4_pow2_full_size_sampled(ds3):
    """The power-of-two path at the benchmark's sizes: Fprop 4096 x 18432 x 7168 (BF16 and FP32 out) and
    Wgrad 18432 x 7168 x 4096 with per-row scales and FP32 accumulation, scales applied by the matrix
    instruction; quantizer outputs bit for bit, GEMM outputs on sampled rows."""
    announce("cfg2/cfg4 pow2 full size sampled")
    x, w = wl.cfg2_x(), wl.cfg2_w()
    qa, sa = ds3.ds3_quant_act_1x128_pow2(dev(x, bf16=True))
    qb, sb = ds3.ds3_quant_w_128x128_pow2(dev(w, bf16=True))
    rng = np.random.default_rng(49)
    rows = np.unique(np.concatenate([[0, 255, 256, 4095], rng.integers(0, 4096, 12)]))
    q_ref, s_ref = orc.quant_act_1x128(x[rows], pow2=True)
    qa_h, sa_h, qb_h, sb_h = host(qa), host(sa), host(qb), host(sb)
    assert np.array_equal(qa_h[rows], q_ref) and np.array_equal(sa_h[rows], s_ref)
    qw_ref, sw_ref = orc.quant_w_128x128(w[:256], pow2=True)
    assert np.array_equal(qb_h[:256], qw_ref) and np.array_equal(sb_h[:2], sw_ref)
    del w
    c = host(ds3.ds3_gemm_fp8_bs_pow2(qa, sa, qb, sb))
    # (the matrix unit adds every block's sum to the running FP32 total itself: its accumulation error is
    # carried along K instead of being renewed per block, and a little more of the outputs land on the other
    # side of a BF16 rounding boundary: 96.4% identical here against 97-99% on the general path)
    _check_bf16("cfg2 pow2 sampled rows", c[rows], qa_h[rows], sa_h[rows], qb_h, sb_h, identical=0.94)
    c32 = ds3.ds3_gemm_fp8_bs_pow2(qa, sa, qb, sb, out_dtype=torch.float32)
    e32 = normwise(host(c32[torch.from_numpy(rows).to("cuda:0")]), orc.gemm_fp8_bs(qa_h[rows], sa_h[rows], qb_h, sb_h))
    print(f"cfg2 pow2 FP32 out: {e32:.3e}")
    assert e32 <= TOL_F32
    del c, c32, qa, sa, qb, sb
    # Wgrad
    dy = wl.cfg4_dy()
    qyt, syt = ds3.ds3_quant_act_128x1_pow2(dev(dy, bf16=True))
    qxt, sxt = ds3.ds3_quant_act_128x1_pow2(dev(x, bf16=True))
    del x, dy
    dw = torch.full((wl.DENSE_INTER, wl.HIDDEN), 0.25, dtype=torch.float32, device="cuda:0")
    ds3.ds3_gemm_fp8_bs_pow2(qyt, syt, qxt, sxt, sb_mode=ds3.DS3_BSCALE_PER_ROW, c=dw, accumulate=True)
    pick = np.unique(np.concatenate([[0, 255, 256, 18431], rng.integers(0, wl.DENSE_INTER, 12)]))
    ref = orc.gemm_fp8_bs(host(qyt)[pick], host(syt)[pick], host(qxt), host(sxt), sb_per_row=True,
                          c_in=np.full((len(pick), wl.HIDDEN), 0.25))
    e = normwise(host(dw[torch.from_numpy(pick).to("cuda:0")]), ref)
    print(f"cfg4 pow2 wgrad sampled: {e:.3e}")
    assert e <= TOL_F32
