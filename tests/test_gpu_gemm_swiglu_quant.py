"""GPU parity of the grouped gate|up GEMM whose epilogue applies SwiGLU and the
1x128 quantizer (Sections 3.3.2 and 3.3.3: the down projection's input is the
SwiGLU output in FP8, cast where it is produced).

The oracle's composition is GEMM -> round to BF16 -> SwiGLU -> round to BF16 ->
1x128 quantization.  Its stages are checked where they can be checked exactly:
  * the GEMM stage against the oracle GEMM (norm-wise, and exactly with
    small-integer codes and power-of-two scales);
  * the quantizer stage bit for bit against the oracle quantizer applied to the
    BF16 activation that the GPU's SwiGLU gives on the BF16-rounded FP32 output
    of the same GEMM (the activation itself is within one BF16 ulp of the
    oracle's, which a max-abs cast does not survive bit for bit);
  * the fused call as a whole bit for bit against the unfused calls.
"""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from synth import workloads as wl
from tests._gpu_util import announce, dev, host, normwise

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TABLE = np.array([0x00, 0x38, 0x40, 0xB8, 0xC0, 0x80], dtype=np.uint8)  # 0, 1, 2, -1, -2, -0


def _rand_codes(rng, shape):
    c = rng.integers(0, 0x7F, size=shape).astype(np.uint8)
    return c | (rng.integers(0, 2, size=shape) << 7).astype(np.uint8)


def _kmajor(s: np.ndarray) -> torch.Tensor:
    return dev(np.ascontiguousarray(s.T)).t()


def _check(ds3, a, sa, off, b, sb, pow2, what):
    """a [rows][K] codes, b [G][2I][K] codes in gate|up order, sb their block scales."""
    g, two_i, k = b.shape
    inter, total = two_i // 2, int(off[-1])
    fused = ds3.ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2 if pow2 else ds3.ds3_grouped_gemm_swiglu_quant_fp8_bs
    gemm = ds3.ds3_grouped_gemm_fp8_bs_pow2 if pow2 else ds3.ds3_grouped_gemm_fp8_bs
    swq = ds3.ds3_swiglu_quant_1x128_pow2 if pow2 else ds3.ds3_swiglu_quant_1x128
    ad, sad, offd = dev(a), _kmajor(sa), dev(off)
    bi, sbi = dev(wl.interleave_gate_up(b)), dev(wl.interleave_gate_up(sb, block=1))
    announce(f"{what}: fused call")
    q, s = fused(ad, sad, offd, bi, sbi)
    q, s = host(q), host(s)
    # the unfused calls on the weight in gate|up order
    announce(f"{what}: unfused calls")
    h = gemm(ad, sad, offd, dev(b), dev(sb), variant=0)
    q2, s2 = swq(h[:total])
    assert np.array_equal(q[:total], host(q2)) and np.array_equal(s[:total], host(s2)), what
    # GEMM stage against the oracle
    ref_h = orc.grouped_gemm_fp8_bs(a[:total], sa[:total], off, b, sb)
    assert normwise(host(h)[:total], ref_h) <= TOL_BF16
    # quantizer stage: oracle cast of the BF16 activation of the BF16-rounded FP32 output of the same GEMM
    h32 = host(gemm(ad, sad, offd, dev(b), dev(sb), out_dtype=torch.float32, variant=0))[:total]
    h16 = orc.round_to_bf16(h32)
    assert np.array_equal(h16, host(h)[:total].astype(np.float64))
    act = ds3.ds3_swiglu(dev(h16.astype(np.float32), bf16=True))
    ref_act = orc.swiglu(h16)
    # (one BF16 ulp; the hardware reciprocal flushes the subnormal 1 / (1 + e^-g) of g near -88 to zero,
    # an absolute error below 2^-100 for the magnitudes here)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref_act), 2.0 ** -100))) - 7)
    assert np.all(np.abs(host(act) - ref_act) <= ulp)
    q_ref, s_ref = orc.quant_act_1x128(host(act), pow2=pow2)
    assert np.array_equal(q[:total], q_ref) and np.array_equal(s[:total], s_ref), what
    return q, s


@pytest.mark.parametrize("pow2", [False, True])
def test_ragged_groups(ds3, pow2):
    rng = np.random.default_rng(71)
    sizes = [3, 0, 300, 129, 0, 1, 257, 128, 130]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    total, inter, k, g = int(off[-1]), 384, 512, len(sizes)
    a, b = _rand_codes(rng, (total, k)), _rand_codes(rng, (g, 2 * inter, k))
    if pow2:
        sa = np.ldexp(1.0, rng.integers(-14, -9, (total, k // 128))).astype(np.float32)
        sb = np.ldexp(1.0, rng.integers(-12, -8, (g, 2 * inter // 128, k // 128))).astype(np.float32)
    else:   # h of the order of 1 to 10, as a gate|up projection's output is
        sa = (np.exp(0.5 * rng.standard_normal((total, k // 128))) * 2.0 ** -11).astype(np.float32)
        sb = (np.exp(0.5 * rng.standard_normal((g, 2 * inter // 128, k // 128))) * 2.0 ** -10).astype(np.float32)
    _check(ds3, a, sa, off, b, sb, pow2, f"ragged groups pow2={pow2}")


def test_exact_gemm_stage_and_untouched_rows(ds3):
    """Small-integer codes and power-of-two scales: h is exact, so the fused result is the oracle
    cast of the GPU's activation of the ORACLE's h; rows beyond the last group keep their contents."""
    announce("fused SwiGLU epilogue: exact GEMM stage")
    rng = np.random.default_rng(72)
    sizes = [255, 256, 2, 0, 511]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    total, inter, k, g = int(off[-1]), 256, 384, len(sizes)
    extra = 7
    a, b = TABLE[rng.integers(0, 6, (total + extra, k))], TABLE[rng.integers(0, 6, (g, 2 * inter, k))]
    sa = np.ldexp(1.0, rng.integers(-4, 0, (total + extra, k // 128))).astype(np.float32)
    sb = np.ldexp(1.0, rng.integers(-4, 0, (g, 2 * inter // 128, k // 128))).astype(np.float32)
    ref_h = orc.round_to_bf16(orc.grouped_gemm_fp8_bs(a[:total], sa[:total], off, b, sb))
    act = host(ds3.ds3_swiglu(dev(ref_h.astype(np.float32), bf16=True)))
    q_ref, s_ref = orc.quant_act_1x128(act)
    m = total + extra
    q = torch.full((m, inter), 0x5A, dtype=torch.uint8, device="cuda:0")
    s = torch.full((inter // 128, m), -3.0, dtype=torch.float32, device="cuda:0").t()
    L = ds3._L()
    bi, sbi = dev(wl.interleave_gate_up(b)), dev(wl.interleave_gate_up(sb, block=1))
    ad, sad, offd = dev(a), _kmajor(sa), dev(off)
    st = L.ds3_grouped_gemm_swiglu_quant_fp8_bs(g, offd.data_ptr(), m, inter, k, ad.data_ptr(), k, sad.data_ptr(),
                                                sad.stride(0), sad.stride(1), bi.data_ptr(), k, sbi.data_ptr(),
                                                q.data_ptr(), inter, s.data_ptr(), s.stride(0), s.stride(1), None, 0,
                                                torch.cuda.current_stream().cuda_stream)
    assert st == 0
    qh, sh = host(q), host(s)
    assert np.array_equal(qh[:total], q_ref) and np.array_equal(sh[:total], s_ref)
    assert np.all(qh[total:] == 0x5A) and np.all(sh[total:] == -3.0)
    # row-major scales
    q3, s3 = ds3.ds3_grouped_gemm_swiglu_quant_fp8_bs(ad, sad, offd, bi, sbi, k_major_scales=False)
    assert np.array_equal(host(q3)[:total], q_ref) and np.array_equal(host(s3)[:total], s_ref)


def test_scaled_down_moe_layer(ds3):
    """Config-3 expert FFN at reduced width with the fused call in the middle."""
    announce("fused SwiGLU epilogue: scaled-down MoE layer")
    sizes, off, _ = wl.cfg3_routing(tokens=1024, local=8)
    total = int(off[-1])
    hidden, inter, g = 1024, 256, 8
    x = wl.cfg3_tokens(total, k=hidden)
    w13 = wl.cfg3_w13(g=g, inter=inter, k=hidden)
    qx, sx = ds3.ds3_quant_act_1x128(dev(x, bf16=True))
    q13 = torch.empty((g, 2 * inter, hidden), dtype=torch.uint8, device="cuda:0")
    s13 = torch.empty((g, 2 * inter // 128, hidden // 128), dtype=torch.float32, device="cuda:0")
    for e in range(g):
        q13[e], s13[e] = ds3.ds3_quant_w_128x128(dev(w13[e], bf16=True))
    _check(ds3, host(qx), host(sx), off, host(q13), host(s13), False, "scaled-down MoE layer")
