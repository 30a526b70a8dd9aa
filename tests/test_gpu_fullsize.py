"""Full-size parity of the MoE, backward and MLA configurations in the launch
configuration `bench.py` times: the oracle computes sampled rows / columns of
the outputs one by one on the very codes and scales the GPU quantizers wrote
(those are bit-checked against the oracle at full size in test_gpu_quant.py and
at reduced sizes for every layout)."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from synth import workloads as wl
from tests._gpu_util import announce, dev, host, normwise

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL_F32 = 1e-4


def test_cfg3_grouped_gate_up_full_size_sampled(ds3):
    """32 local experts, the real routing (120 .. 440 rows per expert), gate|up [n_e x 7168] x [4096 x 7168]^T."""
    announce("cfg3 full size sampled")
    G, H, I = wl.LOCAL_EXPERTS, wl.HIDDEN, wl.MOE_INTER
    sizes, off, _ = wl.cfg3_routing()
    rows = int(off[-1])
    x = wl.cfg3_tokens(rows)
    qx, sx = ds3.ds3_quant_act_1x128(dev(x, bf16=True))
    gen = torch.Generator(device="cuda:0").manual_seed(wl.seed_for(3, 2))
    w13 = (torch.randn((G * 2 * I, H), generator=gen, device="cuda:0") * 0.02).to(torch.bfloat16)
    q13, s13 = ds3.ds3_quant_w_128x128(w13)
    del w13
    q13v, s13v = q13.view(G, 2 * I, H), s13.view(G, 2 * I // 128, H // 128)
    h = host(ds3.ds3_grouped_gemm_fp8_bs(qx, sx, dev(off), q13v, s13v))
    qx_h, sx_h = host(qx), host(sx)
    rng = np.random.default_rng(46)
    errs = []
    for e in [0, 1, 7, 16, 31, int(np.argmin(sizes)), int(np.argmax(sizes))]:
        lo, hi = int(off[e]), int(off[e + 1])
        pick = np.unique(np.concatenate([[lo, hi - 1, min(lo + 255, hi - 1), min(lo + 256, hi - 1)], rng.integers(lo, hi, 4)]))
        ref = orc.gemm_fp8_bs(qx_h[pick], sx_h[pick], host(q13v[e]), host(s13v[e]))
        errs.append(normwise(h[pick], ref))
    print("cfg3 sampled errors", ["%.2e" % v for v in errs])
    assert max(errs) <= TOL_BF16


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
    ref = orc.gemm_fp8_bs(host(qdy)[pick], host(sdy)[pick], host(qwt), host(swt))
    e = normwise(dx[pick], ref)
    print(f"cfg4 dgrad sampled: {e:.3e}")
    assert e <= TOL_BF16


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
        ref = orc.gemm_fp8_bs(host(qa)[pick], host(sa)[pick], host(qb), host(sb))
        e = normwise(host(c[torch.from_numpy(pick).to("cuda:0")]), ref)
        print(f"cfg5 {name} {m}x{n}x{k}: {e:.3e}")
        assert e <= TOL_BF16
