"""Tensors beyond 4 GiB: every byte offset past 2^32 must be formed in 64 bits.  Inputs are drawn on the
device (seeded); the oracle runs on rows sampled from the start, the middle and the far end."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from tests._gpu_util import announce, dev, host, normwise

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3


def _sample_rows(total, rng, n=24):
    edge = np.concatenate([np.arange(0, 8), np.arange(total - 8, total), [total // 2, total // 2 + 1]])
    return np.unique(np.concatenate([edge, rng.integers(0, total, n)]))


def test_quantizers_on_a_5_gb_activation(ds3):
    rows, cols = 1_200_000, 2048                    # 4.9 GB of BF16, 2.46 GB of codes
    announce(f"large quantizers {rows}x{cols}")
    gen = torch.Generator(device="cuda:0").manual_seed(9001)
    x = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda:0")
    step = 100_000
    for r0 in range(0, rows, step):                 # drawn in slices: the FP32 staging tensor stays small
        x[r0:r0 + step] = torch.randn((step, cols), generator=gen, device="cuda:0").to(torch.bfloat16)
    rng = np.random.default_rng(9002)
    pick = _sample_rows(rows, rng)
    xs = host(x[torch.from_numpy(pick).to("cuda:0")])
    # 1x128
    q, s = ds3.ds3_quant_act_1x128(x)
    idx = torch.from_numpy(pick).to("cuda:0")
    q_ref, s_ref = orc.quant_act_1x128(xs)
    assert np.array_equal(host(q[idx]), q_ref) and np.array_equal(host(s[idx]), s_ref)
    del q, s
    # 128x1: token blocks at both ends and in the middle, all channels
    qt, st = ds3.ds3_quant_act_128x1(x)
    for tb in (0, rows // 128 // 2, rows // 128 - 1):
        blk = host(x[tb * 128:(tb + 1) * 128])
        qt_ref, st_ref = orc.quant_act_128x1(blk)
        assert np.array_equal(host(qt[:, tb * 128:(tb + 1) * 128]), qt_ref), tb
        assert np.array_equal(host(st[:, tb]), st_ref[:, 0]), tb
    del qt, st
    # 128x128 blocks of the same tensor taken as a weight
    qw, sw = ds3.ds3_quant_w_128x128(x)
    for nb in (0, rows // 128 // 2, rows // 128 - 1):
        blk = host(x[nb * 128:(nb + 1) * 128])
        qw_ref, sw_ref = orc.quant_w_128x128(blk)
        assert np.array_equal(host(qw[nb * 128:(nb + 1) * 128]), qw_ref), nb
        assert np.array_equal(host(sw[nb]), sw_ref[0]), nb


def test_gemm_with_a_4_gb_output(ds3):
    m, n, k = 70_016, 32_768, 256                   # 2.29e9 outputs: 4.6 GB of BF16
    announce(f"large GEMM {m}x{n}x{k}")
    gen = torch.Generator(device="cuda:0").manual_seed(9003)
    a = torch.randint(0, 256, (m, k), generator=gen, device="cuda:0", dtype=torch.int32).to(torch.uint8)
    a = torch.where((a & 0x7F) == 0x7F, a & 0xFE, a)                # no NaN codes
    b = torch.randint(0, 256, (n, k), generator=gen, device="cuda:0", dtype=torch.int32).to(torch.uint8)
    b = torch.where((b & 0x7F) == 0x7F, b & 0xFE, b)
    sa = torch.exp(torch.randn((k // 128, m), generator=gen, device="cuda:0")).t() * 2.0 ** -8
    sb = torch.exp(torch.randn((n // 128, k // 128), generator=gen, device="cuda:0")) * 2.0 ** -8
    rng = np.random.default_rng(9004)
    pick = _sample_rows(m, rng)
    idx = torch.from_numpy(pick).to("cuda:0")
    ref = orc.gemm_fp8_bs(host(a[idx]), host(sa[idx]), host(b), host(sb))
    c = ds3.ds3_gemm_fp8_bs(a, sa, b, sb)
    e = normwise(host(c[idx]), ref)
    print(f"large GEMM sampled rows: {e:.3e}")
    assert e <= TOL_BF16
    del c
    # the same rows as three expert groups: offsets deep into the activation and the output
    off = np.array([0, 30_000, 30_000, m - 5], dtype=np.int32)      # an empty group, 5 rows beyond the last
    bg = torch.stack([b[:8192], b[8192:16384], b[16384:24576]])
    sbg = torch.stack([sb[:64], sb[64:128], sb[128:192]])
    cg = torch.full((m, 8192), 3.0, dtype=torch.bfloat16, device="cuda:0")
    ds3.ds3_grouped_gemm_fp8_bs(a, sa, dev(off), bg, sbg, c=cg)
    assert torch.all(cg[m - 5:] == 3.0)
    got = host(cg[idx])
    for i, r in enumerate(pick):
        if r >= m - 5:
            continue
        g = 0 if r < 30_000 else 2
        assert normwise(got[i], ref[i, g * 8192:(g + 1) * 8192]) <= 2 * TOL_BF16, int(r)


def test_gemm_with_a_very_long_inner_dimension(ds3):
    """K = 65536 (512 K-steps): small-integer codes and power-of-two scales keep every partial sum exact,
    so the FP32 result equals the oracle bit for bit; with and without tail sharing, both scale paths."""
    m, n, k = 300, 260, 65_536
    announce(f"long K {m}x{n}x{k}")
    rng = np.random.default_rng(9005)
    table = np.array([0x00, 0x38, 0x40, 0xB8, 0xC0, 0x80], dtype=np.uint8)   # 0, 1, 2, -1, -2, -0
    a, b = table[rng.integers(0, 6, (m, k))], table[rng.integers(0, 6, (n, k))]
    sa = np.ldexp(1.0, rng.integers(-1, 2, (m, k // 128))).astype(np.float32)
    sb = np.ldexp(1.0, rng.integers(-1, 3, ((n + 127) // 128, k // 128))).astype(np.float32)
    ref = orc.gemm_fp8_bs(a, sa, b, sb)
    assert np.array_equal(ref.astype(np.float32).astype(np.float64), ref)
    args = (dev(a), dev(np.ascontiguousarray(sa.T)).t(), dev(b), dev(sb))
    for fn in (ds3.ds3_gemm_fp8_bs, ds3.ds3_gemm_fp8_bs_pow2):
        for ws in ("auto", None):
            c = host(fn(*args, out_dtype=torch.float32, workspace=ws))
            assert np.array_equal(c.astype(np.float64), ref), (fn.__name__, ws)
