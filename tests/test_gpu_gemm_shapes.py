"""Seeded sweep of small GEMM shapes with ragged M and N, padded leading dimensions,
both scale layouts, both weight-scale modes, every tile configuration and both the
general and the power-of-two path.  Codes are small integers and scales powers of
two, so every partial sum is exact and the FP32 output must equal the oracle bit for
bit: an edge-handling mistake cannot hide inside a tolerance."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from tests._gpu_util import announce, dev, host

pytestmark = pytest.mark.gpu

TABLE = np.array([0x00, 0x38, 0x40, 0xB8, 0xC0, 0x80], dtype=np.uint8)   # 0, 1, 2, -1, -2, -0


def _padded(a: np.ndarray, ld: int) -> torch.Tensor:
    buf = torch.zeros((a.shape[0], ld), dtype=torch.uint8, device="cuda:0")
    buf[:, : a.shape[1]] = dev(a)
    return buf[:, : a.shape[1]]


def test_seeded_shape_sweep(ds3):
    rng = np.random.default_rng(2024)
    nvar = ds3.ds3_gemm_num_variants()
    for case in range(48):
        m = int(rng.choice([1, 2, 15, 16, 17, 127, 128, 129, 255, 256, 257, 300, 511, 640]))
        n = int(rng.choice([1, 3, 4, 63, 64, 65, 127, 128, 129, 200, 256, 260, 384, 513]))
        k = 128 * int(rng.integers(1, 9))
        per_row = bool(rng.integers(0, 2))
        pow2 = bool(rng.integers(0, 2))
        variant = int(rng.integers(-1, nvar))
        k_major = bool(rng.integers(0, 2))
        accumulate = bool(rng.integers(0, 2))
        lda, ldb = k + 16 * int(rng.integers(0, 3)), k + 16 * int(rng.integers(0, 3))
        announce(f"sweep {case}: {m}x{n}x{k} per_row={per_row} pow2={pow2} variant={variant} k_major={k_major} acc={accumulate} ld=({lda},{ldb})")
        a, b = TABLE[rng.integers(0, 6, (m, k))], TABLE[rng.integers(0, 6, (n, k))]
        sa = np.ldexp(1.0, rng.integers(-2, 2, (m, k // 128))).astype(np.float32)
        nb = n if per_row else (n + 127) // 128
        sb = np.ldexp(1.0, rng.integers(-1, 3, (nb, k // 128))).astype(np.float32)
        c0 = rng.integers(-8, 9, (m, n)).astype(np.float32) if accumulate else None
        ref = orc.gemm_fp8_bs(a, sa, b, sb, sb_per_row=per_row, c_in=c0)
        assert np.array_equal(ref.astype(np.float32).astype(np.float64), ref)
        sa_d = dev(np.ascontiguousarray(sa.T)).t() if k_major else dev(sa)
        ldc = (n + 3) // 4 * 4 + 4 * int(rng.integers(0, 3))
        cbuf = torch.full((m, ldc), 7.0, dtype=torch.float32, device="cuda:0")
        c = cbuf[:, :n]
        if accumulate:
            c.copy_(dev(c0))
        fn = ds3.ds3_gemm_fp8_bs_pow2 if pow2 else ds3.ds3_gemm_fp8_bs
        fn(_padded(a, lda), sa_d, _padded(b, ldb), dev(sb),
           sb_mode=ds3.DS3_BSCALE_PER_ROW if per_row else ds3.DS3_BSCALE_128x128, c=c, accumulate=accumulate, variant=variant)
        got = host(c)
        bad = np.argwhere(got.astype(np.float64) != ref)
        assert bad.size == 0, f"case {case}: {bad.shape[0]} mismatches, first {bad[0]}: {got[tuple(bad[0])]} vs {ref[tuple(bad[0])]}"
        if ldc > n:
            assert torch.all(cbuf[:, n:] == 7.0), "wrote beyond the row"


def test_seeded_grouped_sweep(ds3):
    rng = np.random.default_rng(2025)
    nvar = ds3.ds3_gemm_num_variants()
    for case in range(12):
        g = int(rng.integers(1, 12))
        sizes = rng.choice([0, 0, 1, 15, 16, 100, 128, 129, 256, 257, 300], size=g).astype(np.int32)
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        rows = int(off[-1]) + int(rng.integers(0, 3))          # a few rows past the last group stay untouched
        n = int(rng.choice([64, 128, 200, 256, 384]))
        k = 128 * int(rng.integers(1, 5))
        pow2 = bool(rng.integers(0, 2))
        variant = int(rng.integers(-1, nvar))
        announce(f"grouped sweep {case}: sizes={sizes.tolist()} n={n} k={k} pow2={pow2} variant={variant}")
        a = TABLE[rng.integers(0, 6, (rows, k))]
        b = TABLE[rng.integers(0, 6, (g, n, k))]
        sa = np.ldexp(1.0, rng.integers(-2, 2, (rows, k // 128))).astype(np.float32)
        sb = np.ldexp(1.0, rng.integers(-1, 3, (g, (n + 127) // 128, k // 128))).astype(np.float32)
        ref = orc.grouped_gemm_fp8_bs(a[: off[-1]], sa[: off[-1]], off, b, sb)
        c = torch.full((rows, n), -3.0, dtype=torch.float32, device="cuda:0")
        if rows == 0:
            continue
        fn = ds3.ds3_grouped_gemm_fp8_bs_pow2 if pow2 else ds3.ds3_grouped_gemm_fp8_bs
        fn(dev(a), dev(np.ascontiguousarray(sa.T)).t(), dev(off), dev(b), dev(sb), c=c, variant=variant)
        got = host(c)
        assert np.array_equal(got[: off[-1]].astype(np.float64), ref), case
        assert np.all(got[off[-1]:] == -3.0), "rows beyond the last group were written"


def test_seeded_grouped_sweep(ds3):
    """The same for the grouped GEMM: random group sizes (empty, single rows, around the tile heights),
    ragged N, every tile configuration, both scale paths, static walk and tile queue, rows beyond the
    last group untouched -- bit for bit against the oracle."""
    rng = np.random.default_rng(2025)
    nvar = ds3.ds3_gemm_num_variants()
    for case in range(24):
        g = int(rng.integers(1, 13))
        sizes = rng.choice([0, 0, 1, 5, 64, 65, 127, 128, 129, 200, 256, 257, 300], g)
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        total, extra = int(off[-1]), int(rng.integers(0, 4))
        n = int(rng.choice([64, 128, 200, 256, 384, 640]))
        k = 128 * int(rng.integers(1, 7))
        pow2 = bool(rng.integers(0, 2))
        variant = int(rng.integers(-1, nvar))
        queue = bool(rng.integers(0, 2))
        announce(f"grouped sweep {case}: sizes {list(sizes)} n={n} k={k} pow2={pow2} variant={variant} queue={queue}")
        rows = total + extra
        a, b = TABLE[rng.integers(0, 6, (max(rows, 1), k))], TABLE[rng.integers(0, 6, (g, n, k))]
        sa = np.ldexp(1.0, rng.integers(-2, 2, (max(rows, 1), k // 128))).astype(np.float32)
        sb = np.ldexp(1.0, rng.integers(-1, 3, (g, (n + 127) // 128, k // 128))).astype(np.float32)
        ref = orc.grouped_gemm_fp8_bs(a[:total], sa[:total], off, b, sb)
        ldc = (n + 3) // 4 * 4
        cbuf = torch.full((max(rows, 1), ldc), 7.0, dtype=torch.float32, device="cuda:0")
        c = cbuf[:, :n]
        fn = ds3.ds3_grouped_gemm_fp8_bs_pow2 if pow2 else ds3.ds3_grouped_gemm_fp8_bs
        fn(dev(a), dev(np.ascontiguousarray(sa.T)).t(), dev(off), dev(b), dev(sb), c=c, variant=variant,
           workspace="auto" if queue else None)
        got = host(cbuf)
        assert np.array_equal(got[:total, :n].astype(np.float64), ref), case
        assert np.all(got[total:] == 7.0) and np.all(got[:, n:] == 7.0), case
