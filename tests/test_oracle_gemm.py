"""Pins for the oracle's block-scaled GEMM, grouped GEMM and SwiGLU (CPU only)."""
from fractions import Fraction

import numpy as np
import torch

from oracle import ds3_oracle as orc

_VAL = [None if (c & 0x7F) == 0x7F else Fraction(float(v))
        for c, v in enumerate(orc.e4m3_decode(np.arange(256, dtype=np.uint8)))]


def _codes(rng, shape):
    c = rng.integers(0, 0x7F, size=shape).astype(np.uint8)
    return c | (rng.integers(0, 2, size=shape) << 7).astype(np.uint8)


def _scales(rng, shape):
    return np.exp(rng.standard_normal(shape) * 2).astype(np.float32)


def _brute(a, sa, b, sb, per_row):
    m, k = a.shape
    n = b.shape[0]
    out = [[Fraction(0)] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            acc = Fraction(0)
            for kk in range(k):
                sbv = sb[j, kk // 128] if per_row else sb[j // 128, kk // 128]
                acc += (_VAL[a[i, kk]] * Fraction(float(sa[i, kk // 128]))) * \
                       (_VAL[b[j, kk]] * Fraction(float(sbv)))
            out[i][j] = acc
    return out


def test_gemm_vs_exact_rational_triple_loop():
    rng = np.random.default_rng(31)
    m, n, k = 5, 7, 256
    a, b = _codes(rng, (m, k)), _codes(rng, (n, k))
    sa = _scales(rng, (m, 2))
    sb = _scales(rng, (1, 2))
    y = orc.gemm_fp8_bs(a, sa, b, sb)
    ref = _brute(a, sa, b, sb, per_row=False)
    for i in range(m):
        for j in range(n):
            exact = float(ref[i][j])
            assert abs(y[i, j] - exact) <= 1e-12 * max(1.0, abs(exact))
    # per-row scales on the second operand (weight-gradient form)
    sbr = _scales(rng, (n, 2))
    y2 = orc.gemm_fp8_bs(a, sa, b, sbr, sb_per_row=True)
    ref2 = _brute(a, sa, b, sbr, per_row=True)
    scale = max(abs(float(v)) for row in ref2 for v in row)
    for i in range(m):
        for j in range(n):
            assert abs(y2[i, j] - float(ref2[i][j])) <= 1e-12 * scale


def test_gemm_block_row_index_uses_n_over_128():
    """Block scales of the second operand change at row 128, not elsewhere."""
    rng = np.random.default_rng(32)
    m, n, k = 3, 130, 128
    a, b = _codes(rng, (m, k)), _codes(rng, (n, k))
    sa = np.ones((m, 1), np.float32)
    sb = np.array([[1.0], [4.0]], np.float32)
    y = orc.gemm_fp8_bs(a, sa, b, sb)
    base = orc.gemm_fp8_bs(a, sa, b, np.ones((2, 1), np.float32))
    assert np.array_equal(y[:, :128], base[:, :128]) and np.array_equal(y[:, 128:], 4 * base[:, 128:])


def test_unit_scales_equal_integer_product():
    """All scales 1: the result is the plain product of the decoded codes.  Every
    E4M3 value is a multiple of 2^-9, so the product is computed exactly in
    int64 and the float64 oracle must reproduce it bit for bit."""
    rng = np.random.default_rng(33)
    m, n, k = 64, 48, 1024
    a, b = _codes(rng, (m, k)), _codes(rng, (n, k))
    ai = np.rint(orc.e4m3_decode(a) * 512).astype(np.int64)
    bi = np.rint(orc.e4m3_decode(b) * 512).astype(np.int64)
    exact = (ai @ bi.T).astype(np.float64) / 2.0 ** 18
    assert np.abs(ai @ bi.T).max() < 2 ** 52
    y = orc.gemm_fp8_bs(a, np.ones((m, 8), np.float32), b, np.ones((1, 8), np.float32))
    assert np.array_equal(y, exact)
    # transposed-operand mistakes would show: shapes differ and the result is not symmetric
    assert y.shape == (m, n)


def test_linearity_in_one_scale():
    rng = np.random.default_rng(34)
    m, n, k = 4, 140, 384
    a, b = _codes(rng, (m, k)), _codes(rng, (n, k))
    sa, sb = _scales(rng, (m, 3)), _scales(rng, (2, 3))
    y0 = orc.gemm_fp8_bs(a, sa, b, sb)
    sa2 = sa.copy()
    sa2[2, 1] *= 2
    y1 = orc.gemm_fp8_bs(a, sa2, b, sb)
    contrib = orc.gemm_fp8_bs(a[2:3, 128:256], sa[2:3, 1:2], b[:, 128:256], sb[:, 1:2])
    assert np.allclose(y1[2] - y0[2], contrib[0], rtol=1e-9, atol=1e-9 * np.abs(y0).max())
    assert np.array_equal(np.delete(y1, 2, axis=0), np.delete(y0, 2, axis=0))


def test_accumulate_input_is_added():
    rng = np.random.default_rng(35)
    a, b = _codes(rng, (3, 128)), _codes(rng, (5, 128))
    sa, sb = _scales(rng, (3, 1)), _scales(rng, (5, 1))
    c0 = rng.standard_normal((3, 5)).astype(np.float32)
    y = orc.gemm_fp8_bs(a, sa, b, sb, sb_per_row=True)
    assert np.array_equal(orc.gemm_fp8_bs(a, sa, b, sb, sb_per_row=True, c_in=c0), y + c0.astype(np.float64))


def test_grouped_equals_per_expert_brute_force():
    rng = np.random.default_rng(36)
    off = np.array([0, 3, 3, 4, 9], dtype=np.int32)         # one empty expert
    k, n = 128, 6
    a, sa = _codes(rng, (9, k)), _scales(rng, (9, 1))
    b, sb = _codes(rng, (4, n, k)), _scales(rng, (4, 1, 1))
    y = orc.grouped_gemm_fp8_bs(a, sa, off, b, sb)
    for g in range(4):
        for i in range(off[g], off[g + 1]):
            ref = _brute(a[i:i + 1], sa[i:i + 1], b[g], sb[g], per_row=False)[0]
            for j in range(n):
                assert abs(y[i, j] - float(ref[j])) <= 1e-12 * max(1.0, abs(float(ref[j])))


def test_swiglu_closed_forms_and_library():
    h = np.array([[0.0, np.log(3.0), -np.log(3.0), 30.0, 2.0, 4.0, 4.0, 0.5]])
    out = orc.swiglu(h)[0]                                   # gate = first 4, up = last 4
    assert out[0] == 0.0
    assert abs(out[1] - np.log(3.0) * 0.75 * 4.0) < 1e-14    # sigmoid(ln 3) = 3/4
    assert abs(out[2] + np.log(3.0) * 0.25 * 4.0) < 1e-14    # sigmoid(-ln 3) = 1/4
    assert abs(out[3] - 15.0) < 1e-10                        # silu(30) = 30 to 1e-12
    rng = np.random.default_rng(37)
    hh = rng.standard_normal((16, 64)) * 3
    lib = (torch.nn.functional.silu(torch.from_numpy(hh[:, :32])) * torch.from_numpy(hh[:, 32:])).numpy()
    assert np.allclose(orc.swiglu(hh), lib, rtol=1e-13, atol=1e-15)
