"""Pins for the oracle's power-of-two ("round scaled", Section 3.3.3) quantizers
(CPU only): an independent exact-rational implementation, invariants, the cases
where they coincide with the general quantizers, and the re-tiling property the
report gives as their purpose."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ds3_oracle as orc
from synth import workloads as wl

_TABLE = [Fraction(float(v)) for v in orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))]


def _enc(fr: Fraction, negative: bool) -> int:
    a = abs(fr)
    best = min(range(127), key=lambda c: (abs(_TABLE[c] - a), c % 2))
    return best | (0x80 if negative else 0)


def _quant_group_exact(vals):
    """Smallest power of two s with amax / s <= 448, found by search on exact rationals."""
    fr = [Fraction(v) for v in vals]
    amax = max(abs(f) for f in fr)
    if amax == 0:
        return [0x80 if np.signbit(v) else 0 for v in vals], Fraction(1)
    e = -200
    while amax / Fraction(2) ** e > 448:
        e += 1
    s = Fraction(2) ** e
    assert amax / s <= 448 and amax / (s / 2) > 448
    return [_enc(f / s, np.signbit(v)) for f, v in zip(fr, vals)], s


def _is_pow2(s):
    m, _ = np.frexp(s.astype(np.float64))
    return np.all(m == 0.5)


def test_1x128_vs_exact_rational_implementation():
    rng = np.random.default_rng(61)
    x = rng.standard_normal((5, 256)).astype(np.float32)
    x[0, 5] *= 100
    x[1, 128:] = 0
    x[2, :128] *= 1e-6
    x[3, 130] = -0.0
    x[4, 0], x[4, 1:128] = 448.0 * 4, x[4, 1:128] * 10       # amax/448 exactly a power of two
    x[4, 128] = np.nextafter(np.float32(448.0 * 4), np.float32(1e9))   # one ulp above: the scale doubles
    q, s = orc.quant_act_1x128(x, pow2=True)
    for r in range(5):
        for kb in range(2):
            codes, sc = _quant_group_exact([float(v) for v in x[r, kb * 128:(kb + 1) * 128]])
            assert Fraction(float(s[r, kb])) == sc, (r, kb)
            assert list(q[r, kb * 128:(kb + 1) * 128]) == codes, (r, kb)
    assert s[4, 0] == 4.0 and s[4, 1] == 8.0


def test_128x128_and_128x1_vs_exact_rational_implementation():
    rng = np.random.default_rng(62)
    w = (rng.standard_normal((128, 256)) * 0.02).astype(np.float32)
    w[17, 200] = 3.0
    q, s = orc.quant_w_128x128(w, pow2=True)
    for kb in range(2):
        blk = w[:, kb * 128:(kb + 1) * 128]
        codes, sc = _quant_group_exact([float(v) for v in blk.ravel()])
        assert Fraction(float(s[0, kb])) == sc
        assert list(q[:, kb * 128:(kb + 1) * 128].ravel()) == codes
    x = rng.standard_normal((256, 3)).astype(np.float32)
    x[:, 1] *= 1e3
    qt, st = orc.quant_act_128x1(x, pow2=True)
    assert qt.shape == (3, 256) and st.shape == (3, 2)
    for c in range(3):
        for tb in range(2):
            codes, sc = _quant_group_exact([float(v) for v in x[tb * 128:(tb + 1) * 128, c]])
            assert Fraction(float(st[c, tb])) == sc
            assert list(qt[c, tb * 128:(tb + 1) * 128]) == codes


@pytest.mark.parametrize("maker", ["cfg1", "cfg2"])
def test_invariants(maker):
    x = wl.cfg1()[0] if maker == "cfg1" else wl.cfg2_x(m=64)
    q, s = orc.quant_act_1x128(x, pow2=True)
    assert _is_pow2(s)
    amax = np.abs(x.reshape(x.shape[0], -1, 128)).max(axis=2)
    ratio = amax.astype(np.float64) / s
    assert np.all(ratio <= 448) and np.all(ratio > 224)                  # the smallest such power of two
    # the scaled elements are exact, so the only error is the E4M3 rounding: half a grid step
    y = x.astype(np.float64).reshape(x.shape[0], -1, 128) / s[:, :, None]
    d = orc.e4m3_decode(q).astype(np.float64).reshape(y.shape)
    e = np.floor(np.log2(np.maximum(np.abs(y), 2.0 ** -6)))
    assert np.all(np.abs(d - y) <= 2.0 ** (e - 4) + 1e-300)
    # never coarser than twice the general quantizer's scale, never finer
    _, s_gen = orc.quant_act_1x128(x)
    assert np.all(s >= s_gen) and np.all(s < 2 * s_gen.astype(np.float64))


def test_coincides_with_general_quantizer_when_amax_is_448_times_a_power_of_two():
    rng = np.random.default_rng(63)
    x = rng.standard_normal((8, 384)).astype(np.float32)
    for r in range(8):
        for kb in range(3):
            x[r, kb * 128 + (r + kb) % 128] = 448.0 * 2.0 ** (r - 4 + kb) * 16   # dominates the tile
    q1, s1 = orc.quant_act_1x128(x, pow2=True)
    q0, s0 = orc.quant_act_1x128(x)
    assert np.array_equal(q1, q0) and np.array_equal(s1, s0)


def test_scaling_input_by_power_of_two_shifts_scales_only():
    x = wl.cfg2_x(m=16)
    q, s = orc.quant_act_1x128(x, pow2=True)
    q2, s2 = orc.quant_act_1x128((x * np.float32(2.0 ** -9)).astype(np.float32), pow2=True)
    assert np.array_equal(q, q2)
    assert np.array_equal(s2, s * np.float32(2.0 ** -9))


def test_retiling_to_128x1_adds_no_error_outside_underflow():
    """Section 3.3.3: with power-of-two factors a cached 1x128 activation can be
    re-tiled to 128x1 without a second rounding of the significands.  Elements
    that stay in the normal E4M3 range of their new tile come back exactly."""
    x = wl.cfg2_x(m=256, k=256)
    q, s = orc.quant_act_1x128(x, pow2=True)
    v = orc.dequant_rows(q, s).astype(np.float32)              # the cached values, exact in FP32
    qt, st = orc.quant_act_128x1(v, pow2=True)
    back = orc.dequant_rows(qt, st).T                           # [T][C]
    newscale = np.repeat(st, 128, axis=1).T
    normal = np.abs(v) >= newscale.astype(np.float64) * 2.0 ** -6
    assert normal.mean() > 0.5
    assert np.array_equal(back[normal], v.astype(np.float64)[normal])
    # the same round trip with the general FP32 factors does re-round
    q0, s0 = orc.quant_act_1x128(x)
    v0 = orc.dequant_rows(q0, s0).astype(np.float32)
    qt0, st0 = orc.quant_act_128x1(v0)
    back0 = orc.dequant_rows(qt0, st0).T
    assert np.mean(back0 != v0.astype(np.float64)) > 0.3


def test_zero_group_and_ragged_tail():
    x = np.zeros((2, 200), np.float32)
    x[1, 130] = -3.0
    q, s = orc.quant_act_1x128(x, pow2=True)
    assert s.shape == (2, 2) and s[0, 0] == 1.0 and s[0, 1] == 1.0 and s[1, 0] == 1.0
    assert s[1, 1] == np.float32(2.0 ** -7)                    # 3/448 = 0.0067 <= 2^-7 = 0.0078
    assert q[1, 130] == 0x80 | orc.e4m3_encode_rne_sat(np.array([384.0], np.float32))[0]


# ---- re-tiling of a cached 1x128 activation into 128x1 tiles (Section 3.5.2) ----
def _fl32(fr: Fraction) -> Fraction:
    if fr == 0:
        return Fraction(0)
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    q = Fraction(2) ** (e - 23)
    n = a / q
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return (-1 if fr < 0 else 1) * fl * q


def test_retile_vs_exact_rational_implementation():
    """Dequantize with exact rationals rounded once to FP32, then the general 128x1
    rule (correctly rounded amax/448 and 448/amax, one FP32 multiply, nearest-even cast)."""
    x = wl.cfg2_x(m=128, k=256)[:, 120:136].copy()            # 16 channels straddling two 1x128 tiles
    xp = np.zeros((128, 256), np.float32); xp[:, 120:136] = x
    q, s = orc.quant_act_1x128(xp)
    qt, st = orc.retile_1x128_to_128x1(q, s)
    for c in (120, 127, 128, 135):
        v = [_fl32(_TABLE[q[t, c] & 0x7F] * (-1 if q[t, c] & 0x80 else 1) * Fraction(float(s[t, c // 128]))) for t in range(128)]
        amax = max(abs(f) for f in v)
        sc, r = _fl32(amax / 448), _fl32(Fraction(448) / amax)
        assert Fraction(float(st[c, 0])) == sc
        codes = [_enc(_fl32(f * r), bool(q[t, c] & 0x80)) for t, f in enumerate(v)]
        assert list(qt[c]) == codes, c


def test_retile_identities():
    x = wl.cfg2_x(m=256, k=256)
    q, s = orc.quant_act_1x128(x)
    qt, st = orc.retile_1x128_to_128x1(q, s)
    assert qt.shape == (256, 256) and st.shape == (256, 2)
    # it is the 128x1 quantizer applied to the dequantized cache ...
    v = (orc.e4m3_decode(q).astype(np.float64) * np.repeat(s.astype(np.float64), 128, axis=1)).astype(np.float32)
    q2, s2 = orc.quant_act_128x1(v)
    assert np.array_equal(qt, q2) and np.array_equal(st, s2)
    # ... whose group maxima are reproduced by the new tiles: max |dequant| per (channel, token block) is kept
    back = orc.dequant_rows(qt, st).T
    for tb in range(2):
        blk = slice(tb * 128, (tb + 1) * 128)
        assert np.allclose(np.abs(back[blk]).max(axis=0), np.abs(v[blk].astype(np.float64)).max(axis=0), rtol=2e-7)
    # a matrix whose rows are all equal has one value per channel: every 128x1 tile is constant, code 0x7E
    row = wl.cfg2_x(m=1, k=256)
    q1, s1 = orc.quant_act_1x128(np.repeat(row, 128, axis=0))
    qt1, _ = orc.retile_1x128_to_128x1(q1, s1)
    nz = (q1[0] & 0x7F) != 0
    assert np.all((qt1[nz] & 0x7F) == 0x7E)
    # ragged token count and an all-zero channel
    q3, s3 = orc.quant_act_1x128(x[:130])
    q3[:, 7] = 0
    qt3, st3 = orc.retile_1x128_to_128x1(q3, s3)
    assert qt3.shape == (256, 130) and st3.shape == (256, 2) and st3[7, 0] == 1.0 and st3[7, 1] == 1.0
