"""Pins for the oracle's E5M6 cache format (Section 3.3.3 names the format; the
bit layout is this build's proposal, see the oracle).  CPU only."""
from fractions import Fraction

import numpy as np

from oracle import ds3_oracle as orc
from synth import workloads as wl

VALID = np.array([c for c in range(4096) if ((c >> 6) & 0x1F) != 31], dtype=np.uint16)


def test_codes_are_the_upper_twelve_bits_of_binary16():
    v = orc.e5m6_decode(VALID)
    half = (VALID.astype(np.uint16) << 4).view(np.float16).astype(np.float64)
    assert np.array_equal(v, half)
    assert np.nanmax(v) == 65024.0 and orc.e5m6_decode(np.array([1]))[0] == 2.0 ** -20
    assert np.all(np.isnan(orc.e5m6_decode(np.array([31 << 6, (31 << 6) | 5 | 0x800]))))


def test_encode_inverts_decode_and_is_monotonic():
    v = orc.e5m6_decode(VALID)
    assert np.array_equal(orc.e5m6_encode_rne_sat(v), VALID)
    pos = np.sort(v[v >= 0])
    mids = (pos[:-1] + pos[1:]) / 2
    got = orc.e5m6_decode(orc.e5m6_encode_rne_sat(mids))
    even = np.where((orc.e5m6_encode_rne_sat(pos[:-1]) & 1) == 0, pos[:-1], pos[1:])
    assert np.array_equal(got, even)                                   # ties go to the even code
    x = np.sort(np.random.default_rng(95).standard_normal(5000) * 300)
    assert np.all(np.diff(orc.e5m6_decode(orc.e5m6_encode_rne_sat(x))) >= 0)
    assert orc.e5m6_encode_rne_sat(np.array([1e9, -1e9, -0.0])).tolist() == [0x7BF, 0xFBF, 0x800]


def test_encode_is_nearest_by_brute_force():
    table = [Fraction(float(v)) for v in orc.e5m6_decode(VALID[VALID < 0x800])]
    rng = np.random.default_rng(96)
    ys = np.concatenate([rng.standard_normal(150) * 10.0 ** rng.integers(-7, 5, 150), [2.0 ** -21, 3 * 2.0 ** -21, 65023.9, 64768.0]])
    for y in ys:
        a = abs(Fraction(float(y)))
        best = min(range(len(table)), key=lambda c: (abs(table[c] - a), c % 2))
        assert int(orc.e5m6_encode_rne_sat(np.array([y]))[0]) == (best | (0x800 if y < 0 else 0)), y


def test_pack_round_trip_and_layout():
    rng = np.random.default_rng(97)
    c = rng.integers(0, 4096, (3, 10)).astype(np.uint16)
    p = orc.e5m6_pack(c)
    assert p.shape == (3, 15) and np.array_equal(orc.e5m6_unpack(p), c)
    one = orc.e5m6_pack(np.array([[0xABC, 0x123]], np.uint16))
    assert one.tolist() == [[0xBC, 0x3A, 0x12]]


def test_quantizer_scales_and_error_bound():
    x = wl.cfg2_x(m=32, k=512)
    p, s = orc.quant_act_1x128_e5m6(x)
    assert p.shape == (32, 768) and s.shape == (32, 4)
    m, _ = np.frexp(s.astype(np.float64))
    assert np.all(m == 0.5)                                             # powers of two
    amax = np.abs(x.reshape(32, 4, 128)).max(axis=2)
    ratio = amax / s.astype(np.float64)
    assert np.all(ratio <= 65024) and np.all(ratio > 65024 / 2)
    d = orc.dequant_e5m6(p, s)
    y = x.astype(np.float64)
    # 6 mantissa bits: relative error 2^-7 in the normal range (14 binades below the scaled maximum and more)
    normal = np.abs(y) >= np.repeat(s, 128, axis=1) * 2.0 ** -14
    assert np.all(np.abs(d - y)[normal] <= np.abs(y)[normal] * 2.0 ** -7)
    assert normal.mean() > 0.999
    # a BF16 input has 8 significant bits: the cache keeps 7 of them; E4M3 with the same tiles keeps 4
    q8, s8 = orc.quant_act_1x128(x, pow2=True)
    e12 = np.linalg.norm(d - y) / np.linalg.norm(y)
    e8 = np.linalg.norm(orc.dequant_rows(q8, s8) - y) / np.linalg.norm(y)
    assert e12 < e8 / 6
    # zero tile and amax exactly 65024 * 2^j
    z = np.zeros((1, 128), np.float32); z[0, 3] = 65024.0 * 4
    pz, sz = orc.quant_act_1x128_e5m6(z)
    assert sz[0, 0] == 4.0 and orc.e5m6_unpack(pz)[0, 3] == 0x7BF
    p0, s0 = orc.quant_act_1x128_e5m6(np.zeros((1, 128), np.float32))
    assert s0[0, 0] == 1.0 and not p0.any()
