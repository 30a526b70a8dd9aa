"""Pins for the oracle's E4M3 decode / encode (CPU only)."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc

GOLDEN = __file__.rsplit("/", 1)[0] + "/golden/e4m3_values.txt"
ALL = np.arange(256, dtype=np.uint8)


def test_decode_golden_values_from_format_spec():
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        got = orc.e4m3_decode(np.array([int(code, 16)], dtype=np.uint8))[0]
        assert got == float(val) and np.signbit(got) == val.startswith("-"), (code, val, got)


def test_decode_matches_library_cast_on_all_codes():
    lib = torch.from_numpy(ALL.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = orc.e4m3_decode(ALL)
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    assert np.isnan(mine[0x7F]) and np.isnan(mine[0xFF]) and np.isnan(mine).sum() == 2
    f = ~np.isnan(mine)
    assert np.array_equal(lib[f], mine[f])
    assert np.array_equal(np.signbit(lib[f]), np.signbit(mine[f]))


def test_decode_structure():
    pos = orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))
    assert np.all(np.diff(pos) > 0)                       # strictly monotone in code order
    assert pos.max() == 448.0 and pos[1] == 2.0 ** -9 and pos[8] == 2.0 ** -6
    # eight equally spaced values per binade, spacing doubles each binade
    d = np.diff(pos)
    assert np.all(d[:15] == 2.0 ** -9)                    # subnormals and first binade share the step
    for e in range(1, 15):
        seg = d[8 * e: min(8 * e + 8, len(d))]
        assert np.all(seg == 2.0 ** (e - 10))
    neg = orc.e4m3_decode(np.arange(0x80, 0xFF, dtype=np.uint8))
    assert np.array_equal(neg, -pos)


def test_encode_round_trip_all_finite_codes():
    v = orc.e4m3_decode(ALL)
    f = np.isfinite(v)
    assert np.array_equal(orc.e4m3_encode_rne_sat(v[f].astype(np.float32)), ALL[f])


def test_encode_named_ties_and_saturation():
    cases = [(17.0, 0x58), (19.0, 0x5A), (2.0 ** -10, 0x00), (3 * 2.0 ** -10, 0x02), (464.0, 0x7E),
             (463.9, 0x7E), (1e30, 0x7E), (-1e30, 0xFE), (-0.0, 0x80), (-1e-12, 0x80), (0.0, 0x00),
             (448.0, 0x7E), (432.0, 0x7E), (431.9, 0x7D), (2.0 ** -9, 0x01),
             (1.5 * 2.0 ** -9, 0x02), (2.5 * 2.0 ** -9, 0x02), (0.9999, 0x38), (1.0625, 0x38),
             (1.1875, 0x3A)]
    # 432 is the midpoint of 416 (0x7D, odd mantissa) and 448 (0x7E, even) -> 448
    for y, code in cases:
        assert orc.e4m3_encode_rne_sat(np.array([y], dtype=np.float32))[0] == code, y


def test_encode_every_midpoint_goes_to_even_code():
    pos = orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))
    for c in range(0, 0x7E):
        mid = np.float32((pos[c] + pos[c + 1]) / 2)       # exactly representable in float32
        assert float(mid) * 2 == pos[c] + pos[c + 1]
        even = c if c % 2 == 0 else c + 1
        assert orc.e4m3_encode_rne_sat(np.array([mid]))[0] == even
        lo = np.nextafter(mid, np.float32(0))
        hi = np.nextafter(mid, np.float32(1e9))
        assert orc.e4m3_encode_rne_sat(np.array([lo]))[0] == c
        assert orc.e4m3_encode_rne_sat(np.array([hi]))[0] == c + 1
        assert orc.e4m3_encode_rne_sat(np.array([-mid]))[0] == even | 0x80


def _brute_force_nearest(y: np.ndarray) -> np.ndarray:
    """Nearest finite E4M3 value by exhaustive search over the 127 magnitudes,
    ties to the even code, saturating (anything above 448 is nearest to 448)."""
    table = orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))       # 127 magnitudes
    a = np.abs(y.astype(np.float64))[:, None]
    dist = np.abs(a - table[None, :])
    best = dist.min(axis=1, keepdims=True)
    cand = dist == best                                               # one or two candidates
    codes = np.arange(0x7F)[None, :]
    even_pref = np.where(cand & (codes % 2 == 0), codes, -1).max(axis=1)
    any_pref = np.where(cand, codes, -1).max(axis=1)
    two = cand.sum(axis=1) == 2
    out = np.where(two, even_pref, any_pref)
    return (out | np.where(np.signbit(y), 0x80, 0)).astype(np.uint8)


def test_encode_vs_brute_force_search():
    rng = np.random.default_rng(7)
    ys = [
        rng.standard_normal(200_000).astype(np.float32) * 100,
        (rng.random(200_000).astype(np.float32) * 2 - 1) * 470,
        np.ldexp(rng.random(200_000), rng.integers(-14, 10, 200_000)).astype(np.float32),
        (rng.random(100_000).astype(np.float32) * 2 - 1) * 2.0 ** -6,
    ]
    # every float32 within 2 ulps of a grid point or a midpoint
    pos = orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))
    pts = np.concatenate([pos, (pos[:-1] + pos[1:]) / 2]).astype(np.float32)
    near = [pts]
    for _ in range(2):
        near.append(np.nextafter(near[-1], np.float32(-1)))
    up = pts
    for _ in range(2):
        up = np.nextafter(up, np.float32(1e9))
        near.append(up)
    ys.append(np.concatenate(near))
    ys.append(-ys[-1])
    for y in ys:
        for lo in range(0, y.size, 50_000):
            chunk = y[lo: lo + 50_000]
            assert np.array_equal(orc.e4m3_encode_rne_sat(chunk), _brute_force_nearest(chunk))


def test_encode_vs_exact_rational_rounding():
    """Independent scalar implementation with exact rationals."""
    rng = np.random.default_rng(11)
    table = [Fraction(float(v)) for v in orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))]
    ys = np.concatenate([rng.standard_normal(300).astype(np.float32) * 60,
                         np.array([0.0, 448.0, 2.0 ** -10, 465.0, 1e-20], dtype=np.float32)])
    for y in ys:
        a = abs(Fraction(float(y)))
        best = min(range(127), key=lambda c: (abs(table[c] - a), c % 2))
        want = best | (0x80 if np.signbit(y) else 0)
        assert orc.e4m3_encode_rne_sat(np.array([y]))[0] == want


def test_encode_vs_library_cast_third_opinion():
    """PyTorch's CPU cast to float8_e4m3fn (round-to-nearest-even).  Compared
    inside the finite range only: the library does not saturate."""
    rng = np.random.default_rng(3)
    y = np.concatenate([(rng.random(500_000).astype(np.float32) * 2 - 1) * 448,
                        np.ldexp(rng.random(300_000), rng.integers(-16, 9, 300_000)).astype(np.float32)])
    y = y[np.abs(y) <= 448]
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(orc.e4m3_encode_rne_sat(y), lib)


def test_encode_rejects_non_finite():
    with pytest.raises(ValueError):
        orc.e4m3_encode_rne_sat(np.array([np.inf], dtype=np.float32))
    with pytest.raises(ValueError):
        orc.e4m3_encode_rne_sat(np.array([np.nan], dtype=np.float32))
