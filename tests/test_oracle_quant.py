"""Pins for the oracle's quantizers (CPU only): an independent exact-rational
implementation, invariants and identities.  None of them calls the GPU path."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ds3_oracle as orc
from synth import workloads as wl


# ---- an independent scalar implementation with exact rationals ----------------
def _fl32(fr: Fraction) -> Fraction:
    """Round an exact rational to the nearest float32 (ties to even), normal range."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1) and -126 <= e <= 127
    q = Fraction(2) ** (e - 23)
    n = a / q
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * fl * q


_TABLE = [Fraction(float(v)) for v in orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))]


def _enc(fr: Fraction, negative: bool) -> int:
    a = abs(fr)
    best = min(range(127), key=lambda c: (abs(_TABLE[c] - a), c % 2))
    return best | (0x80 if negative else 0)


def _quant_group_exact(vals):
    """vals: list of python floats (float32-representable).  Returns (codes, scale)."""
    fr = [Fraction(v) for v in vals]
    amax = max(abs(f) for f in fr)
    if amax == 0:
        return [0x80 if np.signbit(v) else 0 for v in vals], Fraction(1)
    s = _fl32(amax / 448)
    r = _fl32(Fraction(448) / amax)
    codes = [_enc(_fl32(f * r), np.signbit(v)) for f, v in zip(fr, vals)]
    return codes, s


def test_1x128_vs_exact_rational_implementation():
    rng = np.random.default_rng(21)
    x = rng.standard_normal((4, 256)).astype(np.float32)
    x[0, 5] *= 100
    x[1, 128:] = 0                      # an all-zero tile
    x[2, :128] *= 1e-6
    x[3, 130] = -0.0
    q, s = orc.quant_act_1x128(x)
    for m in range(4):
        for kb in range(2):
            codes, sc = _quant_group_exact([float(v) for v in x[m, kb * 128:(kb + 1) * 128]])
            assert list(q[m, kb * 128:(kb + 1) * 128]) == codes
            assert Fraction(float(s[m, kb])) == sc


def test_128x128_and_128x1_vs_exact_rational_implementation():
    rng = np.random.default_rng(22)
    w = (rng.standard_normal((130, 136)) * 0.02).astype(np.float32)   # ragged in both directions
    q, s = orc.quant_w_128x128(w)
    assert q.shape == (130, 136) and s.shape == (2, 2)
    for nb, (r0, r1) in enumerate([(0, 128), (128, 130)]):
        for kb, (c0, c1) in enumerate([(0, 128), (128, 136)]):
            blk = w[r0:r1, c0:c1]
            codes, sc = _quant_group_exact([float(v) for v in blk.ravel()])
            assert list(q[r0:r1, c0:c1].ravel()) == codes
            assert Fraction(float(s[nb, kb])) == sc
    x = rng.standard_normal((131, 3)).astype(np.float32)
    qt, st = orc.quant_act_128x1(x)
    assert qt.shape == (3, 131) and st.shape == (3, 2)
    for c in range(3):
        for tb, (t0, t1) in enumerate([(0, 128), (128, 131)]):
            codes, sc = _quant_group_exact([float(v) for v in x[t0:t1, c]])
            assert list(qt[c, t0:t1]) == codes
            assert Fraction(float(st[c, tb])) == sc


# ---- invariants -----------------------------------------------------------------
def _e4m3_ulp(y):
    a = np.abs(y.astype(np.float64))
    e = np.maximum(np.floor(np.log2(np.maximum(a, 2.0 ** -30))), -6)
    return 2.0 ** (e - 3)


@pytest.mark.parametrize("maker", ["cfg1", "cfg2"])
def test_group_max_maps_to_448_and_error_bound(maker):
    if maker == "cfg1":
        x, _ = wl.cfg1()
    else:
        x = wl.cfg2_x(m=64, k=1024)
    q, s = orc.quant_act_1x128(x)
    m, k = x.shape
    xt = x.reshape(m, k // 128, 128)
    qt = q.reshape(m, k // 128, 128)
    amax_pos = np.argmax(np.abs(xt), axis=2)
    top = np.take_along_axis(qt, amax_pos[..., None], axis=2)[..., 0]
    assert np.all((top & 0x7F) == 0x7E)                                  # +-448
    deq = orc.e4m3_decode(q) * np.repeat(s.astype(np.float64), 128, axis=1)
    y = x.astype(np.float64) / np.repeat(s.astype(np.float64), 128, axis=1)
    bound = 0.5 * _e4m3_ulp(y) * np.repeat(s.astype(np.float64), 128, axis=1) + 4 * 2.0 ** -24 * np.abs(x)
    assert np.all(np.abs(deq - x) <= bound)
    # relative error of normal-range elements is at most 2^-4 (half of 3 mantissa bits) plus slack
    normal = np.abs(y) >= 2.0 ** -6
    assert np.all(np.abs(deq - x)[normal] <= (2.0 ** -4 + 1e-6) * np.abs(x)[normal])


def test_power_of_two_inputs_reproduce_exactly():
    rng = np.random.default_rng(5)
    k = rng.integers(-20, 20, size=(16, 1))
    j = k - rng.integers(0, 15, size=(16, 128))              # j >= k - 14
    j[:, 0] = k[:, 0]                                        # the max itself
    sign = rng.choice([-1.0, 1.0], size=(16, 128))
    x = (sign * np.ldexp(1.0, j)).astype(np.float32)
    q, s = orc.quant_act_1x128(x)
    deq32 = (orc.e4m3_decode(q).astype(np.float32) * s).astype(np.float32)
    assert np.array_equal(deq32, x)
    # amax = 448 * 2^k  ->  s = 2^k exactly and any E4M3 value times 2^k round-trips
    codes = rng.integers(0, 0x7F, size=(8, 128)).astype(np.uint8)
    codes[:, 3] = 0x7E
    codes |= (rng.integers(0, 2, size=codes.shape) << 7).astype(np.uint8)
    kk = rng.integers(-10, 10, size=(8, 1))
    x2 = np.ldexp(orc.e4m3_decode(codes), kk).astype(np.float32)
    q2, s2 = orc.quant_act_1x128(x2)
    assert np.array_equal(s2[:, 0], np.ldexp(1.0, kk[:, 0]).astype(np.float32))
    assert np.array_equal(q2, codes)


def test_scaling_by_power_of_two_keeps_codes():
    x, w = wl.cfg1(m=32, n=128, k=256)
    q, s = orc.quant_act_1x128(x)
    for p in (-7, 3, 12):
        qp, sp = orc.quant_act_1x128(np.ldexp(x, p).astype(np.float32))
        assert np.array_equal(qp, q) and np.array_equal(sp, np.ldexp(s, p).astype(np.float32))
    qw, sw = orc.quant_w_128x128(w)
    qp, sp = orc.quant_w_128x128(np.ldexp(w, 5).astype(np.float32))
    assert np.array_equal(qp, qw) and np.array_equal(sp, np.ldexp(sw, 5).astype(np.float32))


def test_transposition_identities():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((300, 200)).astype(np.float32)
    qt, st = orc.quant_act_128x1(x)                       # [C][T], [C][T/128]
    q2, s2 = orc.quant_act_1x128(np.ascontiguousarray(x.T))
    assert np.array_equal(qt, q2) and np.array_equal(st, s2)
    w = rng.standard_normal((256, 384)).astype(np.float32)
    qa, sa = orc.quant_w_128x128(w)
    qb, sb = orc.quant_w_128x128(np.ascontiguousarray(w.T))
    assert np.array_equal(qb, qa.T) and np.array_equal(sb, sa.T)


def test_block_of_identical_rows_equals_tile_result():
    rng = np.random.default_rng(10)
    row = rng.standard_normal((1, 128)).astype(np.float32)
    qa, sa = orc.quant_act_1x128(row)
    qw, sw = orc.quant_w_128x128(np.repeat(row, 128, axis=0))
    assert np.all(qw == qa) and sw[0, 0] == sa[0, 0]


def test_zero_group_and_ragged_tail():
    x = np.zeros((2, 200), dtype=np.float32)
    x[1, 130] = 3.0
    q, s = orc.quant_act_1x128(x)
    assert s.shape == (2, 2) and s[0, 0] == 1 and s[0, 1] == 1 and s[1, 0] == 1
    assert s[1, 1] == np.float32(3.0) / np.float32(448.0)
    assert q[1, 130] == 0x7E and np.count_nonzero(q) == 1


def test_rejects_non_finite_and_wrong_dtype():
    x = np.ones((1, 128), dtype=np.float32)
    x[0, 3] = np.inf
    with pytest.raises(ValueError):
        orc.quant_act_1x128(x)
    with pytest.raises(TypeError):
        orc.quant_act_1x128(np.ones((1, 128)))


def test_fine_grained_beats_per_tensor_on_outliers():
    """Section 3.3.2: group-wise scales accommodate outliers.  Sanity, not a parity pin."""
    x, _ = wl.cfg1()
    q, s = orc.quant_act_1x128(x)
    fine = orc.e4m3_decode(q) * np.repeat(s.astype(np.float64), 128, axis=1) - x
    r = np.float32(448) / np.abs(x).max()
    coarse = orc.e4m3_decode(orc.e4m3_encode_rne_sat((x * r).astype(np.float32))) / r - x
    assert np.linalg.norm(fine) < 0.8 * np.linalg.norm(coarse)


def test_round_to_bf16_against_library_cast_and_ties():
    import torch
    rng = np.random.default_rng(81)
    x = np.concatenate([rng.standard_normal(20000) * np.exp(rng.standard_normal(20000) * 8),
                        [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 0.0, -0.0, 2.0 ** -120]]).astype(np.float32)
    got = orc.round_to_bf16(x)
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), lib.view(np.uint32))
    assert got[-6] == 1.0 and got[-5] == np.float32(1.0 + 2.0 ** -6)     # ties go to the even significand
    assert np.array_equal(got, wl.bf16_round(x))                          # the generators' own rounding agrees


def test_swiglu_quant_is_the_composition_and_closed_forms():
    h = wl.normal((5, 512), 2.0, 82)
    q, s = orc.swiglu_quant_1x128(h)
    act = orc.swiglu(h)
    # every dequantised value is within BF16 rounding plus half an E4M3 step of the FP64 activation
    deq = orc.dequant_rows(q, s)
    amax = np.abs(act.reshape(5, 2, 128)).max(axis=2)
    step = np.repeat(amax / 448 * 2.0 ** 4, 128, axis=1)                  # coarsest E4M3 step, times the scale
    assert np.all(np.abs(deq - act) <= step + np.abs(act) * 2.0 ** -8)
    # gate == 0 gives an all-zero tile: scale 1, zero codes
    h0 = h.copy(); h0[:, :256] = 0
    q0, s0 = orc.swiglu_quant_1x128(h0)
    assert np.all(s0 == 1.0) and np.all((q0 & 0x7F) == 0)
    # a large positive gate passes `up` through: silu(g) -> g
    h1 = np.zeros((1, 256), np.float32); h1[0, :128] = 64.0; h1[0, 128:] = np.linspace(-1, 1, 128, dtype=np.float32)
    q1, s1 = orc.swiglu_quant_1x128(h1)
    q1r, s1r = orc.quant_act_1x128(orc.round_to_bf16(64.0 * h1[:, 128:].astype(np.float64)))
    assert np.array_equal(q1, q1r) and np.array_equal(s1, s1r)
    # power-of-two form: same activation, scales rounded up
    q2, s2 = orc.swiglu_quant_1x128(h, pow2=True)
    assert np.all(s2 >= s) and np.all(s2 < 2 * s.astype(np.float64))


@pytest.mark.parametrize("pow2", [False, True])
def test_dual_weight_quantization_is_a_transposition(pow2):
    """Appendix B.2: block-wise (128x128) tiles only need transposing for the backward
    pass.  The oracle quantizes W and W^T independently; codes and scales must be
    transposes of each other, also with ragged edge blocks."""
    w = wl.normal((200, 392), 0.02, 83)
    w[5, 300] = 1.5
    q, s, q_t, s_t = orc.quant_w_128x128_dual(w, pow2=pow2)
    assert q.shape == (200, 392) and q_t.shape == (392, 200) and s.shape == (2, 4) and s_t.shape == (4, 2)
    assert np.array_equal(q_t, q.T) and np.array_equal(s_t, s.T)
    # and Dgrad through the transposed codes equals the exact product of the dequantized operands
    dy = wl.normal((128, 200), 1.0, 84)[:, :128]
    qa, sa = orc.quant_act_1x128(np.ascontiguousarray(dy))
    wq = orc.dequant_blocks(q, s)[:128]                       # [128][392], rows = the contracted axis
    ref = orc.dequant_rows(qa, sa) @ wq
    got = orc.gemm_fp8_bs(qa, sa, q_t[:, :128], s_t[:, :1])
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_rmsnorm_closed_forms_library_and_composition():
    import torch
    rng = np.random.default_rng(85)
    x = wl.cfg2_x(m=6, k=512)
    gamma = (1.0 + 0.1 * rng.standard_normal(512)).astype(np.float32)
    y = orc.rmsnorm(x, gamma, 1e-6)
    # library third opinion
    lib = torch.nn.functional.rms_norm(torch.from_numpy(x).double(), (512,), torch.from_numpy(gamma).double(), 1e-6).numpy()
    assert np.allclose(y, lib, rtol=1e-12, atol=1e-14)
    # with unit gain and no eps every row has unit mean square; scaling the input changes nothing
    y1 = orc.rmsnorm(x, np.ones(512, np.float32), 0.0)
    assert np.allclose(np.mean(y1 * y1, axis=1), 1.0, rtol=1e-12)
    assert np.allclose(orc.rmsnorm(3.5 * x.astype(np.float64), np.ones(512), 0.0), y1, rtol=1e-12)
    # a constant row normalises to +-gamma
    c = np.full((1, 512), -2.5, np.float32)
    assert np.allclose(orc.rmsnorm(c, gamma, 0.0), -gamma[None, :].astype(np.float64), rtol=1e-12)
    # eps dominates a zero row: output zero, quantized as an all-zero tile
    q0, s0 = orc.rmsnorm_quant_1x128(np.zeros((1, 512), np.float32), gamma, 1e-6)
    assert np.all(s0 == 1.0) and np.all(q0 == 0)
    # the fused definition is the composition of its parts
    q, s = orc.rmsnorm_quant_1x128(x, gamma, 1e-6)
    q2, s2 = orc.quant_act_1x128(orc.round_to_bf16(y))
    assert np.array_equal(q, q2) and np.array_equal(s, s2)
