"""GPU parity of the power-of-two-scale path (Section 3.3.3): the three *_pow2
quantizers bit for bit against the oracle, and the GEMMs that let the matrix
instruction apply the scales against the FP64 oracle on the same codes and
scales (same tolerances as the general GEMM; bit-exact where every partial sum
is exactly representable)."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from synth import workloads as wl
from tests._gpu_util import announce, dev, host, normwise

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL_F32 = 1e-4


def _same(q, s, q_ref, s_ref, what):
    q, s = host(q), host(s)
    assert q.shape == q_ref.shape and s.shape == s_ref.shape, what
    bad = np.argwhere(q != q_ref)
    assert bad.size == 0, f"{what}: {bad.shape[0]} code mismatches, first at {bad[0]}"
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32)), f"{what}: scales differ"


def _kmajor(s):
    return dev(np.ascontiguousarray(s.T)).t()


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("shape", [(512, 7168), (33, 1160), (1, 128), (300, 200)])
def test_quantizers_pow2(ds3, shape, bf16):
    announce(f"pow2 quantizers {shape} bf16={bf16}")
    x = wl.cfg2_x(m=shape[0], k=shape[1])
    if not bf16:
        x = (x * np.float32(1.2345)).astype(np.float32)     # full FP32 significands
    xr = x
    _same(*ds3.ds3_quant_act_1x128_pow2(dev(x, bf16=bf16)), *orc.quant_act_1x128(xr, pow2=True), "1x128")
    _same(*ds3.ds3_quant_act_1x128_pow2(dev(x, bf16=bf16), k_major_scales=False), *orc.quant_act_1x128(xr, pow2=True), "1x128 row-major")
    _same(*ds3.ds3_quant_act_128x1_pow2(dev(x, bf16=bf16)), *orc.quant_act_128x1(xr, pow2=True), "128x1")
    _same(*ds3.ds3_quant_w_128x128_pow2(dev(x, bf16=bf16)), *orc.quant_w_128x128(xr, pow2=True), "128x128")


def test_quantizer_pow2_binade_boundaries(ds3):
    """Tiles whose max-abs sits on, one ulp below and one ulp above 448 * 2^j, and at
    the ends of the supported magnitude range."""
    announce("pow2 boundaries")
    rng = np.random.default_rng(71)
    rows = []
    for j in list(range(-30, 31, 3)) + [-100 + 9, 100 - 9]:
        top = np.float32(448.0) * np.float32(2.0) ** j
        for amax in (top, np.nextafter(top, np.float32(0)), np.nextafter(top, np.float32(np.inf)),
                     np.float32(1.0) * np.float32(2.0) ** j, np.float32(1.9999999) * np.float32(2.0) ** j):
            t = (rng.random(128).astype(np.float32) * 2 - 1) * amax
            t[rng.integers(0, 128)] = amax
            rows.append(t.astype(np.float32))
    x = np.stack(rows)
    _same(*ds3.ds3_quant_act_1x128_pow2(dev(x)), *orc.quant_act_1x128(x, pow2=True), "boundaries")


@pytest.mark.parametrize("shape", [(256, 512, 1024), (300, 576, 256), (17, 130, 384), (1, 4, 128), (2048, 9216, 256)])
def test_gemm_pow2_exact(ds3, shape):
    """Small-integer codes and power-of-two scales over 40 binades: every partial
    sum is exact in FP32 however the scales are applied, so the FP32 output must
    equal the oracle bit for bit, in block mode and in per-row mode."""
    m, n, k = shape
    rng = np.random.default_rng(72)
    table = np.array([0x00, 0x38, 0x40, 0xB8, 0xC0, 0x80], dtype=np.uint8)
    a, b = table[rng.integers(0, 6, (m, k))], table[rng.integers(0, 6, (n, k))]
    # per output element the scale products span at most 2^6, so sums of <= 2^13 terms of |p| <= 512 stay exact
    base_a = rng.integers(-20, 20, (m, 1))
    sa = np.ldexp(1.0, base_a + rng.integers(0, 4, (m, k // 128))).astype(np.float32)
    for per_row in (False, True):
        nb = n if per_row else (n + 127) // 128
        base_b = rng.integers(-20, 20, (nb, 1))
        sb = np.ldexp(1.0, base_b + rng.integers(0, 4, (nb, k // 128))).astype(np.float32)
        ref = orc.gemm_fp8_bs(a, sa, b, sb, sb_per_row=per_row)
        assert np.array_equal(ref.astype(np.float32).astype(np.float64), ref)
        mode = ds3.DS3_BSCALE_PER_ROW if per_row else ds3.DS3_BSCALE_128x128
        for v in range(ds3.ds3_gemm_num_variants()):
            announce(f"pow2 exact {shape} per_row={per_row} variant {v}")
            c = host(ds3.ds3_gemm_fp8_bs_pow2(dev(a), _kmajor(sa), dev(b), dev(sb), sb_mode=mode,
                                              out_dtype=torch.float32, variant=v))
            bad = np.argwhere(c.astype(np.float64) != ref)
            assert bad.size == 0, f"variant {v}: {bad.shape[0]} mismatches, first {bad[0]}: {c[tuple(bad[0])]} vs {ref[tuple(bad[0])]}"


def test_layer_pow2_end_to_end_and_against_general_path(ds3):
    """Quantize with power-of-two factors, multiply with the scaled-MFMA GEMM and with
    the general GEMM: both must meet the oracle on the same codes and scales."""
    x, w = wl.cfg2_x(m=384, k=2048), wl.cfg2_w(n=640, k=2048)
    qa, sa = ds3.ds3_quant_act_1x128_pow2(dev(x, bf16=True))
    qb, sb = ds3.ds3_quant_w_128x128_pow2(dev(w, bf16=True))
    qa_ref, sa_ref = orc.quant_act_1x128(wl.bf16_round(x), pow2=True)
    qb_ref, sb_ref = orc.quant_w_128x128(wl.bf16_round(w), pow2=True)
    _same(qa, sa, qa_ref, sa_ref, "X")
    _same(qb, sb, qb_ref, sb_ref, "W")
    ref = orc.gemm_fp8_bs(qa_ref, sa_ref, qb_ref, sb_ref)
    exact = wl.bf16_round(x).astype(np.float64) @ wl.bf16_round(w).astype(np.float64).T
    print("layer error with power-of-two factors:", normwise(ref, exact))
    for v in range(ds3.ds3_gemm_num_variants()):
        announce(f"pow2 layer variant {v}")
        e32 = normwise(host(ds3.ds3_gemm_fp8_bs_pow2(qa, sa, qb, sb, out_dtype=torch.float32, variant=v)), ref)
        e16 = normwise(host(ds3.ds3_gemm_fp8_bs_pow2(qa, sa, qb, sb, variant=v)), ref)
        g32 = normwise(host(ds3.ds3_gemm_fp8_bs(qa, sa, qb, sb, out_dtype=torch.float32, variant=v)), ref)
        print(f"variant {v}: scaled-MFMA fp32 {e32:.3e} bf16 {e16:.3e}; general path fp32 {g32:.3e}")
        assert e32 <= TOL_F32 and e16 <= TOL_BF16 and g32 <= TOL_F32


@pytest.mark.parametrize("shape", [(200, 576, 7168), (1000, 100, 512)])
def test_gemm_pow2_random_codes(ds3, shape):
    m, n, k = shape
    rng = np.random.default_rng(73)
    a = rng.integers(0, 0x7F, (m, k)).astype(np.uint8) | (rng.integers(0, 2, (m, k)) << 7).astype(np.uint8)
    b = rng.integers(0, 0x7F, (n, k)).astype(np.uint8) | (rng.integers(0, 2, (n, k)) << 7).astype(np.uint8)
    sa = np.ldexp(1.0, rng.integers(-12, 4, (m, k // 128))).astype(np.float32)
    sb = np.ldexp(1.0, rng.integers(-12, 4, ((n + 127) // 128, k // 128))).astype(np.float32)
    ref = orc.gemm_fp8_bs(a, sa, b, sb)
    for v in range(ds3.ds3_gemm_num_variants()):
        announce(f"pow2 random {shape} variant {v}")
        e32 = normwise(host(ds3.ds3_gemm_fp8_bs_pow2(dev(a), _kmajor(sa), dev(b), dev(sb), out_dtype=torch.float32, variant=v)), ref)
        e16 = normwise(host(ds3.ds3_gemm_fp8_bs_pow2(dev(a), _kmajor(sa), dev(b), dev(sb), variant=v)), ref)
        print(f"{shape} variant {v}: fp32 {e32:.3e} bf16 {e16:.3e}")
        assert e32 <= TOL_F32 and e16 <= TOL_BF16


def test_wgrad_pow2_with_accumulate(ds3):
    t, n_out, n_in = 512, 200, 336
    rng = np.random.default_rng(74)
    dy = wl.normal((t, n_out), 1e-2, 741)
    x = wl.cfg2_x(m=t, k=n_in)
    qy, sy = ds3.ds3_quant_act_128x1_pow2(dev(dy, bf16=True))
    qx, sx = ds3.ds3_quant_act_128x1_pow2(dev(x, bf16=True))
    qy_ref, sy_ref = orc.quant_act_128x1(wl.bf16_round(dy), pow2=True)
    qx_ref, sx_ref = orc.quant_act_128x1(wl.bf16_round(x), pow2=True)
    _same(qy, sy, qy_ref, sy_ref, "dY")
    _same(qx, sx, qx_ref, sx_ref, "X")
    dw0 = rng.standard_normal((n_out, n_in)).astype(np.float32)
    ref = orc.gemm_fp8_bs(qy_ref, sy_ref, qx_ref, sx_ref, sb_per_row=True, c_in=dw0)
    for v in range(ds3.ds3_gemm_num_variants()):
        announce(f"pow2 wgrad variant {v}")
        dw = dev(dw0.copy())
        ds3.ds3_gemm_fp8_bs_pow2(qy, sy, qx, sx, sb_mode=ds3.DS3_BSCALE_PER_ROW, c=dw, accumulate=True, variant=v)
        e = normwise(host(dw), ref)
        print(f"pow2 wgrad variant {v}: {e:.3e}")
        assert e <= TOL_F32


def test_grouped_pow2(ds3):
    rng = np.random.default_rng(75)
    sizes = np.array([0, 300, 1, 129, 0, 256, 77], dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    g, n, k, rows = len(sizes), 384, 512, int(off[-1])
    table = np.array([0x00, 0x38, 0x40, 0xB8, 0xC0, 0x80], dtype=np.uint8)
    a, b = table[rng.integers(0, 6, (rows, k))], table[rng.integers(0, 6, (g, n, k))]
    sa = np.ldexp(1.0, rng.integers(-3, 1, (rows, k // 128))).astype(np.float32)
    sb = np.ldexp(1.0, rng.integers(-2, 2, (g, n // 128, k // 128))).astype(np.float32)
    ref = orc.grouped_gemm_fp8_bs(a, sa, off, b, sb)
    for v in range(ds3.ds3_gemm_num_variants()):
        announce(f"pow2 grouped variant {v}")
        c = host(ds3.ds3_grouped_gemm_fp8_bs_pow2(dev(a), _kmajor(sa), dev(off), dev(b), dev(sb), out_dtype=torch.float32, variant=v))
        assert np.array_equal(c.astype(np.float64), ref), v


@pytest.mark.parametrize("pow2", [False, True])
@pytest.mark.parametrize("k_major", [True, False])
@pytest.mark.parametrize("shape", [(512, 1024), (300, 208), (4096, 256), (1, 16), (131, 2048)])
def test_retile_cached_activation(ds3, shape, k_major, pow2):
    """FP8 1x128 cache -> 128x1 tiles (Section 3.5.2), bit for bit against the oracle on
    the same cached codes and scales; the cache itself comes from the GPU quantizer of
    matching kind (checked against the oracle elsewhere)."""
    announce(f"retile {shape} k_major={k_major} pow2={pow2}")
    x = wl.cfg2_x(m=shape[0], k=shape[1])
    q, s = (ds3.ds3_quant_act_1x128_pow2 if pow2 else ds3.ds3_quant_act_1x128)(dev(x, bf16=True), k_major_scales=k_major)
    fn = ds3.ds3_retile_1x128_to_128x1_pow2 if pow2 else ds3.ds3_retile_1x128_to_128x1
    qt, st = fn(q, s, k_major_scales=k_major)
    qt_ref, st_ref = orc.retile_1x128_to_128x1(host(q), host(s), pow2=pow2)
    _same(qt, st, qt_ref, st_ref, "retile")


def test_wgrad_from_retiled_cache(ds3):
    """The weight-gradient GEMM fed from the re-tiled FP8 cache of X (and dY quantized
    along tokens from BF16) against the FP64 oracle on the same codes."""
    announce("wgrad from cache")
    t, n_out, n_in = 512, 256, 384
    x, dy = wl.cfg2_x(m=t, k=n_in), wl.normal((t, n_out), 1e-2, 761)
    qx, sx = ds3.ds3_quant_act_1x128(dev(x, bf16=True))                   # what Fprop cached
    qxt, sxt = ds3.ds3_retile_1x128_to_128x1(qx, sx)
    qyt, syt = ds3.ds3_quant_act_128x1(dev(dy, bf16=True))
    ref = orc.gemm_fp8_bs(host(qyt), host(syt), host(qxt), host(sxt), sb_per_row=True)
    dw = host(ds3.ds3_gemm_fp8_bs(qyt, syt, qxt, sxt, sb_mode=ds3.DS3_BSCALE_PER_ROW, out_dtype=torch.float32))
    assert normwise(dw, ref) <= TOL_F32
    # the extra quantization step costs accuracy against the unquantized gradient, within a few percent
    exact = dy.astype(np.float64).T @ x.astype(np.float64)
    e = normwise(dw, exact)
    print("wgrad from re-tiled cache vs unquantized:", e)
    assert e < 0.06
