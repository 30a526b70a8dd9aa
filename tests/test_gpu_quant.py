"""GPU parity of the three quantizers and SwiGLU against the CPU oracle.
Codes and scales must match bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from synth import workloads as wl
from tests._gpu_util import announce, dev, host

pytestmark = pytest.mark.gpu


def _cmp_codes_scales(q, s, q_ref, s_ref, what):
    q, s = host(q), host(s)
    assert q.shape == q_ref.shape and s.shape == s_ref.shape, what
    bad = np.argwhere(q != q_ref)
    assert bad.size == 0, f"{what}: {bad.shape[0]} code mismatches, first at {bad[0]}: got {q[tuple(bad[0])]:#x} want {q_ref[tuple(bad[0])]:#x}"
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32)), f"{what}: scales differ"


def test_hardware_cast_is_rne_on_every_grid_point_and_tie(ds3):
    """Drive the hardware FP32->E4M3 conversion through the public 1x128 call:
    a tile whose max-abs is exactly 448 has multiplier 1, so its other 127
    elements are converted as they are."""
    announce("hw cast sweep")
    pos = orc.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))
    pts = np.concatenate([pos, (pos[:-1] + pos[1:]) / 2]).astype(np.float32)
    vals = [pts]
    lo = hi = pts
    for _ in range(3):
        lo = np.nextafter(lo, np.float32(-1))
        hi = np.nextafter(hi, np.float32(1e9))
        vals += [lo, hi]
    rng = np.random.default_rng(1)
    vals.append((rng.random(200_000) * 448).astype(np.float32))
    vals.append(np.ldexp(rng.random(100_000), rng.integers(-20, 9, 100_000)).astype(np.float32))
    v = np.concatenate(vals)
    v = v[(v >= 0) & (v <= 448)]
    v = np.concatenate([v, -v])
    pad = (-v.size) % 127
    v = np.concatenate([v, np.zeros(pad, np.float32)]).reshape(-1, 127)
    x = np.concatenate([np.full((v.shape[0], 1), 448.0, np.float32), v], axis=1)
    q, s = ds3.ds3_quant_act_1x128(dev(x))
    q_ref, s_ref = orc.quant_act_1x128(x)
    assert np.all(s_ref == 1.0)
    _cmp_codes_scales(q, s, q_ref, s_ref, "hw cast")


@pytest.mark.parametrize("k_major", [True, False])
def test_1x128_cfg1_fp32(ds3, k_major):
    announce(f"1x128 cfg1 fp32 k_major={k_major}")
    x, _ = wl.cfg1()
    q, s = ds3.ds3_quant_act_1x128(dev(x), k_major_scales=k_major)
    _cmp_codes_scales(q, s, *orc.quant_act_1x128(x), "cfg1 X")


@pytest.mark.parametrize("shape", [(512, 7168), (33, 1160), (1, 128), (17, 8), (1000, 2048)])
def test_1x128_bf16_shapes(ds3, shape):
    announce(f"1x128 bf16 {shape}")
    x = wl.cfg2_x(m=shape[0], k=shape[1])
    x[0, : min(128, shape[1])] = 0                         # an all-zero tile
    q, s = ds3.ds3_quant_act_1x128(dev(x, bf16=True))
    _cmp_codes_scales(q, s, *orc.quant_act_1x128(x), f"bf16 {shape}")


def test_1x128_fp32_ragged_and_strided(ds3):
    announce("1x128 fp32 ragged, ld > cols")
    rng = np.random.default_rng(2)
    full = rng.standard_normal((70, 1024)).astype(np.float32)
    x = full[:, :836]                                      # 836 = 6*128 + 68, ld = 1024
    xt = dev(full)[:, :836]
    q, s = ds3.ds3_quant_act_1x128(xt)
    _cmp_codes_scales(q, s, *orc.quant_act_1x128(np.ascontiguousarray(x)), "fp32 ragged")


def test_w_128x128_cfg1_fp32(ds3):
    announce("128x128 cfg1 fp32")
    _, w = wl.cfg1()
    q, s = ds3.ds3_quant_w_128x128(dev(w))
    _cmp_codes_scales(q, s, *orc.quant_w_128x128(w), "cfg1 W")


@pytest.mark.parametrize("shape", [(1024, 7168), (576, 1024), (130, 136), (128, 128), (5, 8)])
def test_w_128x128_bf16_shapes(ds3, shape):
    announce(f"128x128 bf16 {shape}")
    w = wl.cfg2_w(n=shape[0], k=shape[1])
    q, s = ds3.ds3_quant_w_128x128(dev(w, bf16=True))
    _cmp_codes_scales(q, s, *orc.quant_w_128x128(w), f"W {shape}")


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("shape", [(512, 1024), (300, 200), (131, 8), (4096, 256)])
@pytest.mark.parametrize("k_major", [True, False])
def test_act_128x1(ds3, shape, bf16, k_major):
    announce(f"128x1 {shape} bf16={bf16} k_major={k_major}")
    x = wl.cfg2_x(m=shape[0], k=shape[1]) if bf16 else wl.normal(shape, 1.0, 77, bf16=False)
    q, s = ds3.ds3_quant_act_128x1(dev(x, bf16=bf16), k_major_scales=k_major)
    _cmp_codes_scales(q, s, *orc.quant_act_128x1(x), f"128x1 {shape}")


def test_quantizers_full_size_sampled(ds3):
    """Config-2 sizes in the launch configuration the benchmark times; the
    oracle checks sampled row bands / blocks plus the edges."""
    announce("full-size cfg2 X and W, sampled")
    x = wl.cfg2_x()
    q, s = ds3.ds3_quant_act_1x128(dev(x, bf16=True))
    q, s = host(q), host(s)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 1, x.shape[0] - 1], rng.integers(0, x.shape[0], 200)]))
    q_ref, s_ref = orc.quant_act_1x128(x[rows])
    assert np.array_equal(q[rows], q_ref) and np.array_equal(s[rows], s_ref)
    del x
    w = wl.cfg2_w()
    qw, sw = ds3.ds3_quant_w_128x128(dev(w, bf16=True))
    qw, sw = host(qw), host(sw)
    nb, kb = sw.shape
    blocks = {(0, 0), (nb - 1, kb - 1), (0, kb - 1), (nb - 1, 0)}
    blocks |= {(int(a), int(b)) for a, b in zip(rng.integers(0, nb, 60), rng.integers(0, kb, 60))}
    for (i, j) in sorted(blocks):
        blk = w[i * 128:(i + 1) * 128, j * 128:(j + 1) * 128]
        q_ref, s_ref = orc.quant_w_128x128(np.ascontiguousarray(blk))
        assert np.array_equal(qw[i * 128:(i + 1) * 128, j * 128:(j + 1) * 128], q_ref), (i, j)
        assert sw[i, j] == s_ref[0, 0], (i, j)
    # token-axis tiles at config-4 size (X of config 2 along tokens), sampled channels
    x = wl.cfg2_x()
    qt, st = ds3.ds3_quant_act_128x1(dev(x, bf16=True))
    qt, st = host(qt), host(st)
    cols = np.unique(np.concatenate([[0, x.shape[1] - 1], rng.integers(0, x.shape[1], 100)]))
    q_ref, s_ref = orc.quant_act_128x1(np.ascontiguousarray(x[:, cols]))
    assert np.array_equal(qt[cols], q_ref) and np.array_equal(st[cols], s_ref)


def test_quantizer_is_deterministic(ds3):
    announce("determinism")
    x = dev(wl.cfg2_x(m=256, k=1024), bf16=True)
    q1, s1 = ds3.ds3_quant_act_1x128(x)
    q2, s2 = ds3.ds3_quant_act_1x128(x)
    assert torch.equal(q1, q2) and torch.equal(s1, s2)


def test_empty_inputs_are_noops(ds3):
    announce("empty inputs")
    x = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda:0")
    q, s = ds3.ds3_quant_act_1x128(x)
    assert q.shape == (0, 128)
    q, s = ds3.ds3_quant_w_128x128(x)
    assert q.shape == (0, 128)


def test_swiglu(ds3):
    announce("swiglu")
    h = wl.normal((300, 512), 2.0, 5)
    out = host(ds3.ds3_swiglu(dev(h, bf16=True)))
    ref = orc.swiglu(h)
    # within one BF16 ulp of the FP64 result (8 significant bits, FP32 evaluation)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -120))) - 7)
    assert np.all(np.abs(out - ref) <= ulp)
    assert np.mean(np.abs(out - ref) <= 0.5 * ulp * 1.001) > 0.99


@pytest.mark.parametrize("pow2", [False, True])
@pytest.mark.parametrize("shape", [(300, 512), (64, 4096), (17, 400), (1, 16)])
def test_swiglu_fused_with_quantizer(ds3, shape, pow2):
    """The fused kernel must equal, bit for bit, the 1x128 quantization of the BF16
    activation that ds3_swiglu writes (itself checked against the oracle above); the
    oracle decides the codes from those same BF16 values.  Against the all-oracle
    composition (FP64 exponential) a BF16 ulp of difference in the activation can move
    a code, so there the agreement is statistical."""
    announce(f"swiglu+quant {shape} pow2={pow2}")
    h = wl.normal(shape, 2.0, 6)
    hd = dev(h, bf16=True)
    fused = (ds3.ds3_swiglu_quant_1x128_pow2 if pow2 else ds3.ds3_swiglu_quant_1x128)(hd)
    act = host(ds3.ds3_swiglu(hd))
    _cmp_codes_scales(*fused, *orc.quant_act_1x128(act, pow2=pow2), "fused vs quant(swiglu)")
    q_ref, s_ref = orc.swiglu_quant_1x128(h, pow2=pow2)
    q, s = host(fused[0]), host(fused[1])
    assert np.mean(q == q_ref) > 0.98 and np.mean(s == s_ref) > 0.9
    deq, deq_ref = orc.dequant_rows(q, s), orc.dequant_rows(q_ref, s_ref)
    assert np.linalg.norm(deq - deq_ref) <= 2e-2 * np.linalg.norm(deq_ref)


@pytest.mark.parametrize("pow2", [False, True])
@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("shape", [(1024, 2048), (576, 1024), (130, 136), (5, 8), (300, 200)])
def test_w_128x128_dual_layout(ds3, shape, bf16, pow2):
    announce(f"dual weight quantizer {shape} bf16={bf16} pow2={pow2}")
    w = wl.normal(shape, 0.02, 7)
    if not bf16:
        w = (w * np.float32(1.2345)).astype(np.float32)
    fn = ds3.ds3_quant_w_128x128_dual_pow2 if pow2 else ds3.ds3_quant_w_128x128_dual
    q, s, q_t, s_t = fn(dev(w, bf16=bf16))
    q_ref, s_ref, qt_ref, st_ref = orc.quant_w_128x128_dual(w, pow2=pow2)
    _cmp_codes_scales(q, s, q_ref, s_ref, "W")
    _cmp_codes_scales(q_t, s_t, qt_ref, st_ref, "W^T")


@pytest.mark.parametrize("pow2", [False, True])
@pytest.mark.parametrize("shape", [(512, 7168), (33, 1536), (5, 512), (3, 200), (1, 8), (9, 8192)])
def test_rmsnorm_fused_with_quantizer(ds3, shape, pow2):
    """The BF16 activation the kernel writes is within one BF16 ulp of the FP64 RMSNorm
    (FP32 sum of squares, FP32 products); its codes and scales must equal, bit for bit,
    the oracle's 1x128 quantization of that same BF16 activation."""
    announce(f"rmsnorm+quant {shape} pow2={pow2}")
    rng = np.random.default_rng(8)
    x = wl.cfg2_x(m=shape[0], k=shape[1])
    gamma = (1.0 + 0.1 * rng.standard_normal(shape[1])).astype(np.float32)
    fn = ds3.ds3_rmsnorm_quant_1x128_pow2 if pow2 else ds3.ds3_rmsnorm_quant_1x128
    q, s, y = fn(dev(x, bf16=True), dev(gamma), 1e-6, want_y=True)
    y = host(y)
    ref = orc.rmsnorm(x, gamma, 1e-6)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -120))) - 7)
    assert np.all(np.abs(y - ref) <= ulp)
    assert np.mean(np.abs(y - ref) <= 0.5 * ulp * 1.001) > 0.99
    _cmp_codes_scales(q, s, *orc.quant_act_1x128(y, pow2=pow2), "fused vs quant(rmsnorm)")
    # without the BF16 output the codes are the same
    q2, s2 = fn(dev(x, bf16=True), dev(gamma), 1e-6)
    assert torch.equal(q2, q) and torch.equal(s2, s)


@pytest.mark.parametrize("shape", [(512, 7168), (33, 1160), (1, 128), (300, 200), (17, 8)])
def test_e5m6_cache_quantizer_and_dequantizer(ds3, shape):
    announce(f"e5m6 {shape}")
    x = wl.cfg2_x(m=shape[0], k=shape[1])
    x[0, : min(128, shape[1])] *= np.float32(2.0 ** -20)            # a tile deep in the subnormal-prone range of its neighbours
    x = wl.bf16_round(x)
    q, s = ds3.ds3_quant_act_1x128_e5m6(dev(x, bf16=True))
    q_ref, s_ref = orc.quant_act_1x128_e5m6(x)
    _cmp_codes_scales(q, s, q_ref, s_ref, "e5m6")
    y = host(ds3.ds3_dequant_e5m6(q, s))
    assert np.array_equal(y.astype(np.float64), orc.dequant_e5m6(q_ref, s_ref))


def test_e5m6_device_rounding_on_every_code_and_tie(ds3):
    """A tile whose max-abs is 65024 has scale 1: its other elements are converted as they are."""
    announce("e5m6 rounding sweep")
    codes = np.array([c for c in range(2048) if (c >> 6) != 31], dtype=np.uint16)
    pos = orc.e5m6_decode(codes)
    pts = np.concatenate([pos, (pos[:-1] + pos[1:]) / 2])
    pts = np.concatenate([pts, np.nextafter(pts.astype(np.float32), np.float32(0)), np.nextafter(pts.astype(np.float32), np.float32(1e9))])
    v = wl.bf16_round(pts.astype(np.float32))                        # the kernel takes BF16 input
    v = np.unique(v[(v >= 0) & (v <= 65024)])
    v = np.concatenate([v, -v])
    pad = (-v.size) % 127
    v = np.concatenate([v, np.zeros(pad, np.float32)]).reshape(-1, 127)
    x = np.concatenate([np.full((v.shape[0], 1), 65024.0, np.float32), v], axis=1)
    q, s = ds3.ds3_quant_act_1x128_e5m6(dev(x, bf16=True))
    q_ref, s_ref = orc.quant_act_1x128_e5m6(x)
    assert np.all(s_ref == 1.0)
    _cmp_codes_scales(q, s, q_ref, s_ref, "e5m6 sweep")
