"""Seeded sweep of quantizer shapes: ragged rows and columns, padded input leading
dimension, FP32 and BF16 sources, both scale layouts, general and power-of-two
factors, for every quantizer; codes and scales bit for bit against the oracle."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from synth import workloads as wl
from tests._gpu_util import announce, dev, host

pytestmark = pytest.mark.gpu


def _same(q, s, q_ref, s_ref, what):
    q, s = host(q), host(s)
    assert q.shape == q_ref.shape and s.shape == s_ref.shape, what
    assert np.array_equal(q, q_ref), what + ": codes"
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32)), what + ": scales"


def test_seeded_quantizer_sweep(ds3):
    rng = np.random.default_rng(2026)
    for case in range(40):
        rows = int(rng.choice([1, 2, 15, 16, 17, 100, 127, 128, 129, 255, 256, 257, 400]))
        cols = 16 * int(rng.choice([1, 2, 7, 8, 9, 15, 16, 17, 31, 40, 64, 100]))
        bf16 = bool(rng.integers(0, 2))
        pow2 = bool(rng.integers(0, 2))
        k_major = bool(rng.integers(0, 2))
        pad = 16 * int(rng.integers(0, 3))
        announce(f"quant sweep {case}: {rows}x{cols} bf16={bf16} pow2={pow2} k_major={k_major} pad={pad}")
        x = (rng.standard_normal((rows, cols)) * np.exp(rng.standard_normal((rows, 1)) * 3)).astype(np.float32)
        x[rng.integers(0, rows), rng.integers(0, cols)] *= 300.0
        if rows > 3:
            x[2, : min(cols, 128)] = 0.0                       # an all-zero tile
        if bf16:
            x = wl.bf16_round(x)
        buf = torch.zeros((rows, cols + pad), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda:0")
        buf[:, :cols] = dev(x, bf16=bf16)
        xd = buf[:, :cols]                                      # strided view: ld = cols + pad
        sfx = "_pow2" if pow2 else ""
        _same(*getattr(ds3, "ds3_quant_act_1x128" + sfx)(xd, k_major_scales=k_major), *orc.quant_act_1x128(x, pow2=pow2), "1x128")
        _same(*getattr(ds3, "ds3_quant_act_128x1" + sfx)(xd, k_major_scales=k_major), *orc.quant_act_128x1(x, pow2=pow2), "128x1")
        _same(*getattr(ds3, "ds3_quant_w_128x128" + sfx)(xd), *orc.quant_w_128x128(x, pow2=pow2), "128x128")
        q, s, qt, st = getattr(ds3, "ds3_quant_w_128x128_dual" + sfx)(xd)
        q_ref, s_ref, qt_ref, st_ref = orc.quant_w_128x128_dual(x, pow2=pow2)
        _same(q, s, q_ref, s_ref, "dual W")
        _same(qt, st, qt_ref, st_ref, "dual W^T")
        # the cache re-tiling on the codes just produced
        q1, s1 = getattr(ds3, "ds3_quant_act_1x128" + sfx)(xd, k_major_scales=k_major)
        _same(*getattr(ds3, "ds3_retile_1x128_to_128x1" + sfx)(q1, s1, k_major_scales=k_major),
              *orc.retile_1x128_to_128x1(host(q1), host(s1), pow2=pow2), "retile")
        if bf16:
            _same(*ds3.ds3_quant_act_1x128_e5m6(xd, k_major_scales=k_major), *orc.quant_act_1x128_e5m6(x), "e5m6")
