"""GPU parity of the AdamW step with BF16 moments against the FP64 oracle.
Tolerance: the kernel evaluates the update in FP32 (about 10 roundings per
parameter), so the new master weight may differ from the FP32 rounding of the
FP64 result by a few ulp of the *update* (relative 2e-6 of |delta w|, plus one
ulp of w); a stored moment may differ by one BF16 ulp when the FP32 value falls
within 2^-24 of a rounding boundary, which the test allows for a small fraction
(and where the two terms of a moment cancel, by the FP32 rounding of the terms)."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from tests._gpu_util import announce, dev, host

pytestmark = pytest.mark.gpu

HP = dict(lr=2.2e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


@pytest.mark.parametrize("n", [8, 4096 + 8, 1 << 20])
def test_adamw_bf16_states_three_steps(ds3, n):
    rng = np.random.default_rng(93)
    w = rng.standard_normal(n).astype(np.float32)
    m = orc.round_to_bf16(rng.standard_normal(n) * 1e-3)
    v = orc.round_to_bf16(np.abs(rng.standard_normal(n)) * 1e-5)
    wd, md, vd = dev(w), dev(m, bf16=True), dev(v, bf16=True)
    wb = torch.empty(n, dtype=torch.bfloat16, device=wd.device)
    for t in (3, 4, 5):
        announce(f"adamw n={n} step={t}")
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-4, 0)).astype(np.float32)
        g[::97] = 0.0
        w_ref, m_ref, v_ref, wb_ref = orc.adamw_step(w, g, m, v, step=t, **HP)
        ds3.ds3_adamw_bf16_states(wd, dev(g), md, vd, step=t, w_bf16=wb, **HP)
        w_got, m_got, v_got = host(wd), host(md), host(vd)
        dw = np.abs(w_ref.astype(np.float64) - w.astype(np.float64))
        assert np.all(np.abs(w_got.astype(np.float64) - w_ref) <= 4e-6 * dw + 2.0 ** -23 * np.abs(w_ref) + 1e-30)
        # one BF16 ulp of the result, plus the FP32 rounding of the two terms where they cancel
        for got, ref, mag in ((m_got, m_ref, np.abs(m) + np.abs(g)), (v_got, v_ref, np.abs(v) + g.astype(np.float64) ** 2)):
            assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -7 + mag * 2.0 ** -21 + 1e-37)
            assert np.mean(got == ref) > 0.999
        assert np.array_equal(host(wb), orc.round_to_bf16(w_got))
        w, m, v = w_got, m_got, v_got          # continue from the GPU state


def test_adamw_rejects_bad_arguments(ds3):
    w = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    m = torch.zeros(16, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(ds3.Ds3Error):
        ds3.ds3_adamw_bf16_states(w, w.clone(), m, m.clone(), step=0, **HP)           # steps count from 1
    with pytest.raises(ds3.Ds3Error):
        ds3.ds3_adamw_bf16_states(w[:12], w[:12].clone(), m[:12], m[:12].clone(), step=1, **HP)   # n % 8
