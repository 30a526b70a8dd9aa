"""Pins for the oracle's AdamW step with BF16 moments (Section 3.3.3, Low-Precision
Optimizer States; hyper-parameters of Section 4.2).  CPU only."""
import numpy as np
import torch

from oracle import ds3_oracle as orc

HP = dict(lr=2.2e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def test_textbook_form_matches_library_optimizer_over_several_steps():
    rng = np.random.default_rng(91)
    w0 = rng.standard_normal(257)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.AdamW([p], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"], weight_decay=HP["weight_decay"])
    w, m, v = w0.copy(), np.zeros(257), np.zeros(257)
    for t in range(1, 6):
        g = rng.standard_normal(257) * 10.0 ** rng.integers(-3, 2)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        w, m, v, _ = orc.adamw_step(w, g, m, v, step=t, bf16_moments=False, **HP)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-15), t


def test_first_step_closed_form():
    g = np.array([0.5, -2.0, 1e-3, 0.0])
    w0 = np.array([1.0, -1.0, 0.25, 3.0])
    w, m, v, _ = orc.adamw_step(w0, g, np.zeros(4), np.zeros(4), step=1, bf16_moments=False, **HP)
    # bias correction undoes the (1 - beta) factors: the step is g / (|g| + eps), plus decoupled decay
    want = w0 - HP["lr"] * (g / (np.abs(g) + HP["eps"]) + HP["weight_decay"] * w0)
    assert np.allclose(w, want, rtol=1e-13)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.05 * g * g)


def test_bf16_moment_storage():
    rng = np.random.default_rng(92)
    n = 4096
    w0 = rng.standard_normal(n).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    m0 = orc.round_to_bf16(rng.standard_normal(n) * 1e-3)
    v0 = orc.round_to_bf16(np.abs(rng.standard_normal(n)) * 1e-5)
    w, m, v, wb = orc.adamw_step(w0, g, m0, v0, step=7, **HP)
    wf, mf, vf, _ = orc.adamw_step(w0, g, m0, v0, step=7, bf16_moments=False, **HP)
    # stored moments are BF16 values within half a BF16 ulp of the exact ones; weights are the FP32 rounding
    for got, exact in ((m, mf), (v, vf)):
        assert np.array_equal(got, orc.round_to_bf16(got))
        assert np.all(np.abs(got - exact) <= np.abs(exact) * 2.0 ** -8)
    assert np.array_equal(w, wf.astype(np.float32))
    assert np.array_equal(wb, orc.round_to_bf16(w))
    assert w.dtype == np.float32 and m.dtype == np.float32
