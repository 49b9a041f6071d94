"""Pins of the oracle's optimizer step (Algorithm 1, "optimizer.step()") against PyTorch's CPU
optimizers in float64, closed forms, and the row form against a dense step on the touched rows."""
import numpy as np
import pytest


def test_adam_matches_torch_over_several_steps(orc):
    import torch
    rng = np.random.default_rng(0)
    p0 = rng.normal(0, 1, (7, 5))
    grads = [rng.normal(0, 1, (7, 5)) * 10.0 ** rng.integers(-3, 2) for _ in range(6)]
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.Adam([tp], lr=0.01, betas=(0.9, 0.999), eps=1e-8)
    p = p0.copy(); m = np.zeros_like(p); v = np.zeros_like(p)
    for t, g in enumerate(grads, 1):
        tp.grad = torch.from_numpy(g.copy())
        opt.step()
        orc.optimizer_step(1, p, g, m, v, 0.01, 0.9, 0.999, 1e-8, t)
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_sgd_matches_torch_and_closed_form(orc):
    import torch
    rng = np.random.default_rng(1)
    p0 = rng.normal(0, 1, 33); g = rng.normal(0, 1, 33)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.SGD([tp], lr=0.01)
    tp.grad = torch.from_numpy(g.copy()); opt.step()
    p = p0.copy()
    orc.optimizer_step(0, p, g, None, None, 0.01)
    np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-15)
    np.testing.assert_allclose(p, p0 - 0.01 * g, rtol=1e-15)


def test_first_adam_step_moves_by_lr_times_sign(orc):
    """t = 1: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps)."""
    g = np.array([3.0, -0.5, 1e-3, 0.0, -7.0])
    p = np.zeros(5); m = np.zeros(5); v = np.zeros(5)
    orc.optimizer_step(1, p, g, m, v, 0.01, 0.9, 0.999, 1e-8, 1)
    np.testing.assert_allclose(p, -0.01 * g / (np.abs(g) + 1e-8), rtol=1e-12, atol=0)
    assert p[3] == 0.0 and m[3] == 0.0 and v[3] == 0.0


def test_row_form_touches_only_masked_rows(orc):
    rng = np.random.default_rng(2)
    p0 = rng.normal(0, 1, (9, 4)); g = rng.normal(0, 1, (9, 4))
    m0 = rng.normal(0, 0.1, (9, 4)); v0 = rng.uniform(0, 0.1, (9, 4))
    mask = np.array([1, 0, 0, 1, 1, 0, 0, 0, 1], np.uint8)
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    orc.optimizer_step(1, p, g, m, v, 0.01, 0.9, 0.999, 1e-8, 4, row_mask=mask)
    rows = mask.astype(bool)
    pd, md, vd = p0[rows].copy(), m0[rows].copy(), v0[rows].copy()
    orc.optimizer_step(1, pd, g[rows], md, vd, 0.01, 0.9, 0.999, 1e-8, 4)
    np.testing.assert_array_equal(p[rows], pd); np.testing.assert_array_equal(m[rows], md)
    np.testing.assert_array_equal(v[rows], vd)
    np.testing.assert_array_equal(p[~rows], p0[~rows]); np.testing.assert_array_equal(m[~rows], m0[~rows])
    np.testing.assert_array_equal(v[~rows], v0[~rows])
