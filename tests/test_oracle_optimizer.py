"""Pins for the oracle's Adam step, update schedule and parameter activations."""
import numpy as np
import pytest
import torch

import oracle


def test_adam_matches_the_library_optimizer_over_several_steps():
    rng = np.random.default_rng(0)
    p0 = rng.normal(size=(50, 7))
    grads = [rng.normal(size=p0.shape) * 10.0 ** rng.integers(-6, 2) for _ in range(8)]
    for eps in (1e-15, 1e-8):
        tp = torch.tensor(p0.copy(), dtype=torch.float64, requires_grad=True)
        opt = torch.optim.Adam([tp], lr=3e-3, betas=(0.9, 0.999), eps=eps)
        p = p0.copy(); m = np.zeros_like(p); v = np.zeros_like(p)
        for t, g in enumerate(grads, 1):
            tp.grad = torch.tensor(g)
            opt.step()
            oracle.adam_step(p, g, m, v, t, 3e-3, eps=eps)
            assert np.allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_adam_first_step_closed_form_and_gradient_scale():
    g = np.array([1e-3, -2.0, 0.0, 5e-9])
    p = np.ones(4); m = np.zeros(4); v = np.zeros(4)
    oracle.adam_step(p, g, m, v, 1, 0.01, eps=1e-15)
    # first step: m_hat = g, v_hat = g^2  =>  step = lr * g / (|g| + eps) = lr * sign(g)
    assert np.allclose(p, 1 - 0.01 * np.sign(g), atol=1e-8)
    p2 = np.ones(4); m2 = np.zeros(4); v2 = np.zeros(4)
    oracle.adam_step(p2, 32 * g, m2, v2, 1, 0.01, eps=1e-15, grad_scale=1 / 32)
    assert np.allclose(m2, m) and np.allclose(v2, v) and np.allclose(p2, p)


def test_adam_minimises_a_quadratic():
    p = np.array([3.0, -2.0]); m = np.zeros(2); v = np.zeros(2)
    for t in range(1, 2001):
        oracle.adam_step(p, 2 * (p - np.array([1.0, 0.5])), m, v, t, 0.01)
    assert np.allclose(p, [1.0, 0.5], atol=1e-3)


def test_update_schedule():
    assert [oracle.adam_interval(i) for i in (0, 14999, 15000, 19999, 20000, 29999)] == [1, 1, 32, 32, 64, 64]


def test_activations_and_their_chain_rule_by_finite_differences():
    rng = np.random.default_rng(1)
    rs, rq, ro = rng.normal(-2, 1, (6, 3)), rng.normal(size=(6, 4)), rng.normal(size=6)
    s, q, o = oracle.activate(rs, rq, ro)
    assert np.allclose(np.log(s), rs) and np.allclose((q * q).sum(1), 1) and np.allclose(np.log(o / (1 - o)), ro)
    assert np.allclose(q * np.sqrt((rq * rq).sum(1, keepdims=True)), rq)
    ws, wq, wo = rng.normal(size=s.shape), rng.normal(size=q.shape), rng.normal(size=o.shape)
    f = lambda a, b, c: sum((w * x).sum() for w, x in zip((ws, wq, wo), oracle.activate(a, b, c)))
    gs, gq, go = oracle.activate_bwd(rs, rq, ro, ws, wq, wo)
    h = 1e-6
    for arr, grad in ((rs, gs), (rq, gq), (ro, go)):
        flat, gf = arr.reshape(-1), grad.reshape(-1)
        for j in range(flat.size):
            old = flat[j]
            flat[j] = old + h; fp = f(rs, rq, ro)
            flat[j] = old - h; fm = f(rs, rq, ro)
            flat[j] = old
            assert gf[j] == pytest.approx((fp - fm) / (2 * h), rel=1e-6, abs=1e-9)
