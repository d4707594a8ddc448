"""Pins for the optimizer oracle (oracle/optimizer.py): closed forms of the published update rule, and
the same steps taken by stock PyTorch (torch.optim.AdamW, clip_grad_norm_) in fp64 on the CPU."""
import numpy as np
import pytest
import torch

from oracle import optimizer as oo


def test_first_step_closed_form():
    """With zero moments the bias corrections cancel the (1 - beta) factors: m_hat = g, v_hat = g^2, so
    the step is lr * g / (|g| + eps) on top of the decayed parameter - a sign step for |g| >> eps."""
    rng = np.random.default_rng(0)
    p, g = rng.standard_normal(1000), rng.standard_normal(1000)
    lr, wd, eps = 3e-4, 0.1, 1e-8
    pn, mn, vn = oo.adamw_step(p, g, np.zeros_like(p), np.zeros_like(p), 1, lr, 0.9, 0.95, eps, wd)
    np.testing.assert_allclose(mn, 0.1 * g, rtol=1e-13)
    np.testing.assert_allclose(vn, 0.05 * g * g, rtol=1e-13)
    np.testing.assert_allclose(pn, p * (1 - lr * wd) - lr * g / (np.abs(g) + eps), rtol=0, atol=1e-15)
    big = np.abs(g) > 1e-3
    np.testing.assert_allclose((p * (1 - lr * wd) - pn)[big], lr * np.sign(g)[big], rtol=1e-4)


def test_zero_gradient_is_pure_weight_decay():
    rng = np.random.default_rng(1)
    p = rng.standard_normal(257)
    pn, mn, vn = oo.adamw_step(p, np.zeros_like(p), np.zeros_like(p), np.zeros_like(p), 7, 1e-2, weight_decay=0.3)
    np.testing.assert_allclose(pn, p * (1 - 1e-2 * 0.3), rtol=1e-15)
    assert not mn.any() and not vn.any()
    # and with decay switched off and a gradient present the parameter moves against the gradient
    g = rng.standard_normal(257)
    pn, _, _ = oo.adamw_step(p, g, np.zeros_like(p), np.zeros_like(p), 1, 1e-2, weight_decay=0.0)
    assert np.all(np.sign(p - pn) == np.sign(g))


def test_clipping_closed_forms():
    a, b = np.full((3, 4), 2.0), np.full(5, -1.0)
    n = oo.global_grad_norm([a, b])
    assert n == pytest.approx(np.sqrt(12 * 4 + 5), rel=1e-15)
    assert oo.clip_coefficient(n, 100.0) == 1.0                       # inside the ball: identity
    assert oo.clip_coefficient(n, n * (1 + 1e-3)) == 1.0
    c = oo.clip_coefficient(n, 1.0)
    assert c == pytest.approx(1.0 / (n + 1e-6), rel=1e-15)
    assert oo.global_grad_norm([c * a, c * b]) == pytest.approx(1.0, rel=1e-6)   # clipped onto the sphere
    assert oo.global_grad_norm([]) == 0.0


def test_against_torch_adamw_and_clip_grad_norm():
    """Five steps of three tensors with clipping that binds on some steps: torch.optim.AdamW and
    torch.nn.utils.clip_grad_norm_ in fp64 on the CPU against the oracle, step by step."""
    rng = np.random.default_rng(2)
    shapes = [(17, 5), (64,), (3, 3, 7)]
    hp = dict(lr=2e-3, beta1=0.9, beta2=0.95, eps=1e-3, weight_decay=0.1)   # eps large enough that its place in the formula shows
    max_norm = 4.0
    P = [rng.standard_normal(s) for s in shapes]
    M = [np.zeros(s) for s in shapes]
    V = [np.zeros(s) for s in shapes]
    tp = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in P]
    opt = torch.optim.AdamW(tp, lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"], weight_decay=hp["weight_decay"])
    bound = 0
    for step in range(1, 6):
        G = [rng.standard_normal(s) * (0.2 if step % 2 else 2.0) for s in shapes]
        for t, g in zip(tp, G):
            t.grad = torch.tensor(g, dtype=torch.float64)
        tn = float(torch.nn.utils.clip_grad_norm_(tp, max_norm))
        n = oo.global_grad_norm(G)
        assert n == pytest.approx(tn, rel=1e-13)
        c = oo.clip_coefficient(n, max_norm)
        bound += c < 1.0
        for t, g in zip(tp, G):
            np.testing.assert_allclose(t.grad.numpy(), c * g, rtol=1e-12)
        opt.step()
        for i in range(len(shapes)):
            P[i], M[i], V[i] = oo.adamw_step(P[i], G[i], M[i], V[i], step, clip_coef=c, **hp)
            np.testing.assert_allclose(P[i], tp[i].detach().numpy(), rtol=1e-12, atol=1e-14)
            st = opt.state[tp[i]]
            np.testing.assert_allclose(M[i], st["exp_avg"].numpy(), rtol=1e-12, atol=1e-16)
            np.testing.assert_allclose(V[i], st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-16)
    assert 0 < bound < 5      # the test saw both regimes


def test_a_dropped_term_would_fail():
    """The pins above distinguish the rule from its near misses: no bias correction, coupled (L2) decay,
    eps inside the square root."""
    rng = np.random.default_rng(3)
    p, g = rng.standard_normal(50), rng.standard_normal(50)
    m, v = rng.standard_normal(50) * 0.1, rng.random(50) * 0.1
    lr, b1, b2, eps, wd, t = 1e-2, 0.9, 0.95, 1e-3, 0.2, 3
    ref, _, _ = oo.adamw_step(p, g, m, v, t, lr, b1, b2, eps, wd)
    mn, vn = b1 * m + (1 - b1) * g, b2 * v + (1 - b2) * g * g
    no_bc = p * (1 - lr * wd) - lr * mn / (np.sqrt(vn) + eps)
    l2 = p - lr / (1 - b1 ** t) * (b1 * m + (1 - b1) * (g + wd * p)) / (np.sqrt(b2 * v + (1 - b2) * (g + wd * p) ** 2) / np.sqrt(1 - b2 ** t) + eps)
    eps_in = p * (1 - lr * wd) - lr / (1 - b1 ** t) * mn / np.sqrt(vn / (1 - b2 ** t) + eps)
    for wrong in (no_bc, l2, eps_in):
        assert np.max(np.abs(wrong - ref)) > 1e-5
