"""Pins for the oracle's SGD step (the update that consumes the privatised gradient): closed forms of
the momentum recursion and a library optimiser as an independent route."""
import numpy as np
import torch

import oracle


def test_no_momentum_is_a_plain_axpy():
    rng = np.random.default_rng(3)
    g, th = rng.standard_normal(1000), rng.standard_normal(1000)
    th2, v2 = oracle.sgd_update(g, th, None, 0.05, 0.0)
    assert v2 is None
    assert np.array_equal(th2, th - 0.05 * g)
    # momentum 0 with a buffer: same step, buffer holds the gradient
    th3, v3 = oracle.sgd_update(g, th, np.full(1000, 7.0), 0.05, 0.0)
    assert np.array_equal(th3, th2) and np.array_equal(v3, g)


def test_constant_gradient_gives_the_geometric_series():
    """v_T = g (1 - mu^T) / (1 - mu);  theta_T = theta_0 - lr g sum_{t=1..T} (1 - mu^t) / (1 - mu)."""
    g = np.array([1.0, -2.0, 0.5, 3.0])
    th = np.zeros(4)
    v = np.zeros(4)
    mu, lr, T = 0.9, 0.1, 25
    for _ in range(T):
        th, v = oracle.sgd_update(g, th, v, lr, mu)
    assert np.allclose(v, g * (1 - mu ** T) / (1 - mu), rtol=1e-13)
    s = sum((1 - mu ** t) / (1 - mu) for t in range(1, T + 1))
    assert np.allclose(th, -lr * g * s, rtol=1e-13)


def test_matches_library_sgd_with_momentum_over_several_steps():
    rng = np.random.default_rng(11)
    p = 257
    th0 = rng.standard_normal(p)
    grads = [rng.standard_normal(p) for _ in range(6)]
    lrs = [0.1, 0.1, 0.05, 0.05, 0.01, 0.01]                      # stepped decay is the caller's schedule
    w = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([w], lr=0.1, momentum=0.9)
    th, v = th0.copy(), np.zeros(p)
    for g, lr in zip(grads, lrs):
        for group in opt.param_groups:
            group["lr"] = lr
        w.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, v = oracle.sgd_update(g, th, v, lr, 0.9)
    assert np.allclose(th, w.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_a_sign_or_order_mistake_would_show():
    g, th, v = np.array([2.0]), np.array([1.0]), np.array([0.5])
    th2, v2 = oracle.sgd_update(g, th, v, 0.25, 0.5)
    assert v2[0] == 0.5 * 0.5 + 2.0            # mu v + g, not mu (v + g)
    assert th2[0] == 1.0 - 0.25 * 2.25         # uses the NEW buffer, and subtracts
