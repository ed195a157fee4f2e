"""Pins for the oracle's per-example gradients and norms.

Routes that do not share the oracle's loops: finite differences through a library forward
pass (exact here: each layer is linear in its parameters), library batch weight gradients,
per-example autograd, plain / im2col GEMMs, and closed-form norms."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import Layer, conv, dense, gn_affine

torch.set_num_threads(4)

CONVS = [
    Layer("conv", 3, 4, 7, 6, 3, 3, 1, 1, True),
    Layer("conv", 2, 5, 9, 8, 3, 3, 2, 1, False),
    Layer("conv", 4, 3, 6, 6, 1, 1, 1, 0, True),
    Layer("conv", 4, 6, 7, 9, 1, 1, 2, 0, False),
    Layer("conv", 3, 2, 11, 13, 7, 7, 2, 3, True),
    Layer("conv", 2, 3, 8, 7, 3, 2, 1, 0, True),      # rectangular kernel, no padding
    Layer("conv", 2, 2, 5, 5, 5, 5, 1, 2, False),     # kernel as large as the image
]


def _rand(layer, n, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n,) + tuple(layer.x_shape)).astype(np.float32)
    dy = rng.standard_normal((n,) + tuple(layer.dy_shape)).astype(np.float32)
    return x, dy


def _conv_forward(layer, x, w, b):
    return F.conv2d(x, w, b, stride=layer.stride, padding=layer.pad)


@pytest.mark.parametrize("layer", CONVS)
def test_conv_finite_differences(layer):
    """l(W) = <dY, conv(X; W, b)> is linear in (W, b): a central difference IS the derivative."""
    x, dy = _rand(layer, 1, 11)
    gw, gb = oracle.example_grad(layer, x[0], dy[0])
    xt = torch.from_numpy(x).double()
    dyt = torch.from_numpy(dy).double()
    w0 = torch.from_numpy(np.random.default_rng(5).standard_normal(layer.w_shape))
    b0 = torch.zeros(layer.cout, dtype=torch.float64)
    assert tuple(_conv_forward(layer, xt, w0, b0).shape[1:]) == tuple(layer.dy_shape)

    def loss(w, b):
        return float((dyt * _conv_forward(layer, xt, w, b)).sum())

    flat = gw.reshape(-1)
    for e in range(flat.size):
        d = torch.zeros(flat.size, dtype=torch.float64)
        d[e] = 1.0
        d = d.reshape(layer.w_shape)
        fd = (loss(w0 + d, b0) - loss(w0 - d, b0)) / 2.0
        assert abs(fd - flat[e]) <= 1e-10 * max(1.0, abs(flat[e])), (e, fd, flat[e])
    if layer.has_bias:
        for e in range(layer.cout):
            d = torch.zeros(layer.cout, dtype=torch.float64)
            d[e] = 1.0
            fd = (loss(w0, b0 + d) - loss(w0, b0 - d)) / 2.0
            assert abs(fd - gb[e]) <= 1e-10 * max(1.0, abs(gb[e]))
    else:
        assert gb is None


@pytest.mark.parametrize("layer", CONVS)
def test_conv_sum_of_examples_is_batch_weight_gradient(layer):
    n = 5
    x, dy = _rand(layer, n, 21)
    total = np.zeros(layer.w_shape)
    for i in range(n):
        gw, _ = oracle.example_grad(layer, x[i], dy[i])
        total += gw
    ref = torch.nn.grad.conv2d_weight(torch.from_numpy(x).double(), layer.w_shape,
                                      torch.from_numpy(dy).double(), stride=layer.stride,
                                      padding=layer.pad).numpy()
    assert np.allclose(total, ref, rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("layer", CONVS[:5])
def test_conv_per_example_autograd(layer):
    n = 3
    x, dy = _rand(layer, n, 31)
    for i in range(n):
        w = torch.zeros(layer.w_shape, dtype=torch.float64, requires_grad=True)
        b = torch.zeros(layer.cout, dtype=torch.float64, requires_grad=True)
        y = _conv_forward(layer, torch.from_numpy(x[i:i + 1]).double(), w, b)
        (y * torch.from_numpy(dy[i:i + 1]).double()).sum().backward()
        gw, gb = oracle.example_grad(layer, x[i], dy[i])
        assert np.allclose(gw, w.grad.numpy(), rtol=1e-11, atol=1e-11)
        if layer.has_bias:
            assert np.allclose(gb, b.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_conv1x1_is_a_plain_gemm_and_kxk_is_im2col_gemm():
    l1 = conv(6, 5, 1, 1, 7)
    x, dy = _rand(l1, 1, 41)
    gw, _ = oracle.example_grad(l1, x[0], dy[0])
    ref = dy[0].reshape(5, -1).astype(np.float64) @ x[0].reshape(6, -1).astype(np.float64).T
    assert np.allclose(gw.reshape(5, 6), ref, rtol=1e-12, atol=1e-12)

    for lk in (conv(3, 4, 3, 1, 8), conv(3, 4, 3, 2, 9), conv(2, 3, 7, 2, 12)):
        x, dy = _rand(lk, 1, 43)
        gw, _ = oracle.example_grad(lk, x[0], dy[0])
        cols = F.unfold(torch.from_numpy(x).double(), (lk.kh, lk.kw), padding=lk.pad, stride=lk.stride)[0]
        ref = dy[0].reshape(lk.cout, -1).astype(np.float64) @ cols.numpy().T       # [cout, cin*kh*kw]
        assert np.allclose(gw.reshape(lk.cout, -1), ref, rtol=1e-12, atol=1e-12)


def test_conv_squared_norm_by_gram_identity():
    """||dW||_F^2 = sum_{s,s'} (U^T U)_{ss'} (dY^T dY)_{ss'} with U the im2col matrix:
    the norm without ever forming dW."""
    lk = conv(3, 4, 3, 1, 6, bias=True)
    x, dy = _rand(lk, 1, 47)
    gw, gb = oracle.example_grad(lk, x[0], dy[0])
    u = F.unfold(torch.from_numpy(x).double(), 3, padding=1)[0].numpy()      # [27, S]
    d = dy[0].reshape(4, -1).astype(np.float64)                                # [4, S]
    want = float(((u.T @ u) * (d.T @ d)).sum())
    assert abs(oracle.sqnorm(gw) - want) <= 1e-11 * want
    assert abs(oracle.sqnorm(gb) - float((d.sum(1) ** 2).sum())) <= 1e-11 * want


@pytest.mark.parametrize("tokens", [1, 5])
def test_dense_gradient_and_closed_form_norm(tokens):
    l = dense(7, 4, tokens=tokens, bias=True)
    x, dy = _rand(l, 2, 51)
    for i in range(2):
        gw, gb = oracle.example_grad(l, x[i], dy[i])
        ref = dy[i].astype(np.float64).T @ x[i].astype(np.float64)       # [out, in]
        assert gw.shape == (4, 7)
        assert np.allclose(gw, ref, rtol=1e-13, atol=1e-13)
        assert np.allclose(gb, dy[i].astype(np.float64).sum(0), rtol=1e-13, atol=1e-13)
        if tokens == 1:   # rank one: ||dW||^2 = ||dy||^2 ||x||^2, ||db||^2 = ||dy||^2
            nx = float((x[i].astype(np.float64) ** 2).sum())
            ny = float((dy[i].astype(np.float64) ** 2).sum())
            assert abs(oracle.sqnorm(gw) - nx * ny) <= 1e-12 * nx * ny
            assert abs(oracle.sqnorm(gb) - ny) <= 1e-12 * ny
        # autograd through a library linear layer
        w = torch.zeros(4, 7, dtype=torch.float64, requires_grad=True)
        b = torch.zeros(4, dtype=torch.float64, requires_grad=True)
        (F.linear(torch.from_numpy(x[i]).double(), w, b) * torch.from_numpy(dy[i]).double()).sum().backward()
        assert np.allclose(gw, w.grad.numpy(), rtol=1e-13, atol=1e-13)
        assert np.allclose(gb, b.grad.numpy(), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("c,hw,groups", [(8, 5, 4), (6, 4, 1), (6, 3, 6), (16, 8, 8)])
def test_groupnorm_affine_gradient(c, hw, groups):
    """y = gamma * xhat + beta is linear in (gamma, beta): finite differences through the
    library group_norm are exact; autograd agrees."""
    l = gn_affine(c, hw, groups)
    x, dy = _rand(l, 2, 61)
    x = x * 1.7 + 0.3
    for i in range(2):
        gg, gb = oracle.example_grad(l, x[i], dy[i])
        xt = torch.from_numpy(x[i:i + 1]).double()
        dyt = torch.from_numpy(dy[i:i + 1]).double()

        def loss(gamma, beta):
            return float((dyt * F.group_norm(xt, groups, gamma, beta, eps=l.gn_eps)).sum())

        g0 = torch.ones(c, dtype=torch.float64)
        b0 = torch.zeros(c, dtype=torch.float64)
        for e in range(c):
            d = torch.zeros(c, dtype=torch.float64)
            d[e] = 1.0
            assert abs((loss(g0 + d, b0) - loss(g0 - d, b0)) / 2 - gg[e]) <= 1e-10 * max(1, abs(gg[e]))
            assert abs((loss(g0, b0 + d) - loss(g0, b0 - d)) / 2 - gb[e]) <= 1e-10 * max(1, abs(gb[e]))
        gam = torch.ones(c, dtype=torch.float64, requires_grad=True)
        bet = torch.zeros(c, dtype=torch.float64, requires_grad=True)
        (dyt * F.group_norm(xt, groups, gam, bet, eps=l.gn_eps)).sum().backward()
        assert np.allclose(gg, gam.grad.numpy(), rtol=1e-10, atol=1e-12)
        assert np.allclose(gb, bet.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_groupnorm_uses_biased_variance_and_eps():
    l = gn_affine(4, 2, 2)
    x, dy = _rand(l, 1, 67)
    gg, _ = oracle.example_grad(l, x[0], dy[0])
    xs = x[0].astype(np.float64).reshape(2, -1)
    mean = xs.mean(1, keepdims=True)
    var = ((xs - mean) ** 2).mean(1, keepdims=True)          # divide by count, not count-1
    xhat = ((xs - mean) / np.sqrt(var + 1e-5)).reshape(4, -1)
    assert np.allclose(gg, (dy[0].astype(np.float64).reshape(4, -1) * xhat).sum(1), rtol=1e-13)


def test_single_element_entry_points_agree_with_full_gradient():
    for l in (CONVS[1], CONVS[4], dense(5, 3, tokens=2), gn_affine(8, 3, 2)):
        x, dy = _rand(l, 1, 71)
        gw, gb = oracle.example_grad(l, x[0], dy[0])
        for e in range(l.pw):
            assert oracle.grad_elem(l, x[0], dy[0], e) == gw.reshape(-1)[e]
        for e in range(l.pb):
            assert oracle.grad_elem(l, x[0], dy[0], e, bias=True) == gb[e]


def test_weighted_sum_elements_match_full_route():
    l = CONVS[0]
    n = 6
    x, dy = _rand(l, n, 73)
    f = np.random.default_rng(1).uniform(0.1, 1.0, n)
    full_w = sum(f[i] * oracle.example_grad(l, x[i], dy[i])[0] for i in range(n)).reshape(-1)
    full_b = sum(f[i] * oracle.example_grad(l, x[i], dy[i])[1] for i in range(n))
    idx = np.array([0, 5, 17, l.pw - 1])
    assert np.allclose(oracle.weighted_sum_elems(l, x, dy, f, idx), full_w[idx], rtol=1e-14)
    assert np.allclose(oracle.weighted_sum_elems(l, x, dy, f, np.arange(l.pb), bias=True), full_b, rtol=1e-14)
