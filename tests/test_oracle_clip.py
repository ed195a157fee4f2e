"""Pins for the oracle's clip / accumulate / finalize steps (Section 2, first equation;
Section 3.5 for per-group bounds)."""
import math
from dataclasses import replace

import numpy as np
import torch

import oracle
from workloads import Layer, conv, dense, get_workload, gn_affine, make_inputs
from workloads.configs import Workload

torch.set_num_threads(4)


def _small_net():
    return (conv(3, 4, 3, 1, 6, bias=True, name="c0"), gn_affine(4, 6, 2, name="g0"),
            conv(4, 6, 3, 2, 6, name="c1"), conv(6, 5, 1, 1, 3, name="c2"), dense(5, 3, name="fc"))


def _wl(clip_mode="global", clip_c=1.0, sigma=0.0, n=6, accum=1, dy_std=0.05):
    layers = _small_net()
    return Workload("small", layers, n, accum, "f32", clip_mode, clip_c, sigma,
                    tuple("normal" for _ in layers), dy_std, 4242)


def _per_example_grads(wl, inputs):
    """flat fp64 gradient per example per layer via the oracle's single-example entry."""
    out = []
    for i in range(inputs[0][0].shape[0]):
        row = []
        for l, (x, dy) in zip(wl.layers, inputs):
            gw, gb = oracle.example_grad(l, x[i], dy[i])
            row.append(np.concatenate([gw.reshape(-1), gb if gb is not None else np.zeros(0)]))
        out.append(row)
    return out


def test_every_clipped_example_is_within_bound():
    """spec check 2: ||clip(g_i)|| <= C within 1e-12, and exactly C when clipped."""
    for c in (0.05, 0.5, 50.0):
        wl = _wl(clip_c=c, n=1)
        for seed_step in range(8):
            inputs = make_inputs(wl, seed_step)
            acc_w, acc_b = oracle.new_accumulators(wl.layers)
            n2, f = oracle.clip_accumulate(wl.layers, inputs, wl.group_of_layer, oracle.group_bounds(wl.clip_c, wl.n_groups)[0], acc_w, acc_b)
            tot = sum(oracle.sqnorm(a) for a in acc_w) + sum(oracle.sqnorm(a) for a in acc_b if a is not None)
            assert math.sqrt(tot) <= c * (1 + 1e-12)
            if n2[0, 0] > c * c:
                assert abs(math.sqrt(tot) - c) <= 1e-12 * c and f[0, 0] < 1
            else:
                assert f[0, 0] == 1.0 and abs(tot - n2[0, 0]) <= 1e-12 * tot


def test_infinite_bound_and_zero_sigma_give_plain_mean_gradient():
    """spec check 3, against library batch gradients (one backward over the batch)."""
    wl = _wl(clip_c=math.inf, sigma=0.0, n=5, accum=2)
    steps = [make_inputs(wl, m) for m in range(wl.accum)]
    res = oracle.privatise(wl, steps)
    assert all(np.all(f == 1.0) for f in res["f"])
    for li, l in enumerate(wl.layers):
        x = torch.from_numpy(np.concatenate([s[li][0] for s in steps])).double()
        dy = torch.from_numpy(np.concatenate([s[li][1] for s in steps])).double()
        if l.kind == "conv":
            ref_w = torch.nn.grad.conv2d_weight(x, l.w_shape, dy, stride=l.stride, padding=l.pad)
            ref_b = dy.sum((0, 2, 3))
        elif l.kind == "dense":
            ref_w = torch.einsum("nto,ntk->ok", dy, x)
            ref_b = dy.sum((0, 1))
        else:
            gam = torch.ones(l.cin, dtype=torch.float64, requires_grad=True)
            bet = torch.zeros(l.cin, dtype=torch.float64, requires_grad=True)
            (dy * torch.nn.functional.group_norm(x, l.gn_groups, gam, bet, eps=l.gn_eps)).sum().backward()
            ref_w, ref_b = gam.grad, bet.grad
        assert np.allclose(res["out_w"][li].reshape(-1), ref_w.numpy().reshape(-1) / wl.total_batch,
                           rtol=1e-10, atol=1e-13)
        if l.pb:
            assert np.allclose(res["out_b"][li], ref_b.numpy() / wl.total_batch, rtol=1e-10, atol=1e-13)


def test_clip_factor_definition_both_branches_and_zero_gradient():
    assert oracle.clip_factor(0.0, 1.0) == 1.0
    assert oracle.clip_factor(4.0, 1.0) == 0.5
    assert oracle.clip_factor(0.25, 1.0) == 1.0
    assert oracle.clip_factor(1e30, math.inf) == 1.0
    # norms straddling the bound: C = median norm
    wl = _wl(n=9)
    inputs = make_inputs(wl, 0)
    inputs[0][0][3] = 0.0            # an all-zero example: every layer's input and dy are zero
    for li in range(len(inputs)):
        inputs[li][0][3] = 0.0
        inputs[li][1][3] = 0.0
    grads = _per_example_grads(wl, inputs)
    norms = np.array([math.sqrt(sum(float(g @ g) for g in row)) for row in grads])
    c = float(np.median(norms[norms > 0]))
    wl = replace(wl, clip_c=c)
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    n2, f = oracle.clip_accumulate(wl.layers, inputs, wl.group_of_layer, oracle.group_bounds(wl.clip_c, wl.n_groups)[0], acc_w, acc_b)
    assert np.allclose(np.sqrt(n2[:, 0]), norms, rtol=1e-13)
    assert f[3, 0] == 1.0 and n2[3, 0] == 0.0
    assert (f[:, 0] < 1).sum() >= 3 and (f[:, 0] == 1).sum() >= 3
    want = np.minimum(1.0, c / np.where(norms > 0, norms, 1.0))
    assert np.allclose(f[:, 0], want, rtol=1e-13)
    # the accumulated sum is sum_i f_i g_i, tensor by tensor
    for li, l in enumerate(wl.layers):
        ref = sum(f[i, 0] * grads[i][li] for i in range(9))
        got = np.concatenate([acc_w[li], acc_b[li] if acc_b[li] is not None else np.zeros(0)])
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-15)
    assert all(np.isfinite(a).all() for a in acc_w)


def test_per_group_clipping_respects_the_overall_bound():
    """Section 3.5: M groups each clipped to C/sqrt(M) => sum_g ||clip(g^g)||^2 <= C^2."""
    wl = _wl(clip_mode="per_layer", clip_c=0.3, n=4)
    m = len(wl.layers)
    bounds, total = oracle.group_bounds(0.3, m)
    assert wl.n_groups == m and len(bounds) == m and all(abs(c - 0.3 / math.sqrt(m)) < 1e-15 for c in bounds)
    assert abs(total - 0.3) < 1e-15                      # the noise is scaled by the overall bound C, not by C_g
    assert oracle.group_bounds(1.7, 1) == ([1.7], 1.7)   # one group: the global bound of Section 2
    inputs = make_inputs(wl, 0)
    grads = _per_example_grads(wl, inputs)
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    n2, f = oracle.clip_accumulate(wl.layers, inputs, wl.group_of_layer, oracle.group_bounds(wl.clip_c, wl.n_groups)[0], acc_w, acc_b)
    for i in range(4):
        tot = 0.0
        for g in range(m):
            assert abs(n2[i, g] - float(grads[i][g] @ grads[i][g])) <= 1e-12 * n2[i, g]
            clipped = f[i, g] ** 2 * n2[i, g]
            assert clipped <= (0.3 / math.sqrt(m)) ** 2 * (1 + 1e-12)
            tot += clipped
        assert tot <= 0.3 ** 2 * (1 + 1e-12)


def test_accumulation_is_linear_permutation_invariant_and_resumable():
    wl = _wl(clip_c=0.2, n=4, accum=3)
    steps = [make_inputs(wl, m) for m in range(3)]
    a = oracle.privatise(wl, steps)
    # one micro-step of 12 examples
    merged = [(np.concatenate([s[li][0] for s in steps]), np.concatenate([s[li][1] for s in steps]))
              for li in range(len(wl.layers))]
    b = oracle.privatise(replace(wl, n=12, accum=1), [merged])
    # permuted examples
    perm = np.random.default_rng(0).permutation(12)
    c = oracle.privatise(replace(wl, n=12, accum=1), [[(x[perm], dy[perm]) for x, dy in merged]])
    for li in range(len(wl.layers)):
        assert np.allclose(a["acc_w"][li], b["acc_w"][li], rtol=1e-12, atol=1e-15)
        assert np.allclose(a["acc_w"][li], c["acc_w"][li], rtol=1e-12, atol=1e-15)
    # stop after one micro-step, copy the accumulator out and in, continue: same result
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    oracle.clip_accumulate(wl.layers, steps[0], wl.group_of_layer, oracle.group_bounds(wl.clip_c, wl.n_groups)[0], acc_w, acc_b)
    saved_w = [x.copy() for x in acc_w]
    saved_b = [None if x is None else x.copy() for x in acc_b]
    for m in (1, 2):
        oracle.clip_accumulate(wl.layers, steps[m], wl.group_of_layer, oracle.group_bounds(wl.clip_c, wl.n_groups)[0], saved_w, saved_b)
    for li in range(len(wl.layers)):
        assert np.allclose(saved_w[li], a["acc_w"][li], rtol=1e-13, atol=1e-16)
    # threads do not change the result beyond round-off
    one = oracle.privatise(wl, steps, threads=1)
    for li in range(len(wl.layers)):
        assert np.allclose(one["acc_w"][li], a["acc_w"][li], rtol=1e-13, atol=1e-16)
        assert np.array_equal(one["n2"][0], a["n2"][0])


def test_output_is_clipped_sum_plus_scaled_noise_over_batch():
    wl = _wl(clip_mode="per_layer", clip_c=0.5, sigma=1.3, n=3, accum=2)
    steps = [make_inputs(wl, m) for m in range(2)]
    res = oracle.privatise(wl, steps)
    for li, l in enumerate(wl.layers):
        z = oracle.noise_normal(wl.philox_seed, wl.step, 2 * li, l.pw)
        want = (res["acc_w"][li] + wl.sigma * wl.clip_c * z) / wl.total_batch
        assert np.allclose(res["out_w"][li], want, rtol=1e-14, atol=1e-16)
        if l.pb:
            zb = oracle.noise_normal(wl.philox_seed, wl.step, 2 * li + 1, l.pb)
            assert np.allclose(res["out_b"][li], (res["acc_b"][li] + wl.sigma * wl.clip_c * zb) / 6,
                               rtol=1e-14, atol=1e-16)


def test_expected_norm_of_the_conv3x3_workload():
    """Sanity of scale: E||g_i||^2 = var(dy) * (Cout*Cin*valid_taps + Cout*S) for iid inputs."""
    wl = get_workload("conv3x3", n=4, accum=1, hw=14)
    inputs = make_inputs(wl, 0)
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    n2, _ = oracle.clip_accumulate(wl.layers, inputs, wl.group_of_layer, oracle.group_bounds(wl.clip_c, wl.n_groups)[0], acc_w, acc_b)
    valid = sum((14 - abs(kh - 1)) * (14 - abs(kw - 1)) for kh in range(3) for kw in range(3))
    expect = 1e-4 * (64 * 64 * valid + 64 * 196)
    assert np.all(np.abs(n2[:, 0] / expect - 1) < 0.1)


def test_mlp_workload_matches_rank_one_closed_form():
    wl = get_workload("mlp")
    inputs = make_inputs(wl, 0)
    res = oracle.privatise(wl, [inputs])
    n2 = np.zeros(wl.n)
    for x, dy in inputs:
        x64, dy64 = x.astype(np.float64).reshape(wl.n, -1), dy.astype(np.float64).reshape(wl.n, -1)
        n2 += (dy64 ** 2).sum(1) * ((x64 ** 2).sum(1) + 1.0)      # weight + bias
    assert np.allclose(res["n2"][0][:, 0], n2, rtol=1e-12)
    f = np.minimum(1.0, wl.clip_c / np.sqrt(n2))
    x, dy = inputs[0]
    ref = np.einsum("n,no,nk->ok", f, dy.astype(np.float64).reshape(wl.n, -1), x.astype(np.float64).reshape(wl.n, -1))
    assert np.allclose(res["acc_w"][0].reshape(256, 784), ref, rtol=1e-11, atol=1e-15)
