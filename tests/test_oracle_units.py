"""Pins for the oracle's clipping-unit variant (the micro-batching of the GPU baseline, Abstract and Table 1:
the gradient of a micro-batch of examples is clipped instead of the gradient of each example)."""
import math

import numpy as np
import torch
import torch.nn.functional as F

import oracle
from workloads import conv, dense, gn_affine, make_inputs
from workloads.configs import Workload

torch.set_num_threads(4)


def _net():
    return (conv(3, 4, 3, 1, 6, bias=True, name="c0"), gn_affine(4, 6, 2, name="g0"),
            conv(4, 6, 3, 2, 6, name="c1"), conv(6, 5, 1, 1, 3, name="c2"), dense(5, 3, name="fc"))


def _wl(clip_mode="global", clip_c=1.0, sigma=0.0, n=8, accum=1, dy_std=0.05, layers=None):
    layers = layers or _net()
    return Workload("small", layers, n, accum, "f32", clip_mode, clip_c, sigma,
                    tuple("normal" for _ in layers), dy_std, 777)


def _flat(acc_w, acc_b):
    return np.concatenate([np.concatenate([w.reshape(-1), b if b is not None else np.zeros(0)])
                           for w, b in zip(acc_w, acc_b)])


def _run_units(wl, inputs, unit, clip_c=None):
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    bounds = oracle.group_bounds(wl.clip_c if clip_c is None else clip_c, wl.n_groups)[0]
    n2, f = oracle.clip_accumulate_units(wl.layers, inputs, unit, wl.group_of_layer, bounds, acc_w, acc_b)
    return _flat(acc_w, acc_b), n2, f


def test_worked_scalar_example():
    """One weight, two examples: g_1 = 1*3 = 3, g_2 = 2*5 = 10.  Per-example clipping to C = 1 gives 1 + 1 = 2;
    one unit of two clips their mean 6.5 to 1; with C = 8 the mean passes unclipped."""
    l = dense(1, 1, bias=False, name="w")
    x = np.array([[[1.0]], [[2.0]]], dtype=np.float32)
    dy = np.array([[[3.0]], [[5.0]]], dtype=np.float32)
    for unit, c, want, n2_want in ((1, 1.0, 2.0, None), (2, 1.0, 1.0, 42.25), (2, 8.0, 6.5, 42.25)):
        acc_w, acc_b = oracle.new_accumulators([l])
        n2, f = oracle.clip_accumulate_units([l], [(x, dy)], unit, [0], [c], acc_w, acc_b)
        assert abs(acc_w[0].reshape(-1)[0] - want) < 1e-12
        if n2_want is not None:
            assert n2.shape == (1, 1) and abs(n2[0, 0] - n2_want) < 1e-12


def test_unit_of_one_is_per_example_clipping():
    for mode in ("global", "per_layer"):
        wl = _wl(clip_mode=mode, clip_c=0.3)
        inputs = make_inputs(wl, 0)
        got, n2, f = _run_units(wl, inputs, 1)
        acc_w, acc_b = oracle.new_accumulators(wl.layers)
        n2r, fr = oracle.clip_accumulate(wl.layers, inputs, wl.group_of_layer,
                                        oracle.group_bounds(wl.clip_c, wl.n_groups)[0], acc_w, acc_b)
        # the threads' private sums meet in a different order: the last bits of the sum may differ
        assert np.allclose(got, _flat(acc_w, acc_b), rtol=1e-13, atol=1e-18)
        assert np.array_equal(n2, n2r) and np.array_equal(f, fr) and (f < 1).any()


def test_unit_mean_is_the_gradient_of_the_units_mean_loss():
    """Library autograd: the gradient of (1/unit) sum of the unit's losses, whose output gradients are dy."""
    unit = 4
    l = conv(3, 5, 3, 2, 7, bias=True, name="c")
    wl = _wl(n=8, layers=(l,))
    (x, dy), = make_inputs(wl, 3)
    gw, gb = oracle.unit_mean_grad(l, x, dy, unit)
    for u in range(2):
        w = torch.zeros(l.w_shape, dtype=torch.float64, requires_grad=True)
        b = torch.zeros(l.cout, dtype=torch.float64, requires_grad=True)
        xs = torch.from_numpy(x[u * unit:(u + 1) * unit]).double()
        y = F.conv2d(xs, w, b, stride=l.stride, padding=l.pad)
        ((y * torch.from_numpy(dy[u * unit:(u + 1) * unit]).double()).sum() / unit).backward()
        assert np.allclose(gw[u], w.grad.numpy().reshape(-1), rtol=1e-12, atol=1e-15)
        assert np.allclose(gb[u], b.grad.numpy(), rtol=1e-12, atol=1e-15)


def test_norms_factors_and_sum_from_the_unit_means():
    """n2, f and the clipped sum rebuilt with numpy from unit_mean_grad (itself pinned by autograd above)."""
    for mode, unit in (("global", 2), ("per_layer", 4)):
        wl = _wl(clip_mode=mode, clip_c=0.05, n=8)
        inputs = make_inputs(wl, 1)
        got, n2, f = _run_units(wl, inputs, unit)
        bounds = oracle.group_bounds(wl.clip_c, wl.n_groups)[0]
        means = [oracle.unit_mean_grad(l, x, dy, unit) for l, (x, dy) in zip(wl.layers, inputs)]
        want = [np.zeros(l.pw + l.pb) for l in wl.layers]
        for u in range(wl.n // unit):
            rows = [np.concatenate([mw[u], mb[u] if mb is not None else np.zeros(0)]) for mw, mb in means]
            for g in range(wl.n_groups):
                members = [k for k in range(len(rows)) if wl.group_of_layer[k] == g]
                norm2 = sum(float(np.dot(rows[k], rows[k])) for k in members)
                fac = min(1.0, bounds[g] / math.sqrt(norm2))
                assert abs(n2[u, g] - norm2) <= 1e-12 * norm2 and abs(f[u, g] - fac) <= 1e-12
                for k in members:
                    want[k] += fac * rows[k]
        assert np.allclose(got, np.concatenate(want), rtol=1e-11, atol=1e-16)
        assert (f < 1).any()


def test_sum_form_identity_through_the_token_axis():
    """sum_u clip(mean_u, C) = 1/unit * sum_u clip(sum_u, unit*C).  For a dense layer the SUM of the gradients of
    `unit` one-token examples is the per-example gradient of one example holding those tokens, so the right-hand
    side is the per-example oracle on reshaped inputs with the bound unit*C."""
    unit, units = 4, 5
    one = dense(6, 3, name="fc")                      # one token per example
    many = dense(6, 3, tokens=unit, name="fc")
    rng = np.random.default_rng(8)
    x = rng.standard_normal((unit * units, 1, 6)).astype(np.float32)
    dy = (rng.standard_normal((unit * units, 1, 3)) * 0.3).astype(np.float32)
    for c in (0.05, 0.4, 100.0):
        acc_w, acc_b = oracle.new_accumulators([one])
        _, f = oracle.clip_accumulate_units([one], [(x, dy)], unit, [0], [c], acc_w, acc_b)
        ref_w, ref_b = oracle.new_accumulators([many])
        _, fr = oracle.clip_accumulate([many], [(x.reshape(units, unit, 6), dy.reshape(units, unit, 3))], [0], [unit * c],
                                       ref_w, ref_b)
        assert np.allclose(acc_w[0], ref_w[0] / unit, rtol=1e-12, atol=1e-18)
        assert np.allclose(acc_b[0], ref_b[0] / unit, rtol=1e-12, atol=1e-18)
        assert np.allclose(f, fr, rtol=1e-12)


def test_every_clipped_unit_is_within_bound_and_identical_examples_reduce_to_one():
    wl = _wl(clip_c=0.02, n=4)
    inputs = make_inputs(wl, 2)
    # a unit of four copies of example 0: its mean is that example's gradient
    rep = [(np.repeat(x[:1], 4, axis=0), np.repeat(dy[:1], 4, axis=0)) for x, dy in inputs]
    got, n2, f = _run_units(wl, rep, 4)
    single = [(x[:1], dy[:1]) for x, dy in inputs]
    ref, n2r, fr = _run_units(wl, single, 1)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-18) and np.allclose(n2, n2r, rtol=1e-12)
    assert f[0, 0] < 1 and abs(math.sqrt(float(np.dot(got, got))) - wl.clip_c) <= 1e-12


def test_whole_step_divides_by_the_number_of_units():
    """sigma = 0, infinite bound: the result is the mean over units of the unit means = the plain mean gradient."""
    wl = _wl(clip_c=math.inf, sigma=0.0, n=8, accum=2)
    steps = [make_inputs(wl, m) for m in range(wl.accum)]
    res = oracle.privatise_units(wl, steps, 4)
    plain = oracle.privatise(wl, steps)
    for a, b in zip(res["out_w"], plain["out_w"]):
        assert np.allclose(a, b, rtol=1e-12, atol=1e-18)
    # with noise: the noise term is sigma * C * z / (number of units), z the tensor's Philox normals
    wl2 = _wl(clip_c=0.5, sigma=1.3, n=8, accum=2)
    res2 = oracle.privatise_units(wl2, steps, 4)
    li = 2
    z = oracle.noise_normal(wl2.philox_seed, wl2.step, 2 * li, wl2.layers[li].pw)
    want = (res2["acc_w"][li].reshape(-1) + 1.3 * 0.5 * z) / 4.0
    assert np.allclose(res2["out_w"][li].reshape(-1), want, rtol=1e-12, atol=1e-18)
