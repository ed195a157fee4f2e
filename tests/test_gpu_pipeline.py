"""GPU parity of the whole path (all five steps through the C ABI) against the fp64 oracle,
on the five workloads -- full size where the oracle finishes in seconds, otherwise the same
layer structure on smaller feature maps / fewer examples."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2109_12191_amd as dp
from gpu_util import BF16_TOL, F32_TOL, assert_close, dev, host
from workloads import get_workload, make_inputs

pytestmark = pytest.mark.gpu


def _run_both(wl, mode):
    steps = [make_inputs(wl, m) for m in range(wl.accum)]
    ref = oracle.privatise(wl, steps)
    ps = dp.PrivatiseStep(wl, mode=mode)
    ps.begin_step()
    n2_gpu = []
    for inputs in steps:
        ps.micro_step([(dev(x, wl.dtype), dev(dy, wl.dtype)) for x, dy in inputs])
        n2_gpu.append(host(ps.group_sqnorm).T.copy())          # [n, G]
    acc_gpu = ps.acc.clone()
    ps.finalize()
    torch.cuda.synchronize()
    return ref, ps, n2_gpu, acc_gpu


def _check(wl, mode):
    tol = F32_TOL if wl.dtype == "f32" else BF16_TOL
    ref, ps, n2_gpu, acc_gpu = _run_both(wl, mode)
    # H2: squared norms per example and group
    for m in range(wl.accum):
        assert np.allclose(n2_gpu[m], ref["n2"][m], rtol=tol, atol=0), f"n2 micro-step {m}"
    # H4: clipped sum before noise, tensor by tensor
    for li, l in enumerate(wl.layers):
        a = host(acc_gpu[ps.off_w[li]: ps.off_w[li] + ps.pw[li]])
        assert_close(a, ref["acc_w"][li], tol, f"acc_w[{li}] {l.name} ({ps.form[li]})")
        if l.pb:
            b = host(acc_gpu[ps.off_b[li]: ps.off_b[li] + ps.pb[li]])
            assert_close(b, ref["acc_b"][li], tol, f"acc_b[{li}] {l.name}")
    # H5: final output
    for li, l in enumerate(wl.layers):
        assert_close(host(ps.out_w(li)), ref["out_w"][li], tol, f"out_w[{li}] {l.name}")
        if l.pb:
            assert_close(host(ps.out_b(li)), ref["out_b"][li], tol, f"out_b[{li}] {l.name}")
    return ps


@pytest.mark.parametrize("mode", ["auto", "materialise", "recompute"])
def test_mlp_workload_full_size(mode):
    _check(get_workload("mlp"), mode)


@pytest.mark.parametrize("mode", ["auto", "recompute"])
def test_conv3x3_workload_full_size(mode):
    _check(get_workload("conv3x3"), mode)


@pytest.mark.parametrize("mode", ["auto", "recompute"])
def test_resnet20_workload(mode):
    # config 3 at full size: 39 layers, 256 examples
    _check(get_workload("resnet20"), mode)


@pytest.mark.parametrize("mode", ["auto", "materialise", "recompute"])
def test_resnet50_layer_set_small_maps(mode):
    # all 54 layers with their real channel counts, 64x64 input instead of 224x224
    ps = _check(get_workload("resnet50", n=4, accum=2, hw=64), mode)
    if mode == "auto":
        assert "materialise" in ps.form or "recompute" in ps.form


def test_resnet50_nano_per_layer_clipping_small_maps():
    wl = get_workload("resnet50_nano", accum=4, hw=64)
    assert wl.n == 1 and wl.n_groups == 54
    _check(wl, "auto")


def test_split_and_resume_gives_same_bits():
    """State between micro-steps is only the accumulator: copy it out and in mid-step."""
    wl = get_workload("conv3x3", n=4, accum=3, hw=14)
    steps = [[(dev(x), dev(dy)) for x, dy in make_inputs(wl, m)] for m in range(3)]
    a = dp.PrivatiseStep(wl)
    a.run(steps)
    b = dp.PrivatiseStep(wl)
    b.begin_step()
    b.micro_step(steps[0])
    saved = b.acc.clone()
    c = dp.PrivatiseStep(wl)
    c.begin_step()
    c.acc.copy_(saved)
    c.micro_step(steps[1])
    c.micro_step(steps[2])
    c.finalize()
    torch.cuda.synchronize()
    assert torch.equal(a.out, c.out)


def test_graph_replay_with_side_streams_matches_eager_every_time():
    """The whole step recorded into a HIP graph (layers spread over side streams) gives the same bits as the
    call-by-call path at the same optimiser step, on every replay, with eager work in between; consecutive
    steps draw different noise (the step counter is a device word that the graph itself advances)."""
    wl = get_workload("resnet50", n=4, accum=2, hw=64)
    steps = [[(dev(x, wl.dtype), dev(dy, wl.dtype)) for x, dy in make_inputs(wl, m)] for m in range(wl.accum)]
    eager = dp.PrivatiseStep(wl, streams=1)
    want = []
    for k in range(3):
        assert eager.step == k
        want.append(eager.run(steps).clone())
    torch.cuda.synchronize()
    assert not torch.equal(want[0], want[1]) and not torch.equal(want[1], want[2])
    g = dp.PrivatiseStep(wl, streams=4)
    g.capture(steps)
    assert g.step == 0
    for rep in range(3):
        g.out.zero_()
        g.acc.fill_(123.0)                 # the graph must clear the accumulator itself
        torch.cuda.synchronize()
        got = g.replay()
        torch.cuda.synchronize()
        assert torch.equal(got, want[rep]), f"replay {rep}"
        eager.set_step(rep)                # eager work between replays
        again = eager.run(steps)
        torch.cuda.synchronize()
        assert torch.equal(again, want[rep])
    assert g.step == 3 and int(g._step_dev.item()) == 3
    # multi-stream without a graph as well
    ms = dp.PrivatiseStep(wl, streams=3)
    assert torch.equal(ms.run(steps), want[0])


def test_consecutive_optimiser_steps_draw_fresh_noise_and_match_the_oracle():
    """Two optimiser steps in a row on the same data: the released gradients carry different noise, and each
    matches the oracle evaluated at its own step number (eager and graph replay)."""
    from dataclasses import replace
    wl = get_workload("conv3x3", n=4, accum=2, hw=14)
    host_steps = [make_inputs(wl, m) for m in range(wl.accum)]
    refs = [oracle.privatise(replace(wl, step=wl.step + k), host_steps) for k in range(2)]
    steps = [[(dev(x), dev(dy)) for x, dy in inputs] for inputs in host_steps]
    for use_graph in (False, True):
        ps = dp.PrivatiseStep(wl, streams=2 if use_graph else 1)
        if use_graph:
            ps.capture(steps)
        outs = []
        for k in range(2):
            out = ps.replay() if use_graph else ps.run(steps)
            torch.cuda.synchronize()
            outs.append(out.clone())
            for li, l in enumerate(wl.layers):
                assert_close(host(ps.out_w(li)), refs[k]["out_w"][li], F32_TOL, f"graph={use_graph} step {k} out_w")
                assert_close(host(ps.out_b(li)), refs[k]["out_b"][li], F32_TOL, f"graph={use_graph} step {k} out_b")
        diff = host(outs[1] - outs[0])[: ps.pw[0]]
        # the clipped sums cancel; what is left is the difference of two independent noise draws
        sigma_c_over_b = wl.sigma * wl.clip_c / wl.total_batch
        assert abs(diff.std() / (math.sqrt(2.0) * sigma_c_over_b) - 1.0) < 0.05


def test_fused_optimiser_update_over_two_steps():
    """finalize with the SGD step fused in: theta after two optimiser steps (momentum carried) against the
    oracle's finalize + update."""
    wl = get_workload("conv3x3", n=4, accum=2, hw=14)
    steps = [[(dev(x), dev(dy)) for x, dy in make_inputs(wl, m)] for m in range(wl.accum)]
    ref = oracle.privatise(wl, [make_inputs(wl, m) for m in range(wl.accum)])
    ps = dp.PrivatiseStep(wl, streams=2)
    rng = np.random.default_rng(23)
    theta0 = rng.standard_normal(ps.p_total).astype(np.float32)
    ps.enable_update(lr=0.05, momentum=0.9, theta=dev(theta0))
    from dataclasses import replace
    ref1 = oracle.privatise(replace(wl, step=wl.step + 1), [make_inputs(wl, m) for m in range(wl.accum)])
    ps.run(steps)
    ps.set_lr(0.025)
    ps.run(steps)                                    # same data, next optimiser step: fresh noise
    torch.cuda.synchronize()
    for li, l in enumerate(wl.layers):
        for off, cnt, g, g1 in ((ps.off_w[li], ps.pw[li], ref["out_w"][li], ref1["out_w"][li]),
                                (ps.off_b[li], ps.pb[li], ref["out_b"][li], ref1["out_b"][li])):
            if not cnt:
                continue
            th, v = theta0[off: off + cnt].astype(np.float64), np.zeros(cnt)
            th, v = oracle.sgd_update(g.reshape(-1), th, v, 0.05, 0.9)
            th, v = oracle.sgd_update(g1.reshape(-1), th, v, 0.025, 0.9)
            assert_close(host(ps.theta[off: off + cnt]), th, F32_TOL, f"theta layer {li}")
            assert_close(host(ps.out[off: off + cnt]), g1.reshape(-1), F32_TOL, f"gradient layer {li}")


@pytest.mark.parametrize("streams", [1, 3])
def test_per_example_noise_form_whole_path(streams):
    """The paper's as-built form: noise per clipped example, nothing added in finalize."""
    wl = get_workload("resnet50", n=4, accum=2, hw=64)
    host_steps = [make_inputs(wl, m) for m in range(wl.accum)]
    ref = oracle.privatise(wl, host_steps, noise_form="per_example")
    steps = [[(dev(x, wl.dtype), dev(dy, wl.dtype)) for x, dy in inputs] for inputs in host_steps]
    ps = dp.PrivatiseStep(wl, streams=streams, noise="per_example")
    ps.run(steps)
    torch.cuda.synchronize()
    for li, l in enumerate(wl.layers):
        assert_close(host(ps.out_w(li)), ref["out_w"][li], BF16_TOL, f"out_w[{li}] {l.name}")
        if l.pb:
            assert_close(host(ps.out_b(li)), ref["out_b"][li], BF16_TOL, f"out_b[{li}]")


@pytest.mark.parametrize("name,n,accum,hw", [("resnet18_gn", 3, 2, 16), ("resnet50_gn", 2, 1, 64), ("resnet101_gn", 2, 1, 32)])
def test_further_layer_sets_with_groupnorm(name, n, accum, hw):
    """The paper's other networks (ResNet-18-GN, ResNet-101-GN32) and ResNet-50 with its GroupNorm gradients:
    same kernels, more shapes; whole path against the oracle on small maps."""
    wl = get_workload(name, n=n, accum=accum, hw=hw)
    assert any(l.kind == "gn" for l in wl.layers)
    _check(wl, "auto")


def test_both_clip_branches_zero_example_and_infinite_bound():
    """The five workloads clip every example; here the bound is the median norm (half the examples keep their
    gradient), one example is all zeros (factor 1, contributes nothing), and a second run has C = inf, sigma = 0
    (the result is the plain mean gradient)."""
    import math
    from dataclasses import replace
    base = get_workload("resnet50", n=6, accum=2, hw=64)
    host_steps = [make_inputs(base, m) for m in range(base.accum)]
    for li in range(len(base.layers)):                     # example 3 of micro-step 0: all-zero gradient
        host_steps[0][li][1][3] = 0.0
    probe = oracle.privatise(base, host_steps)
    med = float(np.sqrt(np.median(np.concatenate([n2[:, 0] for n2 in probe["n2"]]))))
    for wl in (replace(base, clip_c=med), replace(base, clip_c=math.inf, sigma=0.0)):
        ref = oracle.privatise(wl, host_steps)
        f_all = np.concatenate([f[:, 0] for f in ref["f"]])
        if math.isfinite(wl.clip_c):
            assert (f_all < 1).sum() >= 4 and (f_all == 1).sum() >= 4          # both branches are taken
        steps = [[(dev(x, wl.dtype), dev(dy, wl.dtype)) for x, dy in inputs] for inputs in host_steps]
        for mode in ("auto", "recompute"):
            ps = dp.PrivatiseStep(wl, mode=mode, streams=2)
            ps.begin_step()
            ps.micro_step(steps[0])
            torch.cuda.synchronize()
            assert host(ps.group_sqnorm)[0, 3] == 0.0                           # the zero example
            ps.micro_step(steps[1])
            ps.finalize()
            torch.cuda.synchronize()
            for li, l in enumerate(wl.layers):
                assert_close(host(ps.out_w(li)), ref["out_w"][li], BF16_TOL, f"{mode} C={wl.clip_c} out_w[{li}] {l.name}")
