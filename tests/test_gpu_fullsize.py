"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(HIP graph, side streams, per-layer choice of the clipped-sum form).

Config 4 (ResNet-50 layer set, 224x224, micro-batch 32 x 8 accumulation): the WHOLE optimiser step, all 256
examples, every element of every tensor of the clipped sum, the norms of every example, and the released
gradient.  Config 5 (micro-batch 1, 54 clipping groups): 36 micro-steps, so both buffer copies wrap many times.
The oracle needs about 8 GFLOP of plain fp64 loops per example: about 10 s per 32 examples on 16 host cores."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_12191_amd as dp
from gpu_util import BF16_TOL, assert_close, host, progress
from workloads import get_workload
from workloads.device import make_device_inputs

pytestmark = pytest.mark.gpu


def _host_inputs(dev_inputs):
    return [(x.float().cpu().numpy(), dy.float().cpu().numpy()) for x, dy in dev_inputs]


def _compare(wl, ps, ref_acc_w, ref_acc_b, what):
    worst = 0.0
    for li, l in enumerate(wl.layers):
        a = host(ps.acc_w(li))
        l2, mx = assert_close(a, ref_acc_w[li], BF16_TOL, f"{what} acc_w[{li}] {l.name} ({ps.form[li]})")
        worst = max(worst, l2, mx)
        if l.pb:
            assert_close(host(ps.acc_b(li)), ref_acc_b[li], BF16_TOL, f"{what} acc_b[{li}] {l.name}")
    return worst


@pytest.mark.timeout(900)
def test_resnet50_full_size_whole_step_every_element():
    wl = get_workload("resnet50")                     # config 4: micro-batch 32, 8 micro-steps, 256 examples
    assert wl.n == 32 and wl.accum == 8
    progress(f"[fullsize] {wl.name}: n={wl.n} x {wl.accum}, {wl.n_params} parameters, drawing inputs")
    steps = make_device_inputs(wl, wl.accum, torch.device("cuda:0"))
    ps = dp.PrivatiseStep(wl, mode="auto", streams=8)
    ps.capture(steps)
    ps.replay()
    torch.cuda.synchronize()
    # the two buffer copies still hold the norms of the last two micro-steps
    n2_gpu = {6: host(ps._group_sqnorm[0])[0].copy(), 7: host(ps._group_sqnorm[1])[0].copy()}
    group_clip, clip_total = oracle.group_bounds(wl.clip_c, wl.n_groups)
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    for m in range(wl.accum):
        n2, f = oracle.clip_accumulate(wl.layers, _host_inputs(steps[m]), wl.group_of_layer, group_clip, acc_w, acc_b)
        progress(f"[fullsize] oracle micro-step {m} done")
        assert (f < 1).all()                           # every example is clipped in this workload
        if m in n2_gpu:
            assert np.allclose(n2_gpu[m], n2[:, 0], rtol=BF16_TOL, atol=0), (m, n2_gpu[m][:4], n2[:4, 0])
    worst = _compare(wl, ps, acc_w, acc_b, "config4")
    progress(f"[fullsize] worst relative error of the clipped sum over all tensors: {worst:.2e}")
    # H5 on the full parameter vector (part of the replayed graph): every tensor
    for li, l in enumerate(wl.layers):
        ref = oracle.noise_finalize(acc_w[li], wl.sigma, clip_total, wl.total_batch, wl.philox_seed, wl.step, 2 * li)
        assert_close(host(ps.out_w(li)), ref, BF16_TOL, f"out_w[{li}]")
    ref = oracle.noise_finalize(acc_b[53], wl.sigma, clip_total, wl.total_batch, wl.philox_seed, wl.step, 2 * 53 + 1)
    assert_close(host(ps.out_b(53)), ref, BF16_TOL, "out_b[53]")
    progress(f"[fullsize] forms: { {k: ps.form.count(k) for k in set(ps.form)} }")


@pytest.mark.timeout(600)
def test_resnet50_nano_full_size_36_micro_steps_every_element():
    accum = 36
    wl = get_workload("resnet50_nano", accum=accum)   # config 5 shapes: micro-batch 1, 54 clipping groups
    steps = make_device_inputs(wl, accum, torch.device("cuda:0"))
    ps = dp.PrivatiseStep(wl, mode="auto", streams=8)
    ps.capture(steps)
    ps.replay()
    torch.cuda.synchronize()
    progress(f"[fullsize] nano GPU done; oracle on {accum} examples")
    # every example is clipped on its own and per group, so the oracle may take the 36 one-example micro-steps
    # as one batch of 36 (linearity over micro-steps is one of the oracle's own pinned properties)
    stacked = [(torch.cat([steps[m][li][0] for m in range(accum)]).float().cpu().numpy(),
                torch.cat([steps[m][li][1] for m in range(accum)]).float().cpu().numpy()) for li in range(len(wl.layers))]
    group_clip, _ = oracle.group_bounds(wl.clip_c, wl.n_groups)
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    n2, f = oracle.clip_accumulate(wl.layers, stacked, wl.group_of_layer, group_clip, acc_w, acc_b)
    progress("[fullsize] nano oracle done")
    # the last two micro-steps' norms are still in the two buffer copies
    for m in (accum - 2, accum - 1):
        got = host(ps._group_sqnorm[m % 2])[:, 0]
        assert np.allclose(got, n2[m], rtol=BF16_TOL, atol=0), m
        # per-group bound on the GPU's own norms: the clipped squared group norms add up to at most C^2 (Section 3.5)
        fac = np.minimum(1.0, np.array(group_clip) / np.sqrt(got))
        assert (fac ** 2 * got).sum() <= wl.clip_c ** 2 * (1 + 1e-5)
    _compare(wl, ps, acc_w, acc_b, "config5")


def test_recompute_form_full_size_late_layers():
    """The weighted-recomputation form at full size on the late ResNet-50 layers, whatever the
    per-layer policy picks today: norms fed in are the oracle's."""
    wl = get_workload("resnet50", accum=1)
    picks = [i for i, l in enumerate(wl.layers) if l.name in ("s3b2.c2", "s4b1.c2", "s4b2.c1", "s4b1.down", "s3b1.c3")]
    dev_all = make_device_inputs(wl, 1, torch.device("cuda:0"))[0]
    rng = np.random.default_rng(5)
    n2 = (rng.uniform(0.4, 2.0, wl.n) ** 2).astype(np.float32)      # both clip branches
    fvec = np.array([oracle.clip_factor(float(v), 1.0) for v in n2])
    for li in picks:
        l = wl.layers[li]
        x, dy = dev_all[li]
        d = dp.make_desc(l, wl.n, "bf16")
        ws = torch.empty(max(16, dp.dp_workspace_bytes(d, dp.DP_WS_RECOMPUTE)), dtype=torch.uint8, device="cuda:0")
        acc = torch.zeros(l.pw, device="cuda:0")
        dp.dp_clip_accumulate_recompute(d, x, dy, torch.from_numpy(n2).cuda(), 1.0, acc, None, ws)
        idx = rng.choice(l.pw, size=4096, replace=False)
        ref = oracle.weighted_sum_elems(l, x.float().cpu().numpy(), dy.float().cpu().numpy(), fvec, idx)
        assert_close(host(acc)[idx], ref, BF16_TOL, f"recompute {l.name}")
