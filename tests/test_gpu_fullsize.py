"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(HIP graph, side streams, per-layer choice of the clipped-sum form).

The oracle needs about 8 GFLOP of plain fp64 loops per ResNet-50 example, so the comparison is
made on ONE micro-step of each ResNet-50 configuration (32 examples of config 4; two single-example
micro-steps of config 5), every output element of every tensor against the oracle.  The remaining
micro-steps run the same kernels on the same shapes; accumulation over micro-steps and the
reduced-size whole-step runs are covered in test_gpu_pipeline.py."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_12191_amd as dp
from gpu_util import BF16_TOL, assert_close, host
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


def test_resnet50_full_size_micro_step_every_element():
    wl = get_workload("resnet50", accum=1)            # config 4 shapes, one micro-step of 32 examples
    print(f"\n[fullsize] {wl.name}: n={wl.n}, {wl.n_params} parameters, drawing inputs", flush=True)
    steps = make_device_inputs(wl, 1, torch.device("cuda:0"))
    ps = dp.PrivatiseStep(wl, mode="auto", streams=8)
    ps.capture(steps)
    ps.replay()
    torch.cuda.synchronize()
    n2_gpu = host(ps.group_sqnorm)[0]
    print("[fullsize] GPU done; running the fp64 oracle on the same 32 examples", flush=True)
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    n2, f = oracle.clip_accumulate(wl.layers, _host_inputs(steps[0]), wl.group_of_layer, wl.group_clip, acc_w, acc_b)
    print("[fullsize] oracle done", flush=True)
    assert np.allclose(n2_gpu, n2[:, 0], rtol=BF16_TOL, atol=0), (n2_gpu[:4], n2[:4, 0])
    assert (f < 1).all()                               # every example is clipped in this workload
    worst = _compare(wl, ps, acc_w, acc_b, "config4")
    print(f"[fullsize] worst relative error over all tensors: {worst:.2e}", flush=True)
    # H5 on the full parameter vector: finalize is part of the replayed graph
    for li in (0, 20, 53):
        ref = oracle.noise_finalize(acc_w[li], wl.sigma, wl.clip_total, wl.total_batch, wl.philox_seed, wl.step, 2 * li)
        assert_close(host(ps.out_w(li)), ref, BF16_TOL, f"out_w[{li}]")
    # both forms were exercised unless the policy currently picks only one
    print("[fullsize] forms:", {k: ps.form.count(k) for k in set(ps.form)}, flush=True)


def test_resnet50_nano_full_size_two_micro_steps_every_element():
    wl = get_workload("resnet50_nano", accum=2)       # config 5 shapes: micro-batch 1, 54 clipping groups
    steps = make_device_inputs(wl, 2, torch.device("cuda:0"))
    ps = dp.PrivatiseStep(wl, mode="auto", streams=8)
    ps.capture(steps)
    ps.replay()
    torch.cuda.synchronize()
    print("\n[fullsize] nano GPU done; oracle on 2 examples", flush=True)
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    n2s = []
    for m in range(2):
        n2, f = oracle.clip_accumulate(wl.layers, _host_inputs(steps[m]), wl.group_of_layer, wl.group_clip, acc_w, acc_b)
        n2s.append(n2[0])
    # the last micro-step's norms are still in the buffers
    assert np.allclose(host(ps.group_sqnorm)[:, 0], n2s[1], rtol=BF16_TOL, atol=0)
    _compare(wl, ps, acc_w, acc_b, "config5")
    # per-group bound: sum over groups of the clipped squared norms stays below C^2 (Section 3.5)
    fac = np.minimum(1.0, np.array(wl.group_clip) / np.sqrt(n2s[1]))
    assert (fac ** 2 * n2s[1]).sum() <= wl.clip_c ** 2 * (1 + 1e-9)


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
