#!/usr/bin/env python3
"""Benchmark of the DPSGD gradient-privatisation hot path on one MI355X.

A "step" is one optimiser step of the whole path on the ResNet-50 layer set (config 4 of the
build's workloads): 8 micro-steps of 32 examples (per-example gradients + norms, clip factors,
clipped sum) followed by Philox noise + finalize on all 25.5 M parameters = 256 privatised
examples.  Inputs (bf16 activations and output gradients of all 54 layers, 8 distinct
micro-batches, about 11 GB) are synthetic, seeded, and resident in HBM before the timed region.

Prints ONE JSON line (see the keys below).  `roofline` describes the dominant kernel (the bf16
MFMA contraction variant with the most work against the chip's roofs per step), each launch timed with events on
the stream it runs on, lists every variant's figures under `variants`, and gives the whole step's algorithmic bytes
against the HBM roof under `whole_step`; `cpu_baseline` is the fp64 oracle timed on this machine's host cores on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK = {"bf16": 2.5e15, "f32": 157.3e12}     # dense MFMA peaks of MI355X, flop/s
HBM_PEAK = 8.0e12

# HBM bytes per launch of the contraction variants from the two rocprofv3 --pmc runs summarised in
# profiles/contraction_resnet50_hbm_traffic.txt: mean FETCH_SIZE and WRITE_SIZE per dispatch in KiB (a dispatch is one
# grouped launch: all layers of the variant in a micro-step), each scaled by what the same counter reads for plain
# streaming kernels of known size in the same runs (clip_accumulate_kernel and noise_finalize_flat_kernel, 16 bytes
# per lane like the contraction's loads: FETCH_SIZE reads half of their bytes, WRITE_SIZE all of them).
PMC_FETCH_SCALE, PMC_WRITE_SCALE = 2.0, 1.0
PMC_KIB_PER_LAUNCH = {          # variant -> (FETCH_SIZE, WRITE_SIZE)
    "conv_contract<bf16,256x256rows,per_example>": (105134.5, 491793.3),
    "conv_contract<bf16,128x128,per_example>": (194900.0, 98327.9),
    "conv_contract<bf16,64x64,per_example>": (201359.4, 12813.6),
    "conv_contract<bf16,128x128,weighted>": (137733.2, 37888.0),
}


def measured_traffic(variant):
    if variant not in PMC_KIB_PER_LAUNCH:
        return None
    f, w = PMC_KIB_PER_LAUNCH[variant]
    return 1024.0 * (f * PMC_FETCH_SCALE + w * PMC_WRITE_SCALE)


class Probe:
    """Asks the library to bracket every contraction kernel with a pair of events recorded on the
    stream the kernel is launched on (dp_profile_next_contraction): the elapsed time of a pair is
    that one kernel's duration, without the small kernels around it."""

    def __init__(self):
        self.pairs = {}     # variant -> list of (start, stop, flops, in_bytes)
        self.enabled = False

    def arm(self, variant, flops, nbytes, n_layers=1):
        import torch
        import paper_2109_12191_amd as dp
        if not self.enabled:
            return
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()          # creates the HIP handles; the library records both again
        b.record()
        self.pairs.setdefault(variant, []).append((a, b, flops, nbytes, n_layers))
        dp.dp_profile_next_contraction(a, b)

    def summary(self):
        out = {}
        for variant, lst in self.pairs.items():
            ms = sum(p[0].elapsed_time(p[1]) for p in lst)
            out[variant] = dict(launches=len(lst), total_ms=ms, flops=sum(p[2] for p in lst),
                                bytes=sum(p[3] for p in lst), layers=sum(p[4] for p in lst))
        return out


def cpu_baseline(wl, inputs0, budget_examples):
    """The oracle as it stands on the host cores, on the first `budget_examples` examples of
    micro-batch 0 (same bits the GPU got); examples/s scales linearly (examples are independent)."""
    import numpy as np
    import oracle
    cores = oracle.max_threads()
    s = min(budget_examples, wl.n)
    host_inputs = [(x[:s].float().cpu().numpy(), dy[:s].float().cpu().numpy()) for x, dy in inputs0]
    acc_w, acc_b = oracle.new_accumulators(wl.layers)
    t0 = time.perf_counter()
    oracle.clip_accumulate(wl.layers, host_inputs, wl.group_of_layer, oracle.group_bounds(wl.clip_c, wl.n_groups)[0], acc_w, acc_b, threads=cores)
    # noise + finalize on every parameter, once (amortised over the whole batch in `value`)
    t1 = time.perf_counter()
    p_sample = 0
    for li, l in enumerate(wl.layers):
        if li % 8 == 0:      # a bounded sample of tensors, scaled to all parameters below
            oracle.noise_finalize(acc_w[li], wl.sigma, oracle.group_bounds(wl.clip_c, wl.n_groups)[1], wl.total_batch, wl.philox_seed, wl.step, 2 * li)
            p_sample += l.pw
    t2 = time.perf_counter()
    per_example = (t1 - t0) / s
    finalize_all = (t2 - t1) * (wl.n_params / max(p_sample, 1))
    step_time = per_example * wl.total_batch + finalize_all
    return dict(value=wl.total_batch / step_time, unit="examples/s", cores=min(cores, s), kind="oracle",
                sample=f"{s} examples of micro-batch 0 through all {len(wl.layers)} layers "
                       f"({t1 - t0:.1f} s) + noise/finalize on {p_sample} of {wl.n_params} parameters "
                       f"({t2 - t1:.1f} s), scaled linearly to one step of {wl.total_batch} examples")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--mode", default="auto", choices=["auto", "materialise", "recompute"])
    ap.add_argument("--n", type=int, default=None, help="override examples per micro-step (tests)")
    ap.add_argument("--accum", type=int, default=None)
    ap.add_argument("--hw", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-examples", type=int, default=32,
                    help="examples of micro-batch 0 the oracle is timed on (32 = about 10 s on 16 cores)")
    ap.add_argument("--table", action="store_true", help="per-variant timing table on stderr")
    ap.add_argument("--streams", type=int, default=None,
                    help="side streams for independent layers (default 8; 4 for micro-steps of one or two examples)")
    ap.add_argument("--clip-unit", type=int, default=1,
                    help="examples per clipping unit (1: every example is clipped; 2, 4: the micro-batch clipping of the GPU baseline)")
    ap.add_argument("--fork", default=None, choices=("micro_step", "step"),
                    help="whether the side streams wait for the main stream every micro-step or once per step (default: by micro-batch size)")
    ap.add_argument("--lanes", default="balanced", choices=("round_robin", "balanced", "flops"),
                    help="how the batch calls of a phase are dealt to the side streams")
    ap.add_argument("--batching", default="variant", choices=("variant", "all"),
                    help="layers per batch call: those of one kernel variant, or all layers of a phase")
    ap.add_argument("--noise", default="once", choices=["once", "per_example"],
                    help="once: N(0, sigma^2 C^2) in finalize; per_example: every clipped example brings N(0, sigma^2 C^2/|B|)")
    ap.add_argument("--fused-update", action="store_true",
                    help="finalize applies the SGD-with-momentum step in the same kernel (extra work inside the step)")
    ap.add_argument("--no-graph", action="store_true", help="issue every call from the host instead of a HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of it); "
                 "run with --gpus 1")

    import torch
    import paper_2109_12191_amd as dp
    from workloads import get_workload
    from workloads.device import make_device_inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dp.load_library()
    device = torch.device("cuda:0")
    wl = get_workload(args.workload, n=args.n, accum=args.accum, hw=args.hw)
    if args.streams is None:
        args.streams = 4 if wl.n <= 2 else 8
    ps = dp.PrivatiseStep(wl, device="cuda:0", mode=args.mode, streams=args.streams, noise=args.noise,
                          batching=args.batching, lanes=args.lanes, clip_unit=args.clip_unit, fork=args.fork)
    inputs = make_device_inputs(wl, wl.accum, device)
    if args.fused_update:
        ps.enable_update(lr=0.1, momentum=0.9, keep_gradient=False)
    torch.cuda.synchronize()

    # The timed step: the whole path (8 micro-steps + finalize).  By default it is recorded once
    # into a HIP graph (independent layers on side streams) and replayed, so the host issues one
    # launch per step.
    if args.no_graph:
        one_step = lambda: ps.run(inputs)
    else:
        ps.capture(inputs)
        one_step = ps.replay
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # Roofline of the dominant kernel: the same steps issued call by call on ONE stream right
    # after the timed region, every contraction kernel bracketed by events on that stream.
    pe = dp.PrivatiseStep(wl, device="cuda:0", mode=args.mode, streams=1, noise=args.noise, clip_unit=args.clip_unit)
    probe = Probe()
    pe.probe = probe
    pe.run(inputs)
    torch.cuda.synchronize()
    probe.enabled = True
    probe_steps = min(args.steps, 3)
    tp0 = time.perf_counter()
    for _ in range(probe_steps):
        pe.run(inputs)
    torch.cuda.synchronize()
    probe_elapsed = time.perf_counter() - tp0
    probe.enabled = False

    summary = probe.summary()
    esize = wl.elem_bytes
    contraction = {k: v for k, v in summary.items() if k.startswith("conv")}
    if not contraction:
        # a workload without convolutions (the two-layer MLP): no contraction kernel to report on
        roofline = None
    else:
        # The dominant kernel: the contraction variant with the most work against the chip's roofs (the time its launches
        # would take at the peak that binds them, max(flop / MFMA peak, bytes / HBM peak)): the kernel that bounds the step
        # once every kernel runs at its roof.  The measured time of the single-stream pass below is NOT the criterion:
        # inside a batch call some launches are planned narrow on purpose (one example range per tile, no partial
        # blocks, no slice-sum launch), because the other streams of the replayed step fill the compute units they
        # leave free; alone on the chip, as this pass runs them, those launches are slow.  `variants` lists every
        # contraction variant with its time in this pass, so nothing hides behind the choice.
        peak = MFMA_PEAK[wl.dtype]
        def at_roof(v):
            return max(v["flops"] / peak, v["bytes"] / HBM_PEAK)
        dom_name, dom = max(contraction.items(), key=lambda kv: at_roof(kv[1]))
        # which roof binds this kernel: its arithmetic intensity against the ridge of the chip
        secs = dom["total_ms"] * 1e-3
        flop_rate, byte_rate = dom["flops"] / secs, dom["bytes"] / secs
        intensity = dom["flops"] / dom["bytes"]
        hbm_bound = intensity < peak / HBM_PEAK
        roofline = dict(bound="hbm" if hbm_bound else "mfma",
                        achieved=byte_rate / 1e9 if hbm_bound else flop_rate / 1e12,
                        peak=HBM_PEAK / 1e9 if hbm_bound else peak / 1e12,
                        unit="GB/s" if hbm_bound else "TFLOP/s",
                        frac=byte_rate / HBM_PEAK if hbm_bound else flop_rate / peak,
                        traffic=measured_traffic(dom_name) if (args.workload == "resnet50" and args.mode == "auto" and args.n is None
                                                               and args.hw is None and args.accum is None) else None,
                        traffic_unit="HBM bytes per launch (rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, see profiles/contraction_resnet50_hbm_traffic.txt)",
                        kernel=dom_name, launches=dom["launches"], avg_launch_us=dom["total_ms"] * 1e3 / dom["launches"],
                        algorithmic_bytes_per_launch=dom["bytes"] / dom["launches"],
                        algorithmic_flop_per_launch=dom["flops"] / dom["launches"],
                        flop_per_byte=intensity, ridge_flop_per_byte=peak / HBM_PEAK,
                        mfma_tflops=flop_rate / 1e12, mfma_frac=flop_rate / peak,
                        share_of_contraction_time=dom["total_ms"] / sum(v["total_ms"] for v in contraction.values()),
                        share_of_contraction_work_at_roof=at_roof(dom) / sum(at_roof(v) for v in contraction.values()),
                        selection="the contraction variant with the largest max(flop / MFMA peak, bytes / HBM peak) per step",
                        variants=[dict(kernel=k, launches_per_step=v["launches"] // probe_steps,
                                       ms_per_step=round(v["total_ms"] / probe_steps, 4),
                                       tflops=round(v["flops"] / (v["total_ms"] * 1e-3) / 1e12, 1),
                                       GBps=round(v["bytes"] / (v["total_ms"] * 1e-3) / 1e9, 1),
                                       frac_of_its_roof=round(at_roof(v) / (v["total_ms"] * 1e-3), 3))
                                  for k, v in sorted(contraction.items(), key=lambda kv: -at_roof(kv[1]))],
                        measured="HIP events recorded by the library around each launch of this kernel, on its stream, "
                                 "in a call-by-call single-stream pass over the same steps right after the timed region")
    # The streaming kernels of the step, each launched as the step launches it (same buffers, same sizes) and
    # bracketed by events on its stream: H4a, the clip-scale-accumulate pass over the materialised gradients of one
    # micro-step, and H5, noise + finalize over the whole parameter vector in one launch.
    streaming = {}
    def _time_stream(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        pairs = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in pairs)
        return ts[len(ts) // 2] * 1e-3
    if pe.p_mat and pe.n_groups == 1:
        g_bufs = [pe._g[0], ps._g[0]] if ps._g[0] is not None else [pe._g[0]]      # alternate: not cache resident
        k = [0]
        def _ca():
            k[0] += 1
            dp.dp_clip_accumulate(g_bufs[k[0] % len(g_bufs)], pe._group_sqnorm[0][0], pe.group_clip[0], pe.rows, pe.p_mat,
                                  pe.acc, g_stride=pe.p_mat)
        sec = _time_stream(_ca)
        nbytes = 4.0 * pe.rows * pe.p_mat + 8.0 * pe.p_mat
        streaming["clip_accumulate"] = dict(kernel="clip_accumulate_kernel", bytes=nbytes, us=sec * 1e6,
                                            achieved_GBps=nbytes / sec / 1e9, frac=nbytes / sec / HBM_PEAK,
                                            what=f"reads the [{pe.rows}, {pe.p_mat}] fp32 gradient matrix once, reads and writes the accumulator")
    def _fin():
        dp.dp_add_noise_finalize_flat(pe.acc, pe.out, pe._tensors, wl.sigma, pe.clip_total, wl.total_batch, wl.philox_seed,
                                      step_dev=pe._step_dev)
    sec = _time_stream(_fin)
    nbytes = 8.0 * wl.n_params
    streaming["noise_finalize"] = dict(kernel="noise_finalize_flat_kernel", bytes=nbytes, us=sec * 1e6,
                                       achieved_GBps=nbytes / sec / 1e9, frac=nbytes / sec / HBM_PEAK,
                                       what=f"{wl.n_params} parameters in one launch: 4 B read + 4 B written each, Philox4x32-10 + Box-Muller per 4")
    if roofline is not None:
        roofline["streaming"] = streaming
        roofline["streaming_measured"] = ("median of 10 launches, each bracketed by events on its stream (the events add 1-2 us "
                                          "to a launch; rocprofv3 durations of the same kernels are in profiles/)")
    if args.table:
        for k, v in streaming.items():
            print(f"{k:50s} {v['us']:9.1f} us  {v['achieved_GBps']:8.1f} GB/s  {v['frac']:.2f} of HBM peak", file=sys.stderr)
        for k, v in sorted(summary.items(), key=lambda kv: -kv[1]["total_ms"]):
            tf = v["flops"] / (v["total_ms"] * 1e-3) / 1e12 if v["total_ms"] else 0.0
            gb = v["bytes"] / (v["total_ms"] * 1e-3) / 1e9 if v["total_ms"] else 0.0
            print(f"{k:50s} launches {v['launches']:6d}  {v['total_ms'] / probe_steps:9.3f} ms/step  "
                  f"{tf:8.1f} TFLOP/s  {gb:8.1f} GB/s (algorithmic)  {v['flops'] / v['bytes']:6.1f} flop/B", file=sys.stderr)
        print("forms:", {f: ps.form.count(f) for f in set(ps.form)}, f"eager ms/step {probe_elapsed / probe_steps * 1e3:.2f}",
              file=sys.stderr)

    # The whole step against the HBM roof: algorithmic bytes of every call of a step (operands once per call, per-example
    # gradients written and read back where they are materialised, the accumulator read and written by every clipped
    # sum, finalize) over the measured step time.
    step_bytes = wl.accum * (sum(w[1] for w in ps.work) + sum(w[2] for w, f in zip(ps.work, ps.form) if f == "recompute")
                             + (4.0 * ps.rows * ps.p_mat + 8.0 * ps.p_mat)) + 8.0 * wl.n_params
    step_flops = wl.accum * (sum(w[0] for w in ps.work) + sum(w[0] for w, f in zip(ps.work, ps.form) if f == "recompute"))
    step_sec = elapsed / args.steps
    if roofline is not None:
        roofline["whole_step"] = dict(algorithmic_bytes=step_bytes, algorithmic_flop=step_flops, GBps=step_bytes / step_sec / 1e9,
                                      frac_of_hbm_peak=step_bytes / step_sec / HBM_PEAK, tflops=step_flops / step_sec / 1e12)
    line = {
        "metric": "privatised examples/sec at ResNet-50 layer shapes",
        "value": args.steps * wl.total_batch / elapsed,
        "unit": "examples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {len(wl.layers)} layers, {wl.n_params} parameters, micro-batch {wl.n} x "
                               f"{wl.accum} accumulation = {wl.total_batch} examples/step, {wl.clip_mode} clipping "
                               f"C={wl.clip_c}, sigma={wl.sigma}, {wl.dtype} inputs, fp32 accumulators"
                               + (f", clipping units of {args.clip_unit} examples" if args.clip_unit > 1 else ""),
                   "clipped_sum_forms": {f: ps.form.count(f) for f in sorted(set(ps.form))},
                   "issue": "host calls" if args.no_graph else f"HIP graph, {args.streams} side streams",
                   "finalize": "noise + SGD-momentum update fused" if args.fused_update else "noise + divide by |B|",
                   "noise_form": args.noise,
                   "flop_per_example": wl.flops_per_example, "input_bytes_per_example": wl.in_bytes_per_example},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, inputs[0], args.cpu_examples)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
