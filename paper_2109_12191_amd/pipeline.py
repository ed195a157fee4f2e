"""Sequencing of the C-ABI calls for one optimiser step of a layer set.

This class owns device buffers (allocated through torch) and issues the library calls in
order; it performs no arithmetic of its own.  Per micro-step:
    dp_per_example_grad_batch (one call per group of layers that run the same kernel)  ->  dp_norms  ->
    dp_clip_accumulate (materialised layers) and dp_clip_accumulate_recompute_batch (the rest);
once per optimiser step: dp_add_noise_finalize per parameter tensor.

Each layer uses one of the two forms of the clipped sum.  "materialise" keeps the layer's
per-example gradients of the micro-step in a [n, P] matrix (written by the contraction's
epilogue, read once by the streaming accumulate); "recompute" keeps nothing and runs a
second, clip-factor-weighted contraction.  `mode="auto"` picks per layer whichever moves
fewer bytes / flops; early conv layers (few parameters, large feature maps) materialise,
late ones (many parameters, tiny feature maps) recompute.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B

def _pad4(v: int) -> int:
    return (v + 3) & ~3


class PrivatiseStep:
    def __init__(self, wl, device: str = "cuda:0", mode: str = "auto", streams: int = 1, noise: str = "once",
                 batching: str = "variant", lanes: str = "balanced", clip_unit: int = 1, fork: Optional[str] = None):
        B.load_library()
        self.wl = wl
        if batching not in ("variant", "all"):
            raise ValueError(batching)
        # "variant": one batch call per kernel variant, spread over the side streams (large micro-batches: the
        # launches are long and overlap); "all": one batch call per phase with every layer in it, so that also the
        # pre-passes and slice sums of all layers share launches (one-example micro-steps: launches are what costs)
        self.batching = batching
        if lanes not in ("round_robin", "balanced", "flops"):
            raise ValueError(lanes)
        self.lanes = lanes                     # how the batch calls of a phase are dealt to the side streams
        # "micro_step": the side streams of the per-example phase start every micro-step behind everything issued so
        # far; "step": only the first micro-step of a step does -- later ones follow their own stream's previous
        # micro-step (and the clipped sum that last read their buffer copy), so they overlap the norm launches and the
        # clipped sum of the micro-step before.  Worth it when the launches are short (one or two examples each).
        if fork not in (None, "micro_step", "step"):
            raise ValueError(fork)
        self.fork = fork if fork is not None else ("step" if wl.n <= 2 else "micro_step")
        if noise not in ("once", "per_example"):
            raise ValueError(noise)
        # "once": N(0, sigma^2 C^2) added in finalize (first equation of the Algorithm section);
        # "per_example": every clipped example brings N(0, sigma^2 C^2 / |B|) (second equation)
        self.noise = noise
        self.device = torch.device(device)
        self.layers = list(wl.layers)
        self.n = wl.n
        # Clipping units of several consecutive examples (the micro-batching of the GPU baseline, Abstract and
        # Table 1): the path runs on the unit SUMS with every bound multiplied by the unit size, which gives
        # (noise + sum of the clipped unit means) / (number of units); a unit is one row wherever an example is.
        self.clip_unit = int(clip_unit)
        if self.clip_unit < 1 or wl.n % self.clip_unit:
            raise ValueError("the micro-step size must be a multiple of clip_unit")
        if self.clip_unit > 1 and noise != "once":
            raise ValueError("per-example noise is defined for units of one example")
        self.rows = wl.n // self.clip_unit
        L = len(self.layers)
        self.descs = [B.make_desc(l, wl.n, wl.dtype) for l in self.layers]
        self.pw = [B.dp_weight_count(d) for d in self.descs]
        self.pb = [B.dp_bias_count(d) for d in self.descs]
        self.group_of_layer = list(wl.group_of_layer)
        self.group_clip, self.clip_total = B.dp_group_clip_bounds(wl.clip_c, wl.n_groups)
        if self.clip_unit > 1:
            self.group_clip = [c * self.clip_unit for c in self.group_clip]
            self.clip_total *= self.clip_unit
            mode = "materialise"                   # the unit sums are 1/unit of the per-example matrix: keep them
        self.n_groups = wl.n_groups
        self.form = [self._choose(l, mode) for l in self.layers]

        # flat parameter vector: materialised layers first (their columns double as the
        # layout of the per-example gradient matrix), then the recomputed ones
        order = [i for i in range(L) if self.form[i] == "materialise"] + \
                [i for i in range(L) if self.form[i] == "recompute"]
        self.off_w = [0] * L
        self.off_b = [0] * L
        pos = 0
        self.p_mat = 0
        for i in order:
            self.off_w[i] = pos
            pos += _pad4(self.pw[i])
            self.off_b[i] = pos
            pos += _pad4(self.pb[i])
            if self.form[i] == "materialise":
                self.p_mat = pos
        self.p_total = max(pos, 4)
        # every tensor of the flat vector with its Philox tensor id (2*layer weight, 2*layer+1 bias), in
        # the order they lie in memory: the table of the one-launch finalize
        tensors = sorted([(self.off_w[i], self.pw[i], 2 * i) for i in range(L)] +
                         [(self.off_b[i], self.pb[i], 2 * i + 1) for i in range(L) if self.pb[i]])
        self._tensors = B.TensorTable([t[0] for t in tensors], [t[1] for t in tensors], [t[2] for t in tensors])
        mat = [i for i in order if self.form[i] == "materialise"]
        self._segments = B.SegmentTable([self.off_w[i] for i in mat], [self.group_of_layer[i] for i in mat],
                                        [self.group_clip[self.group_of_layer[i]] for i in mat]) if mat else None
        dev = self.device
        f32 = torch.float32
        self.acc = torch.zeros(self.p_total, dtype=f32, device=dev)
        self.out = torch.zeros(self.p_total, dtype=f32, device=dev)
        # Workspaces and per-micro-step buffers.  With one stream all calls run in order and share
        # one workspace.  With side streams the layers of a phase run concurrently (a workspace per
        # layer) and the two phases of consecutive micro-steps overlap: everything a micro-step
        # writes before its clipped sum is done -- the gradient matrix, the norms, the workspaces --
        # exists twice and micro-steps alternate between the copies.
        self.n_streams = max(1, int(streams))
        self.copies = 2 if self.n_streams > 1 else 1
        self._g = [torch.zeros((self.rows, self.p_mat), dtype=f32, device=dev) if self.p_mat else None
                   for _ in range(self.copies)]
        self._group_sqnorm = [torch.zeros((self.n_groups, self.rows), dtype=f32, device=dev) for _ in range(self.copies)]
        self.group_of_layer_dev = torch.tensor(self.group_of_layer, dtype=torch.int32, device=dev)
        need = [max(16, B.dp_workspace_bytes(d, B.DP_WS_PER_EXAMPLE_GRAD),
                    B.dp_workspace_bytes(d, B.DP_WS_RECOMPUTE) if form == "recompute" else 0,
                    B.dp_unit_workspace_bytes(d, self.clip_unit) if self.clip_unit > 1 else 0)
                for d, form in zip(self.descs, self.form)]
        # a workspace per layer (the layers of a phase are in flight together)
        self._ws = [[torch.empty(b, dtype=torch.uint8, device=dev) for b in need] for _ in range(self.copies)]
        self._layer_sqnorm = [torch.zeros((L, self.rows), dtype=f32, device=dev) for _ in range(self.copies)]
        # Layers that run the same kernel variant go to the library in ONE batch call, which puts them into one
        # launch (at most 16 per launch): per phase a micro-step is a dozen launches, not a hundred.
        self.variant = [(B.dp_kernel_variant(d, B.DP_WS_PER_EXAMPLE_GRAD | B.DP_VARIANT_SHARED |
                                             (B.DP_VARIANT_MATERIALISE if form == "materialise" else 0)),
                         B.dp_kernel_variant(d, B.DP_WS_RECOMPUTE | B.DP_VARIANT_SHARED))
                        for d, form in zip(self.descs, self.form)]
        import ctypes
        self._partial_counts = (ctypes.c_int32 * L)()
        self._partials = [(ctypes.c_void_p * L)(*[self._ws[c][i].data_ptr() for i in range(L)]) for c in range(self.copies)]
        self._layer_sqnorm_ptrs = [(ctypes.c_void_p * L)(*[self._layer_sqnorm[c][i].data_ptr() for i in range(L)])
                                   for c in range(self.copies)]
        esize = 2 if wl.dtype == "bf16" else 4
        # algorithmic work of one call per layer: (flop, HBM bytes of the per-example call, HBM bytes of the
        # recomputing clipped-sum call).  Bytes = the operands read once, plus the per-example gradients
        # written when the layer materialises them, or the accumulator read and written by form (b).
        self.work = [(l.flops * wl.n,
                      l.in_bytes(esize) * wl.n + (4 * wl.n * (pw + pb) if form == "materialise" else 0),
                      l.in_bytes(esize) * wl.n + 8 * (pw + pb))
                     for l, pw, pb, form in zip(self.layers, self.pw, self.pb, self.form)]
        self._groups_a = self._make_groups(range(L), 0)
        self._groups_b = self._make_groups([i for i in range(L) if self.form[i] == "recompute"], 1)
        self._groups_u = self._make_groups(range(L), 2) if self.clip_unit > 1 else []
        # side streams: `side` for the per-example phase, `side_b` for the clipped-sum phase
        self.side = [torch.cuda.Stream(device=dev) for _ in range(self.n_streams)] if self.n_streams > 1 else []
        # (three clipped-sum streams for eight per-example streams: measured 3 % better over the whole step than four)
        self.side_b = [torch.cuda.Stream(device=dev) for _ in range(max(2, 3 * self.n_streams // 8))] if self.n_streams > 1 else []
        # optional fused optimiser step (enable_update): parameters and momentum buffer, laid out like acc
        self.theta = None
        self.velocity = None
        self._update = None                      # (lr, momentum, keep_gradient)
        self._b_done = [None] * self.copies      # per copy: events after which its buffers are free again
        self._last = 0                           # copy used by the most recent micro-step
        self.graph = None
        self.micro_steps_done = 0
        # Optimiser-step counter: the `step` word of the Philox counters.  The kernels read it from a device
        # word, so a captured graph draws fresh noise on every replay; finalize() advances it, `step` mirrors
        # it on the host.  Two optimiser steps never share a noise draw.
        self.step = int(wl.step)
        self._step_dev = torch.tensor([self.step], dtype=torch.int64, device=dev)
        # optional timing probe (bench.py): an object with arm(variant, flops, bytes) that asks the
        # library to bracket the next contraction kernel with a pair of events
        self.probe = None

    def _make_groups(self, layer_ids, use: int):
        """Groups of at most 16 layers with the same kernel variant for phase `use` (0: per-example gradients,
        1: recomputing clipped sum), largest total work first.  Each group: dict(layers, name, batch per copy,
        constant pointer arrays)."""
        by_name = {}
        family = "conv3x3_rows<bf16,all widths,%s>" % ("weighted" if use else "per_example")
        for li in layer_ids:
            key = self.variant[li][1 if use == 2 else use]      # same name, same kernel: storing and norm-only layers share a launch
            if self.batching == "all":
                key = "all layers"
            elif key.startswith("conv3x3_rows<"):
                # inside a batch call the library runs all variants of the raw-row 3x3 kernel in one launch (only
                # four kernels run at a time on the chip: the few workgroups of a narrow layer cost none of the
                # four inside a wide launch), so the family is one batch call
                key = family
            by_name.setdefault(key, []).append(li)
        groups = []
        for key, ids in by_name.items():
            width = len(ids) if (self.batching == "all" or key == family) else 16
            for k in range(0, len(ids), width):
                part = ids[k: k + width]
                name = key.split("|")[0]
                if len(part) == 1:           # a single layer is planned as a launch of its own
                    name = B.dp_kernel_variant(self.descs[part[0]], B.DP_WS_RECOMPUTE if use else (
                        B.DP_WS_PER_EXAMPLE_GRAD | (B.DP_VARIANT_MATERIALISE if self.form[part[0]] == "materialise" else 0)))
                g = dict(layers=part, name=name, conv=all(self.layers[i].kind == "conv" for i in part))
                g["batch"] = [B.LayerBatch([self.descs[i] for i in part], [self._ws[c][i].data_ptr() for i in part],
                                           [self._ws[c][i].numel() for i in part]) for c in range(self.copies)]
                if use == 2:
                    g["usq"] = [g["batch"][c].ptrs([self._layer_sqnorm[c][i].data_ptr() for i in part])
                                for c in range(self.copies)]
                if use != 1:
                    g["counted"] = False
                    mat = [self.form[i] == "materialise" for i in part]
                    g["gw"] = [g["batch"][c].ptrs([self._g[c][:, self.off_w[i]:].data_ptr() if m else None
                                                   for i, m in zip(part, mat)]) for c in range(self.copies)] if any(mat) else None
                    g["gb"] = [g["batch"][c].ptrs([self._g[c][:, self.off_b[i]:].data_ptr() if (m and self.pb[i]) else None
                                                   for i, m in zip(part, mat)]) for c in range(self.copies)] if any(mat) else None
                else:
                    g["sq"] = [g["batch"][c].ptrs([self._group_sqnorm[c][self.group_of_layer[i]].data_ptr() for i in part])
                               for c in range(self.copies)]
                    g["clip"] = g["batch"][0].floats([self.group_clip[self.group_of_layer[i]] for i in part])
                    g["acc_w"] = g["batch"][0].ptrs([self.acc[self.off_w[i]:].data_ptr() for i in part])
                    g["acc_b"] = g["batch"][0].ptrs([self.acc[self.off_b[i]:].data_ptr() if self.pb[i] else None
                                                     for i in part])
                g["flops"] = sum(self.layers[i].flops for i in part) * self.n
                g["bytes"] = sum(self.work[i][2 if use == 1 else 1] for i in part)
                g["seconds"] = self._estimate(g)
                groups.append(g)
        groups.sort(key=lambda g: -g["seconds"])
        # side stream of each group: longest first onto the least loaded stream
        load = [0.0] * max(1, self.n_streams)
        for gi, g in enumerate(groups):
            k = load.index(min(load)) if self.lanes != "round_robin" else gi % max(1, self.n_streams)
            g["lane"] = k
            load[k] += g["seconds"]
        return groups

    def _estimate(self, g) -> float:
        """Duration of a group's launch for the lane balance: its work at the rates its kernel family sustains on
        MI355X when it has the chip to itself (measured call by call on ResNet-50 at n = 32), plus a few
        microseconds per launch however small it is."""
        if self.lanes == "flops" or self.wl.n <= 2:
            # micro-steps of one or two examples: launches are bound by the walk along K of a few workgroups, not by
            # the chip's rates; flops alone order them better (measured: 5.6 k against 5.1 k examples/s)
            return g["flops"] / 150.0e12 + 8.0e-6
        name = g["name"]
        if name.startswith("conv3x3_rows"):
            rate = 300.0e12                      # (100 .. 300: the same step time; the family is one launch per phase)
        elif "gather" in name:
            rate = 130.0e12
        else:
            rate = 400.0e12
        return max(g["flops"] / rate, g["bytes"] / 4.5e12) + 8.0e-6

    def _arm(self, group, use: int):
        if self.probe is not None and group["conv"]:
            self.probe.arm(group["name"], sum(self.work[i][0] for i in group["layers"]),
                           sum(self.work[i][1 + use] for i in group["layers"]), len(group["layers"]))

    def _choose(self, layer, mode: str) -> str:
        if mode in ("materialise", "recompute"):
            return mode
        if mode != "auto":
            raise ValueError(mode)
        # Cost model fitted to the measured throughput of whole replayed steps on MI355X (micro-batch n, layers launched
        # in groups, kernels of several streams overlapping):
        #   materialise: the [n, P] fp32 gradients are written by the contraction's epilogue and read back by the
        #     streaming accumulate -- 8 n P bytes at ~5 TB/s;
        #   recompute: a second (clip-weighted) contraction -- the layer's inputs once more at ~4 TB/s and its flops
        #     at ~275 TFLOP/s sustained (no fixed cost: the weighted kernels run one example range per tile inside
        #     batch calls, without partial blocks or slice sums).
        # ResNet-50 at n = 32: the stride-1 3x3 layers of stage 3, stage 4 but its first 1x1 layer, and the classifier
        # recompute (15 layers, 19.4 M parameters).  Whole-step throughput around this split: 37/17 (300 TFLOP/s: the
        # strided 3x3 layer of stage 3, whose weighted form has no raw-row kernel, and the first 1x1 of stage 4 recompute
        # too) - 2 %, 44/10 (250) - 9 %, 26/28 (360) - 3 %.
        if self.n <= 2:
            # micro-steps of one or two examples are bound by their launches, and a recomputing layer brings launches of its
            # own to the clipped-sum phase (measured: 5.9 k against 5.6 k examples/s with the split above)
            return "materialise"
        p = layer.pw + layer.pb
        esize = 2 if self.wl.dtype == "bf16" else 4
        materialise = 8.0 * p * self.n / 5.0e12
        recompute = layer.in_bytes(esize) * self.n / 4.0e12 + layer.flops * self.n / 275.0e12
        return "materialise" if materialise <= recompute else "recompute"

    # ---- views of one layer's tensors in the flat vectors
    def acc_w(self, li: int) -> torch.Tensor:
        return self.acc[self.off_w[li]: self.off_w[li] + self.pw[li]]

    def acc_b(self, li: int) -> Optional[torch.Tensor]:
        return self.acc[self.off_b[li]: self.off_b[li] + self.pb[li]] if self.pb[li] else None

    def out_w(self, li: int) -> torch.Tensor:
        return self.out[self.off_w[li]: self.off_w[li] + self.pw[li]]

    def out_b(self, li: int) -> Optional[torch.Tensor]:
        return self.out[self.off_b[li]: self.off_b[li] + self.pb[li]] if self.pb[li] else None

    @property
    def group_sqnorm(self) -> torch.Tensor:
        """[groups, n] squared norms of the most recent micro-step."""
        return self._group_sqnorm[self._last]

    @property
    def g(self) -> Optional[torch.Tensor]:
        return self._g[self._last]

    def enable_update(self, lr: float, momentum: float = 0.0, theta: Optional[torch.Tensor] = None,
                      keep_gradient: bool = True):
        """Make finalize() apply the SGD step in the same kernel (dp_add_noise_finalize_update): theta and the
        momentum buffer are flat vectors laid out like the accumulator.  `lr` can be changed per step with set_lr."""
        self.theta = torch.zeros_like(self.acc) if theta is None else theta
        self.velocity = torch.zeros_like(self.acc) if momentum != 0.0 else None
        self._update = [float(lr), float(momentum), bool(keep_gradient)]

    def set_lr(self, lr: float):
        self._update[0] = float(lr)

    def theta_w(self, li: int) -> torch.Tensor:
        return self.theta[self.off_w[li]: self.off_w[li] + self.pw[li]]

    def theta_b(self, li: int) -> Optional[torch.Tensor]:
        return self.theta[self.off_b[li]: self.off_b[li] + self.pb[li]] if self.pb[li] else None

    def set_step(self, step: int):
        """Set the optimiser-step counter (e.g. when a run is resumed)."""
        self.step = int(step)
        self._step_dev.fill_(self.step)

    def begin_step(self):
        self.acc.zero_()
        self.micro_steps_done = 0
        self._b_done = [None] * self.copies

    def micro_step(self, inputs: Sequence):
        """inputs: per layer (x, dy) device tensors of the workload's dtype, n examples each.

        Phase A (per-example gradients + norms of every layer) and phase B (clipped sum) of one
        micro-step are separated by dp_norms.  Layers within a phase are independent; with side
        streams they are spread over them, and phase A of the next micro-step does not wait for
        phase B of this one (they work on different buffer copies).  The clipped sums reach the
        accumulator in the same order on every run: each tensor is updated by one call per
        micro-step, always issued on the same stream."""
        L = len(self.layers)
        gs = self.p_mat
        c = self.micro_steps_done % self.copies
        self._last = c
        g_buf, gsq, wss = self._g[c], self._group_sqnorm[c], self._ws[c]
        main = torch.cuda.current_stream()
        # ---- phase A
        for st in self.side:
            if self.fork == "micro_step" or self.micro_steps_done == 0:
                st.wait_stream(main)
            if self._b_done[c] is not None:           # this copy's previous clipped sum has finished
                for ev in self._b_done[c]:
                    st.wait_event(ev)
        if self.clip_unit > 1:
            # unit sums and their norms: one batch call per kernel variant of the clip-weighted form (the kernels
            # that run), dealt to the side streams
            for grp in self._groups_u:
                st = self.side[grp["lane"]] if self.side else None
                bt = grp["batch"][c]
                xs = bt.ptrs([inputs[i][0].data_ptr() for i in grp["layers"]])
                dys = bt.ptrs([inputs[i][1].data_ptr() for i in grp["layers"]])
                B.dp_unit_grad_batch(bt, self.clip_unit, xs, dys, grp["gw"][c], grp["gb"][c], grp["usq"][c], g_stride=gs,
                                     stream=st)
        for gi, grp in enumerate(self._groups_a if self.clip_unit == 1 else ()):
            st = self.side[grp["lane"]] if self.side else None
            bt = grp["batch"][c]
            xs = bt.ptrs([inputs[i][0].data_ptr() for i in grp["layers"]])
            dys = bt.ptrs([inputs[i][1].data_ptr() for i in grp["layers"]])
            self._arm(grp, 0)
            B.dp_per_example_grad_batch(bt, xs, dys, grp["gw"][c] if grp["gw"] else None,
                                        grp["gb"][c] if grp["gb"] else None, None, g_stride=gs, stream=st)
            if not grp["counted"]:                     # how many partial sums per example each layer leaves behind
                for k, i in enumerate(grp["layers"]):
                    self._partial_counts[i] = bt.partial_counts[k]
                grp["counted"] = True
        for st in self.side:
            main.wait_stream(st)
        # H2: every layer's partial sums -> per-layer norms in one launch, per-group norms in a second
        if self.clip_unit == 1:
            B.dp_layer_norms_from_partials(self._partials[c], self._partial_counts, self._layer_sqnorm_ptrs[c], L, self.n)
        B.dp_norms(self._layer_sqnorm[c], self.group_of_layer_dev, L, self.rows, self.n_groups, gsq)
        # ---- phase B
        for st in self.side_b:
            st.wait_stream(main)
        sb = self.side_b
        if self.p_mat:
            st0 = sb[0] if sb else None
            if self.n_groups == 1:
                # one clipping group: every materialised tensor shares the factors -> one pass
                B.dp_clip_accumulate(g_buf, gsq[0], self.group_clip[0], self.rows, self.p_mat,
                                     self.acc, g_stride=gs, stream=st0)
            else:
                # several clipping groups: one launch over all materialised tensors, a segment per layer
                B.dp_clip_accumulate_segments(g_buf, gsq, self.n_groups, self._segments, self.rows, self.p_mat,
                                              self.acc, g_stride=gs, stream=st0)
        if self.noise == "per_example":
            for li in range(L):
                if self.form[li] == "materialise":
                    self._example_noise(li, sb[0] if sb else None)
        for gi, grp in enumerate(self._groups_b):
            st = sb[(1 + gi) % len(sb)] if sb else None
            bt = grp["batch"][c]
            xs = bt.ptrs([inputs[i][0].data_ptr() for i in grp["layers"]])
            dys = bt.ptrs([inputs[i][1].data_ptr() for i in grp["layers"]])
            self._arm(grp, 1)
            B.dp_clip_accumulate_recompute_batch(bt, xs, dys, grp["sq"][c], grp["clip"], grp["acc_w"], grp["acc_b"],
                                                 stream=st)
            if self.noise == "per_example":
                for li in grp["layers"]:
                    self._example_noise(li, st)
        if sb:
            evs = []
            for st in sb:
                ev = torch.cuda.Event()
                ev.record(st)
                evs.append(ev)
            self._b_done[c] = evs
        self.micro_steps_done += 1

    def _example_noise(self, li: int, st):
        """Per-example noise of this micro-step's examples for the tensors of layer li, on the stream that
        updates those tensors."""
        wl = self.wl
        first = self.micro_steps_done * self.n
        B.dp_add_example_noise(self.acc_w(li).data_ptr(), self.pw[li], wl.sigma, self.clip_total, wl.total_batch,
                               wl.philox_seed, 0, 2 * li, first, self.n, step_dev=self._step_dev, stream=st)
        if self.pb[li]:
            B.dp_add_example_noise(self.acc_b(li).data_ptr(), self.pb[li], wl.sigma, self.clip_total, wl.total_batch,
                                   wl.philox_seed, 0, 2 * li + 1, first, self.n, step_dev=self._step_dev, stream=st)

    def _drain(self):
        """The current stream waits for every clipped sum issued so far."""
        main = torch.cuda.current_stream()
        for st in self.side_b:
            main.wait_stream(st)

    def finalize(self):
        """H5 on the whole flat parameter vector in one launch (every tensor keeps its own Philox counters),
        with the SGD step fused in when enable_update() was called; then the step counter advances."""
        wl = self.wl
        self._drain()
        sigma = wl.sigma if self.noise == "once" else 0.0        # per-example form: the noise is already in acc
        if self._update is None:
            B.dp_add_noise_finalize_flat(self.acc, self.out, self._tensors, sigma, self.clip_total, wl.total_batch,
                                         wl.philox_seed, step_dev=self._step_dev)
        else:
            lr, momentum, keep = self._update
            B.dp_add_noise_finalize_flat(self.acc, self.out if keep else None, self._tensors, sigma, self.clip_total,
                                         wl.total_batch, wl.philox_seed, step_dev=self._step_dev, theta=self.theta,
                                         velocity=self.velocity, lr=lr, momentum=momentum)
        self._step_dev.add_(1)
        self.step += 1

    def run(self, inputs_per_micro_step: Sequence[Sequence]):
        self.begin_step()
        for inputs in inputs_per_micro_step:
            self.micro_step(inputs)
        self.finalize()
        return self.out

    def capture(self, inputs_per_micro_step: Sequence[Sequence]):
        """Record one whole optimiser step on these (persistent) input tensors into a HIP graph:
        replay() then re-issues every launch without host work.  Only kernels are recorded (the
        accumulator is cleared by a fill kernel, never by a memset node)."""
        assert self.probe is None or not getattr(self.probe, "enabled", False)
        step0 = self.step
        self.run(inputs_per_micro_step)          # warm-up outside capture (lazy module loads)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run(inputs_per_micro_step)
        self.graph = graph
        self.set_step(step0)                     # recording consumed no optimiser step
        return graph

    def replay(self):
        """Re-issue the recorded step.  The step counter lives in device memory and is advanced by the graph
        itself, so every replay draws fresh noise."""
        self.graph.replay()
        self.step += 1
        return self.out
