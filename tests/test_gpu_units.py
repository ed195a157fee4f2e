"""GPU parity for clipping units of several examples (the micro-batching of the GPU baseline, Abstract and Table 1):
dp_unit_grad against the oracle's unit means, and a whole optimiser step with units through the C ABI against
oracle.privatise_units."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2109_12191_amd as dp
from gpu_util import BF16_TOL, F32_TOL, assert_close, dev, host
from workloads import conv, dense, gn_affine, to_bf16_grid
from workloads.configs import Workload

pytestmark = pytest.mark.gpu


def _inputs(layer, n, seed, dtype, dy_std=0.05):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n,) + tuple(layer.x_shape)).astype(np.float32)
    dy = (rng.standard_normal((n,) + tuple(layer.dy_shape)) * dy_std).astype(np.float32)
    if dtype == "bf16":
        x, dy = to_bf16_grid(x), to_bf16_grid(dy)
    return x, dy


UNIT_CASES = [
    ("1x1 aligned rows 64x64 tile", conv(64, 64, 1, 1, 12), "bf16"),
    ("1x1 aligned rows 128x128 tiles ragged", conv(160, 136, 1, 1, 10), "bf16"),
    ("1x1 odd S gather bias", conv(40, 72, 1, 1, 7, bias=True), "bf16"),
    ("1x1 stride 2", conv(48, 80, 1, 2, 14), "bf16"),
    ("3x3 raw rows w14", conv(64, 128, 3, 1, 14), "bf16"),
    ("3x3 raw rows w28 ragged channels", conv(72, 136, 3, 1, 28), "bf16"),
    ("3x3 stride 2", conv(64, 64, 3, 2, 16), "bf16"),
    ("3x3 small channels", conv(8, 24, 3, 1, 9, bias=True), "bf16"),
    ("7x7 stride 2 stem", conv(3, 32, 7, 2, 30), "bf16"),
    ("fp32 3x3 bias", conv(12, 20, 3, 1, 11, bias=True), "f32"),
    ("fp32 1x1", conv(70, 90, 1, 1, 8), "f32"),
    ("dense tokens", dense(100, 36, tokens=3), "bf16"),
    ("dense fp32 one token", dense(784, 50), "f32"),
    ("gn affine", gn_affine(32, 10, 8), "f32"),
    ("gn affine bf16 wide groups", gn_affine(512, 4, 2), "bf16"),
]


@pytest.mark.parametrize("unit,units", [(2, 3), (4, 2), (3, 1)])
@pytest.mark.parametrize("materialise", [True, False])
@pytest.mark.parametrize("name,layer,dtype", UNIT_CASES, ids=[c[0] for c in UNIT_CASES])
def test_unit_sums_and_norms_match_the_oracle(name, layer, dtype, unit, units, materialise):
    n = unit * units
    x, dy = _inputs(layer, n, 4100 + unit, dtype)
    d = dp.make_desc(layer, n, dtype)
    need = dp.dp_unit_workspace_bytes(d, unit)
    ws = torch.empty(max(16, need), dtype=torch.uint8, device="cuda:0")
    sq = torch.full((units,), -1.0, device="cuda:0")
    gw = torch.full((units, layer.pw), 7.0, device="cuda:0") if materialise else None
    gb = torch.full((units, max(layer.pb, 1)), 7.0, device="cuda:0") if materialise else None
    dp.dp_unit_grad(d, unit, dev(x, dtype), dev(dy, dtype), gw, gb if (materialise and layer.pb) else None, sq, ws,
                    g_stride=0)
    torch.cuda.synchronize()
    mean_w, mean_b = oracle.unit_mean_grad(layer, x, dy, unit)
    tol = BF16_TOL if dtype == "bf16" else F32_TOL
    want_n2 = np.array([oracle.sqnorm(mean_w[u]) + (oracle.sqnorm(mean_b[u]) if layer.pb else 0.0) for u in range(units)])
    assert np.allclose(host(sq) / unit ** 2, want_n2, rtol=tol, atol=0), (host(sq) / unit ** 2, want_n2)
    if materialise:
        for u in range(units):
            assert_close(host(gw[u]) / unit, mean_w[u], tol, f"{name} unit {u} dW")
            if layer.pb:
                assert_close(host(gb[u, :layer.pb]) / unit, mean_b[u], tol, f"{name} unit {u} db")


@pytest.mark.parametrize("unit,units", [(2, 3), (4, 1)])
def test_unit_batch_call_matches_the_oracle_and_the_single_layer_calls(unit, units):
    """dp_unit_grad_batch over all bf16 geometries of UNIT_CASES at once (layers of one kernel share a launch)."""
    cases = [c for c in UNIT_CASES if c[2] == "bf16"]
    n = unit * units
    layers = [c[1] for c in cases]
    ins = [_inputs(l, n, 5200 + k, "bf16") for k, l in enumerate(layers)]
    descs = [dp.make_desc(l, n, "bf16") for l in layers]
    xs = [dev(x, "bf16") for x, _ in ins]
    dys = [dev(dy, "bf16") for _, dy in ins]
    wss = [torch.empty(max(16, dp.dp_unit_workspace_bytes(d, unit)), dtype=torch.uint8, device="cuda:0") for d in descs]
    sq = torch.full((len(layers), units), -1.0, device="cuda:0")
    gws = [torch.full((units, l.pw), 7.0, device="cuda:0") for l in layers]
    gbs = [torch.full((units, max(l.pb, 1)), 7.0, device="cuda:0") for l in layers]
    batch = dp.LayerBatch(descs, [w.data_ptr() for w in wss], [w.numel() for w in wss])
    for rep in range(2):                                   # twice: same bits on every call
        dp.dp_unit_grad_batch(batch, unit, batch.ptrs([t.data_ptr() for t in xs]), batch.ptrs([t.data_ptr() for t in dys]),
                              batch.ptrs([t.data_ptr() for t in gws]),
                              batch.ptrs([t.data_ptr() if l.pb else None for t, l in zip(gbs, layers)]),
                              batch.ptrs([sq[k].data_ptr() for k in range(len(layers))]))
        torch.cuda.synchronize()
        if rep == 0:
            first = (sq.clone(), [g.clone() for g in gws])
        else:
            assert torch.equal(sq, first[0]) and all(torch.equal(a, b) for a, b in zip(gws, first[1]))
    for k, l in enumerate(layers):
        x, dy = ins[k]
        mean_w, mean_b = oracle.unit_mean_grad(l, x, dy, unit)
        want_n2 = np.array([oracle.sqnorm(mean_w[u]) + (oracle.sqnorm(mean_b[u]) if l.pb else 0.0) for u in range(units)])
        assert np.allclose(host(sq[k]) / unit ** 2, want_n2, rtol=BF16_TOL, atol=0), (cases[k][0], host(sq[k]) / unit ** 2, want_n2)
        for u in range(units):
            assert_close(host(gws[k][u]) / unit, mean_w[u], BF16_TOL, f"{cases[k][0]} unit {u} dW")
            if l.pb:
                assert_close(host(gbs[k][u, :l.pb]) / unit, mean_b[u], BF16_TOL, f"{cases[k][0]} unit {u} db")
        one = torch.zeros((units, l.pw), device="cuda:0")
        oneb = torch.zeros((units, max(l.pb, 1)), device="cuda:0")
        sq1 = torch.zeros(units, device="cuda:0")
        dp.dp_unit_grad(descs[k], unit, xs[k], dys[k], one, oneb if l.pb else None, sq1, wss[k])
        torch.cuda.synchronize()
        assert_close(host(gws[k]), host(one), 2e-5, f"{cases[k][0]} against the single-layer call")
        assert np.allclose(host(sq[k]), host(sq1), rtol=3e-5, atol=0)


def test_unit_call_rejects_bad_arguments():
    l = conv(64, 64, 1, 1, 12)
    d = dp.make_desc(l, 6, "bf16")
    x, dy = _inputs(l, 6, 1, "bf16")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    sq = torch.zeros(6, device="cuda:0")
    with pytest.raises(dp.DpError):
        dp.dp_unit_grad(d, 4, dev(x, "bf16"), dev(dy, "bf16"), None, None, sq, ws)           # 6 is not a multiple of 4
    with pytest.raises(dp.DpError):
        dp.dp_unit_grad(d, 0, dev(x, "bf16"), dev(dy, "bf16"), None, None, sq, ws)
    with pytest.raises(dp.DpError):
        dp.dp_unit_grad(d, 2, dev(x, "bf16"), dev(dy, "bf16"), None, None, sq, ws[:16])      # workspace too small
    assert dp.dp_unit_workspace_bytes(d, 4) == 0 and dp.dp_unit_workspace_bytes(d, 3) > 0


def _net():
    return (conv(3, 16, 3, 1, 12, bias=True, name="c0"), gn_affine(16, 12, 4, name="g0"),
            conv(16, 64, 3, 2, 12, name="c1"), conv(64, 64, 3, 1, 6, name="c2"), conv(64, 80, 1, 1, 6, name="c3"),
            dense(80, 10, name="fc"))


@pytest.mark.parametrize("clip_mode,dtype", [("global", "f32"), ("per_layer", "bf16")])
def test_whole_step_with_units_matches_the_oracle(clip_mode, dtype):
    """Units of 4 examples, 2 micro-steps of 8: dp_unit_grad, dp_norms, dp_clip_accumulate(_segments) with the bound
    unit * C on the unit sums, dp_add_noise_finalize_flat with clip_total * unit and the number of examples."""
    unit, n, accum = 4, 8, 2
    layers = _net()
    wl = Workload("small", layers, n, accum, dtype, clip_mode, 0.05, 0.7, tuple("normal" for _ in layers), 0.05, 99)
    steps = []
    for m in range(accum):
        steps.append([_inputs(l, n, 7000 + 10 * m + k, dtype) for k, l in enumerate(layers)])
    ref = oracle.privatise_units(wl, steps, unit)
    assert any((f < 1).any() for f in ref["f"])

    L, units = len(layers), n // unit
    descs = [dp.make_desc(l, n, dtype) for l in layers]
    offs, p = [], 0
    for l in layers:                                   # every tensor starts on a 16-byte boundary
        pw4 = (l.pw + 3) // 4 * 4
        offs.append((p, p + pw4))
        p += pw4 + (l.pb + 3) // 4 * 4
    p4 = p
    group_clip, clip_total = dp.dp_group_clip_bounds(wl.clip_c, wl.n_groups)
    acc = torch.zeros(p4, device="cuda:0")
    out = torch.zeros(p4, device="cuda:0")
    g = torch.zeros((units, p4), device="cuda:0")
    layer_sq = torch.zeros((L, units), device="cuda:0")
    group_sq = torch.zeros((wl.n_groups, units), device="cuda:0")
    gol = torch.tensor(wl.group_of_layer, dtype=torch.int32, device="cuda:0")
    wss = [torch.empty(max(16, dp.dp_unit_workspace_bytes(d, unit)), dtype=torch.uint8, device="cuda:0") for d in descs]
    seg = dp.SegmentTable([o[0] for o in offs], list(wl.group_of_layer), [c * unit for c in group_clip])
    for inputs in steps:
        for k, (l, d) in enumerate(zip(layers, descs)):
            x, dy = inputs[k]
            dp.dp_unit_grad(d, unit, dev(x, dtype), dev(dy, dtype), g[:, offs[k][0]:], g[:, offs[k][1]:] if l.pb else None,
                            layer_sq[k], wss[k], g_stride=p4)
        dp.dp_norms(layer_sq, gol, L, units, wl.n_groups, group_sq)
        if wl.n_groups == 1:
            dp.dp_clip_accumulate(g, group_sq[0], group_clip[0] * unit, units, p4, acc, g_stride=p4)
        else:
            dp.dp_clip_accumulate_segments(g, group_sq, wl.n_groups, seg, units, p4, acc, g_stride=p4)
    table = dp.TensorTable([b for k, l in enumerate(layers) for b in ([offs[k][0], offs[k][1]] if l.pb else [offs[k][0]])],
                           [s for l in layers for s in ([l.pw, l.pb] if l.pb else [l.pw])],
                           [t for k, l in enumerate(layers) for t in ([2 * k, 2 * k + 1] if l.pb else [2 * k])])
    dp.dp_add_noise_finalize_flat(acc, out, table, wl.sigma, clip_total * unit, wl.total_batch, wl.philox_seed, step=wl.step)
    torch.cuda.synchronize()
    tol = BF16_TOL if dtype == "bf16" else F32_TOL
    got_n2 = host(group_sq).T / unit ** 2                      # last micro-step
    assert np.allclose(got_n2, ref["n2"][-1], rtol=tol, atol=0)
    for k, l in enumerate(layers):
        assert_close(host(acc[offs[k][0]:offs[k][0] + l.pw]) / unit, ref["acc_w"][k].reshape(-1), tol, f"layer {k} clipped sum")
        assert_close(host(out[offs[k][0]:offs[k][0] + l.pw]), ref["out_w"][k].reshape(-1), tol, f"layer {k} released gradient")
        if l.pb:
            assert_close(host(out[offs[k][1]:offs[k][1] + l.pb]), ref["out_b"][k], tol, f"layer {k} released bias gradient")


def test_pipeline_with_units_matches_the_oracle_eager_and_graph():
    """PrivatiseStep(clip_unit=4): side streams, two buffer copies, graph replay; against oracle.privatise_units."""
    from workloads import make_inputs
    unit = 4
    layers = _net()
    wl = Workload("small", layers, 8, 3, "bf16", "global", 0.05, 0.9, tuple("normal" for _ in layers), 0.05, 321)
    steps = [make_inputs(wl, m) for m in range(wl.accum)]
    ref = oracle.privatise_units(wl, steps, unit)
    assert any((f < 1).any() for f in ref["f"])
    dev_steps = [[(dev(x, wl.dtype), dev(dy, wl.dtype)) for x, dy in inputs] for inputs in steps]
    for streams in (1, 4):
        ps = dp.PrivatiseStep(wl, streams=streams, clip_unit=unit)
        assert all(f == "materialise" for f in ps.form)
        ps.run(dev_steps)
        torch.cuda.synchronize()
        for k, l in enumerate(layers):
            assert_close(host(ps.out_w(k)), ref["out_w"][k].reshape(-1), BF16_TOL, f"streams {streams} layer {k}")
            if l.pb:
                assert_close(host(ps.out_b(k)), ref["out_b"][k], BF16_TOL, f"streams {streams} layer {k} bias")
        eager = ps.out.clone()
    ps.set_step(wl.step)
    ps.capture(dev_steps)
    ps.replay()
    torch.cuda.synchronize()
    assert torch.equal(ps.out, eager)
