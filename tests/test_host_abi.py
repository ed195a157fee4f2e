"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad arguments on the host before anything could be launched (no GPU needed; no
compute call is made with valid arguments here)."""
import math
import os
import re

import pytest

import paper_2109_12191_amd as dp
from paper_2109_12191_amd import binding as B
from workloads import conv, dense, gn_affine, get_workload

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000          # a non-null, 16-byte aligned "device pointer" that is never dereferenced


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dp.lib_path()):
        from paper_2109_12191_amd.build import build
        build(verbose=False)
    return dp.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "dp_privatise.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dp_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTED)
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in dp.dp_version()


def test_parameter_counts_and_workspace_are_pure_host(lib):
    d = dp.make_desc(conv(64, 64, 3, 1, 56, bias=True), 16)
    assert dp.dp_weight_count(d) == 64 * 64 * 9 and dp.dp_bias_count(d) == 64
    assert dp.dp_workspace_bytes(d, dp.DP_WS_PER_EXAMPLE_GRAD) >= 16 * 4
    d = dp.make_desc(dense(2048, 1000), 32, "bf16")
    assert dp.dp_weight_count(d) == 2048000 and dp.dp_bias_count(d) == 1000
    d = dp.make_desc(gn_affine(64, 8, 8), 4)
    assert dp.dp_weight_count(d) == 64 and dp.dp_bias_count(d) == 64
    assert dp.dp_workspace_bytes(d, dp.DP_WS_RECOMPUTE) >= 4 * 2 * 64 * 4
    # the ResNet-50 layer set adds up to the published parameter count
    wl = get_workload("resnet50")
    total = sum(dp.dp_weight_count(dp.make_desc(l, 1, "bf16")) + dp.dp_bias_count(dp.make_desc(l, 1, "bf16"))
                for l in wl.layers)
    assert total == 25_503_912
    bad = dp.make_desc(conv(8, 8, 3, 1, 8), 0)
    assert dp.dp_weight_count(bad) == 0 and dp.dp_workspace_bytes(bad) == 0


def _raises(status, fn, *a, **k):
    with pytest.raises(dp.DpError) as ei:
        fn(*a, **k)
    assert ei.value.status == status, str(ei.value)
    assert dp.dp_last_error() != ""
    return str(ei.value)


def test_per_example_grad_argument_errors(lib):
    good = dp.make_desc(conv(8, 8, 3, 1, 8, bias=True), 4)
    ws = dp.dp_workspace_bytes(good)
    call = lambda d, x=FAKE, dy=FAKE, gw=FAKE, gb=FAKE, sq=FAKE, w=FAKE, wb=ws, gs=0: dp.dp_per_example_grad(
        d, x, dy, gw, gb, sq, w, g_stride=gs, ws_bytes=wb, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, call, good, x=None)
    _raises(B.DP_ERR_INVALID_ARG, call, good, dy=None)
    _raises(B.DP_ERR_INVALID_ARG, call, good, x=FAKE + 4)                 # misaligned
    _raises(B.DP_ERR_INVALID_ARG, call, good, gw=None, gb=None, sq=None)  # nothing to compute
    _raises(B.DP_ERR_INVALID_ARG, call, good, gb=None)                    # bias layer needs g_b with g_w
    _raises(B.DP_ERR_INVALID_ARG, call, good, gw=None)                    # g_b without g_w
    _raises(B.DP_ERR_INVALID_ARG, call, good, gs=6)                       # stride not a multiple of 4
    _raises(B.DP_ERR_INVALID_ARG, call, good, gs=8)                       # stride smaller than the tensor
    _raises(B.DP_ERR_WORKSPACE, call, good, w=None)
    _raises(B.DP_ERR_WORKSPACE, call, good, wb=ws - 1)
    for field, val in (("n", 0), ("cin", 0), ("cout", -1), ("h", 0), ("kh", 0), ("stride", 0), ("pad", -1),
                       ("kind", 7), ("in_dtype", 5), ("layout", 9)):
        d = dp.make_desc(conv(8, 8, 3, 1, 8, bias=True), 4)
        setattr(d, field, val)
        _raises(B.DP_ERR_INVALID_ARG, call, d)
    # channels-last inputs are read through a transposed copy in the workspace: both tensors more of it
    d = dp.make_desc(conv(8, 8, 3, 1, 8), 4)
    plain = dp.dp_workspace_bytes(d)
    d.layout = dp.DP_NHWC
    assert dp.dp_workspace_bytes(d) == plain + 2 * 4 * 8 * 8 * 8 * 4
    _raises(B.DP_ERR_WORKSPACE, call, d, wb=plain)
    d = dp.make_desc(dense(8, 4), 2)
    plain = dp.dp_workspace_bytes(d)
    d.layout = dp.DP_NHWC                                                 # a dense layer has no channel axis to move
    assert dp.dp_workspace_bytes(d) == plain
    d = dp.make_desc(conv(8, 8, 3, 1, 8), 4)
    d.kh = 20                                                             # kernel larger than padded input
    _raises(B.DP_ERR_INVALID_ARG, call, d)
    d = dp.make_desc(gn_affine(6, 4, 4), 2)                               # groups do not divide channels
    _raises(B.DP_ERR_INVALID_ARG, call, d)
    d = dp.make_desc(dense(8, 4), 2)
    d.w = 3
    _raises(B.DP_ERR_INVALID_ARG, call, d)


def test_streaming_calls_argument_errors(lib):
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_norms, None, FAKE, 2, 4, 1, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_norms, FAKE, FAKE, 0, 4, 1, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_norms, FAKE, FAKE, 2, 4, 0, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_factors, FAKE, 0.0, 4, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_factors, FAKE, float("nan"), 4, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_accumulate, FAKE, FAKE, -1.0, 4, 16, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_accumulate, FAKE, FAKE, 1.0, 0, 16, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_accumulate, FAKE, FAKE, 1.0, 4, 0, FAKE, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_accumulate, FAKE, FAKE, 1.0, 4, 16, FAKE, g_stride=8, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_accumulate, FAKE, FAKE, 1.0, 4, 16, None, stream=0)
    fin = lambda **k: dp.dp_add_noise_finalize(k.get("acc", FAKE), k.get("out", FAKE), k.get("p", 16),
                                               k.get("sigma", 1.0), k.get("c", 1.0), k.get("b", 8), 0, 0, 0, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, fin, acc=None)
    _raises(B.DP_ERR_INVALID_ARG, fin, out=FAKE + 8)
    _raises(B.DP_ERR_INVALID_ARG, fin, p=0)
    _raises(B.DP_ERR_INVALID_ARG, fin, sigma=-0.1)
    _raises(B.DP_ERR_INVALID_ARG, fin, sigma=float("nan"))
    _raises(B.DP_ERR_INVALID_ARG, fin, c=0.0)
    _raises(B.DP_ERR_INVALID_ARG, fin, c=math.inf)
    _raises(B.DP_ERR_INVALID_ARG, fin, b=0)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_philox_raw, None, 16, 0, 0, 0, stream=0)


def test_recompute_argument_errors(lib):
    d = dp.make_desc(conv(8, 8, 3, 1, 8, bias=True), 64)
    ws = dp.dp_workspace_bytes(d, dp.DP_WS_RECOMPUTE)
    assert ws > 0
    call = lambda sq=FAKE, c=1.0, aw=FAKE, ab=FAKE, w=FAKE, wb=ws: dp.dp_clip_accumulate_recompute(
        d, FAKE, FAKE, sq, c, aw, ab, w, ws_bytes=wb, stream=0)
    _raises(B.DP_ERR_INVALID_ARG, call, sq=None)
    _raises(B.DP_ERR_INVALID_ARG, call, c=0.0)
    _raises(B.DP_ERR_INVALID_ARG, call, aw=None)
    _raises(B.DP_ERR_INVALID_ARG, call, ab=None)          # bias layer
    _raises(B.DP_ERR_WORKSPACE, call, w=None)
    _raises(B.DP_ERR_WORKSPACE, call, wb=16)
    nb = dp.make_desc(conv(8, 8, 3, 1, 8), 4)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_clip_accumulate_recompute, nb, FAKE, FAKE, FAKE, 1.0, FAKE, FAKE, FAKE,
            ws_bytes=1 << 20, stream=0)                    # acc_b for a layer without bias


def test_profile_hook_accepts_null_events(lib):
    """The benchmark timing aid can be armed / cancelled without a GPU (no HIP call is made until
    a contraction is launched)."""
    assert B.load_library().dp_profile_next_contraction(None, None) == 0


def test_norms_from_partials_rejects_bad_tables(lib):
    import ctypes as C
    ok_ptrs = (C.c_void_p * 2)(FAKE, FAKE)
    ok_counts = (C.c_int32 * 2)(3, 1)
    ok_groups = (C.c_int32 * 2)(0, 0)
    f = lib.dp_norms_from_partials
    cast = lambda a: C.cast(a, C.c_void_p)
    assert f(None, cast(ok_counts), cast(ok_groups), 2, 4, 1, FAKE, None) == B.DP_ERR_INVALID_ARG
    assert f(cast(ok_ptrs), cast(ok_counts), cast(ok_groups), 0, 4, 1, FAKE, None) == B.DP_ERR_INVALID_ARG
    assert f(cast(ok_ptrs), cast(ok_counts), cast(ok_groups), 2, 4, 1, None, None) == B.DP_ERR_INVALID_ARG
    assert f(cast((C.c_void_p * 2)(FAKE, 0)), cast(ok_counts), cast(ok_groups), 2, 4, 1, FAKE, None) == B.DP_ERR_INVALID_ARG
    assert f(cast(ok_ptrs), cast((C.c_int32 * 2)(3, 0)), cast(ok_groups), 2, 4, 1, FAKE, None) == B.DP_ERR_INVALID_ARG
    assert f(cast(ok_ptrs), cast(ok_counts), cast((C.c_int32 * 2)(0, 1)), 2, 4, 1, FAKE, None) == B.DP_ERR_INVALID_ARG
    assert "group_of_layer" in dp.dp_last_error()


def test_norm_partial_count_is_positive_and_needs_a_valid_descriptor(lib):
    for layer in (conv(64, 64, 3, 1, 14), conv(3, 16, 3, 2, 9, bias=True), dense(20, 7), dense(20, 7, tokens=3), gn_affine(16, 8, 4)):
        for dtype in ("f32", "bf16"):
            d = dp.make_desc(layer, 5, dtype)
            for mat in (False, True):
                c = dp.dp_norm_partial_count(d, mat)
                assert c >= 1
                assert dp.dp_workspace_bytes(d, dp.DP_WS_PER_EXAMPLE_GRAD) >= 4 * 5 * c
    bad = dp.make_desc(conv(4, 4, 3, 1, 8), 0, "f32")
    assert dp.dp_norm_partial_count(bad, False) == 0


def test_fused_update_rejects_bad_arguments(lib):
    f = lib.dp_add_noise_finalize_update
    ok = dict(acc=FAKE, theta=FAKE, velocity=FAKE, out=None, p=16, sigma=1.0, clip=1.0, batch=8, seed=0, step=0, tid=0,
              lr=0.1, mom=0.9)
    def call(**kw):
        a = dict(ok, **kw)
        return f(a["acc"], a["theta"], a["velocity"], a["out"], a["p"], a["sigma"], a["clip"], a["batch"], a["seed"],
                 a["step"], a["tid"], a["lr"], a["mom"], None)
    assert call(acc=None) == B.DP_ERR_INVALID_ARG
    assert call(theta=None) == B.DP_ERR_INVALID_ARG
    assert call(theta=FAKE + 4) == B.DP_ERR_INVALID_ARG
    assert call(p=0) == B.DP_ERR_INVALID_ARG
    assert call(sigma=-1.0) == B.DP_ERR_INVALID_ARG
    assert call(clip=0.0) == B.DP_ERR_INVALID_ARG
    assert call(batch=0) == B.DP_ERR_INVALID_ARG
    assert call(lr=float("nan")) == B.DP_ERR_INVALID_ARG
    assert call(mom=-0.1) == B.DP_ERR_INVALID_ARG
    assert call(mom=float("inf")) == B.DP_ERR_INVALID_ARG
    assert call(velocity=None, mom=0.9) == B.DP_ERR_INVALID_ARG
    assert "velocity" in dp.dp_last_error()


def test_example_noise_rejects_bad_arguments(lib):
    f = lib.dp_add_example_noise
    def call(acc=FAKE, p=16, sigma=1.0, clip=1.0, batch=8, first=0, cnt=4):
        return f(acc, p, sigma, clip, batch, 0, 0, 0, first, cnt, None, None)
    assert call(acc=None) == B.DP_ERR_INVALID_ARG
    assert call(p=0) == B.DP_ERR_INVALID_ARG
    assert call(sigma=float("nan")) == B.DP_ERR_INVALID_ARG
    assert call(clip=-1.0) == B.DP_ERR_INVALID_ARG
    assert call(batch=0) == B.DP_ERR_INVALID_ARG
    assert call(cnt=0) == B.DP_ERR_INVALID_ARG
    assert call(first=6, cnt=4) == B.DP_ERR_INVALID_ARG          # examples beyond the step
    assert "outside" in dp.dp_last_error()


def test_infinite_bound_is_legal_only_without_noise(lib):
    """C = inf with sigma = 0 (plain mean gradient) is a legal finalize; with noise it has no meaning."""
    f = lib.dp_add_noise_finalize
    assert f(FAKE, FAKE, 16, 1.0, float("inf"), 8, 0, 0, 0, None) == B.DP_ERR_INVALID_ARG
    assert "clip_total" in dp.dp_last_error()


def test_clip_accumulate_segments_rejects_bad_tables(lib):
    import ctypes as C
    f = lib.dp_clip_accumulate_segments
    def call(begins=(0, 8), groups=(0, 1), clips=(1.0, 1.0), n_groups=2, n=4, p=16, g=FAKE, acc=FAKE, sq=FAKE):
        k = len(begins)
        return f(g, 0, sq, n_groups, C.cast((C.c_size_t * k)(*begins), C.c_void_p), C.cast((C.c_int32 * k)(*groups), C.c_void_p),
                 C.cast((C.c_float * k)(*clips), C.c_void_p), k, n, p, acc, None)
    assert call(g=None) == B.DP_ERR_INVALID_ARG
    assert call(p=18) == B.DP_ERR_INVALID_ARG                    # not a multiple of 4
    assert call(begins=(4, 8)) == B.DP_ERR_INVALID_ARG           # must start at 0
    assert call(begins=(0, 6)) == B.DP_ERR_INVALID_ARG           # not a multiple of 4
    assert call(begins=(0, 16)) == B.DP_ERR_INVALID_ARG          # empty last segment
    assert call(groups=(0, 2)) == B.DP_ERR_INVALID_ARG           # group out of range
    assert call(clips=(1.0, 0.0)) == B.DP_ERR_INVALID_ARG
    assert call(n=0) == B.DP_ERR_INVALID_ARG


def test_group_clip_bounds_follow_section_3_5(lib):
    """M groups -> C / sqrt(M) each; the bound on the whole gradient (the noise scale) stays C.  Literal values:
    these are the library's own numbers, not the oracle's."""
    gc, tot = dp.dp_group_clip_bounds(1.0, 54)
    assert len(gc) == 54 and all(abs(c - 0.13608276348795434) < 1e-8 for c in gc)
    assert abs(tot - 1.0) < 1e-6
    gc, tot = dp.dp_group_clip_bounds(1.5, 1)
    assert gc == [1.5] and tot == 1.5
    gc, tot = dp.dp_group_clip_bounds(0.3, 4)
    assert all(abs(c - 0.15) < 1e-8 for c in gc) and abs(tot - 0.3) < 1e-7
    gc, tot = dp.dp_group_clip_bounds(math.inf, 3)
    assert all(math.isinf(c) for c in gc) and math.isinf(tot)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_group_clip_bounds, 0.0, 4)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_group_clip_bounds, float("nan"), 4)
    _raises(B.DP_ERR_INVALID_ARG, dp.dp_group_clip_bounds, 1.0, 0)
    assert lib.dp_group_clip_bounds(1.0, 2, None, None) == B.DP_ERR_INVALID_ARG


def test_flat_finalize_rejects_bad_tables(lib):
    import ctypes as C
    f = lib.dp_add_noise_finalize_flat
    def call(begins=(0, 8), sizes=(8, 5), ids=(0, 1), acc=FAKE, out=FAKE, theta=None, vel=None, sigma=1.0, clip=1.0,
             batch=4, lr=0.1, mom=0.0, step_dev=None):
        k = len(begins)
        return f(acc, out, theta, vel, C.cast((C.c_uint64 * k)(*begins), C.c_void_p), C.cast((C.c_uint64 * k)(*sizes), C.c_void_p),
                 C.cast((C.c_uint32 * k)(*ids), C.c_void_p), k, sigma, clip, batch, 0, 0, step_dev, lr, mom, None)
    assert call(acc=None) == B.DP_ERR_INVALID_ARG
    assert call(out=None) == B.DP_ERR_INVALID_ARG                 # no output and no theta: nothing to write
    assert call(begins=(0, 6)) == B.DP_ERR_INVALID_ARG            # not a multiple of 4
    assert call(begins=(0, 4)) == B.DP_ERR_INVALID_ARG            # overlaps the first tensor
    assert call(sizes=(8, 0)) == B.DP_ERR_INVALID_ARG
    assert call(sizes=(8, 1 << 32)) == B.DP_ERR_UNSUPPORTED
    assert call(sigma=-1.0) == B.DP_ERR_INVALID_ARG
    assert call(clip=float("inf")) == B.DP_ERR_INVALID_ARG
    assert call(batch=0) == B.DP_ERR_INVALID_ARG
    assert call(vel=FAKE) == B.DP_ERR_INVALID_ARG                 # velocity without theta
    assert call(theta=FAKE, mom=0.9) == B.DP_ERR_INVALID_ARG      # momentum without a velocity buffer
    assert call(theta=FAKE, lr=float("nan")) == B.DP_ERR_INVALID_ARG
    assert call(step_dev=FAKE + 4) == B.DP_ERR_INVALID_ARG        # 8-byte alignment
    assert lib.dp_add_noise_finalize_flat(FAKE, FAKE, None, None, None, None, None, 1, 1.0, 1.0, 4, 0, 0, None, 0.0, 0.0, None) == B.DP_ERR_INVALID_ARG
