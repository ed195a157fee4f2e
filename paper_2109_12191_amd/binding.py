"""ctypes binding of libdp_privatise.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

DP_OK, DP_ERR_INVALID_ARG, DP_ERR_UNSUPPORTED, DP_ERR_WORKSPACE, DP_ERR_DEVICE = range(5)
DP_DENSE, DP_CONV2D, DP_GN_AFFINE = 0, 1, 2
DP_F32, DP_BF16 = 0, 1
DP_NCHW, DP_NHWC = 0, 1
DP_WS_PER_EXAMPLE_GRAD, DP_WS_RECOMPUTE = 0, 1
DP_VARIANT_SHARED = 2
DP_VARIANT_MATERIALISE = 4

_STATUS_NAMES = {1: "DP_ERR_INVALID_ARG", 2: "DP_ERR_UNSUPPORTED", 3: "DP_ERR_WORKSPACE", 4: "DP_ERR_DEVICE"}
_KINDS = {"dense": DP_DENSE, "conv": DP_CONV2D, "gn": DP_GN_AFFINE}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdp_privatise.so")
_lib = None


class DpError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class LayerDesc(C.Structure):
    """Mirror of dp_layer_desc."""
    _fields_ = [("kind", C.c_int), ("in_dtype", C.c_int), ("layout", C.c_int), ("n", C.c_int),
                ("cin", C.c_int), ("cout", C.c_int), ("h", C.c_int), ("w", C.c_int),
                ("kh", C.c_int), ("kw", C.c_int), ("stride", C.c_int), ("pad", C.c_int),
                ("has_bias", C.c_int), ("gn_groups", C.c_int), ("gn_eps", C.c_float)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the HIP library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2109_12191_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(_LIB_PATH)
    vp, sz, u64, u32, fl, it = C.c_void_p, C.c_size_t, C.c_uint64, C.c_uint32, C.c_float, C.c_int
    dpp = C.POINTER(LayerDesc)
    sigs = {
        "dp_group_clip_bounds": (it, [fl, it, vp, vp]),
        "dp_weight_count": (sz, [dpp]),
        "dp_bias_count": (sz, [dpp]),
        "dp_workspace_bytes": (sz, [dpp, it]),
        "dp_kernel_variant": (C.c_char_p, [dpp, it]),
        "dp_per_example_grad": (it, [dpp, vp, vp, vp, vp, sz, vp, vp, sz, vp]),
        "dp_static_scratch_bytes": (sz, []),
        "dp_per_example_grad_static": (it, [dpp, vp, vp, vp, vp, sz, vp, vp]),
        "dp_norms": (it, [vp, vp, it, it, it, vp, vp]),
        "dp_norm_partial_count": (sz, [dpp, it]),
        "dp_unit_workspace_bytes": (sz, [dpp, it]),
        "dp_unit_grad": (it, [dpp, it, vp, vp, vp, vp, sz, vp, vp, sz, vp]),
        "dp_unit_grad_batch": (it, [vp, it, vp, vp, vp, vp, sz, vp, vp, vp, it, vp]),
        "dp_per_example_grad_partials": (it, [dpp, vp, vp, vp, vp, sz, vp, sz, vp]),
        "dp_norms_from_partials": (it, [vp, vp, vp, it, it, it, vp, vp]),
        "dp_per_example_grad_batch": (it, [vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, it, vp]),
        "dp_layer_norms_from_partials": (it, [vp, vp, vp, it, it, vp]),
        "dp_clip_accumulate_recompute_batch": (it, [vp, vp, vp, vp, vp, vp, vp, vp, vp, it, vp]),
        "dp_clip_factors": (it, [vp, fl, it, vp, vp]),
        "dp_clip_accumulate": (it, [vp, sz, vp, fl, it, sz, vp, vp]),
        "dp_clip_accumulate_segments": (it, [vp, sz, vp, it, vp, vp, vp, it, it, sz, vp, vp]),
        "dp_clip_accumulate_recompute": (it, [dpp, vp, vp, vp, fl, vp, vp, vp, sz, vp]),
        "dp_add_noise_finalize": (it, [vp, vp, sz, fl, fl, u64, u64, u64, u32, vp]),
        "dp_add_example_noise": (it, [vp, sz, fl, fl, u64, u64, u64, u32, u64, it, vp, vp]),
        "dp_add_noise_finalize_update": (it, [vp, vp, vp, vp, sz, fl, fl, u64, u64, u64, u32, fl, fl, vp]),
        "dp_add_noise_finalize_flat": (it, [vp, vp, vp, vp, vp, vp, vp, it, fl, fl, u64, u64, u64, vp, fl, fl, vp]),
        "dp_philox_raw": (it, [vp, sz, u64, u64, u32, vp]),
        "dp_profile_next_contraction": (it, [vp, vp]),
        "dp_last_error": (C.c_char_p, []),
        "dp_version": (C.c_char_p, []),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


EXPORTED = ("dp_group_clip_bounds", "dp_weight_count", "dp_bias_count", "dp_workspace_bytes", "dp_kernel_variant", "dp_per_example_grad", "dp_norms",
            "dp_static_scratch_bytes", "dp_per_example_grad_static",
            "dp_unit_workspace_bytes", "dp_unit_grad", "dp_unit_grad_batch",
            "dp_norm_partial_count", "dp_per_example_grad_partials", "dp_norms_from_partials",
            "dp_per_example_grad_batch", "dp_layer_norms_from_partials", "dp_clip_accumulate_recompute_batch",
            "dp_clip_factors", "dp_clip_accumulate", "dp_clip_accumulate_segments", "dp_clip_accumulate_recompute", "dp_add_noise_finalize", "dp_add_noise_finalize_update", "dp_add_example_noise",
            "dp_add_noise_finalize_flat", "dp_philox_raw", "dp_profile_next_contraction", "dp_last_error", "dp_version")


def make_desc(layer, n: int, dtype: str = "f32", layout: int = DP_NCHW) -> LayerDesc:
    """dp_layer_desc from a workload layer (anything with kind/cin/cout/h/w/kh/kw/stride/pad/...)."""
    return LayerDesc(_KINDS[layer.kind], DP_BF16 if dtype == "bf16" else DP_F32, layout, n,
                     layer.cin, layer.cout, layer.h, layer.w, layer.kh, layer.kw, layer.stride, layer.pad,
                     int(bool(layer.has_bias)), layer.gn_groups, float(layer.gn_eps))


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(status: int):
    if status != DP_OK:
        raise DpError(status, dp_last_error())


def dp_last_error() -> str:
    return load_library().dp_last_error().decode()


def dp_version() -> str:
    return load_library().dp_version().decode()


def dp_group_clip_bounds(clip_c: float, n_groups: int):
    """(list of per-group bounds, bound on the whole clipped gradient), both computed by the library."""
    gc = (C.c_float * max(n_groups, 1))()
    tot = C.c_float()
    _check(load_library().dp_group_clip_bounds(clip_c, n_groups, C.cast(gc, C.c_void_p), C.cast(C.byref(tot), C.c_void_p)))
    return [float(v) for v in gc], float(tot.value)


def dp_weight_count(desc: LayerDesc) -> int:
    return int(load_library().dp_weight_count(C.byref(desc)))


def dp_bias_count(desc: LayerDesc) -> int:
    return int(load_library().dp_bias_count(C.byref(desc)))


def dp_workspace_bytes(desc: LayerDesc, use: int = DP_WS_PER_EXAMPLE_GRAD) -> int:
    return int(load_library().dp_workspace_bytes(C.byref(desc), use))


def dp_kernel_variant(desc: LayerDesc, use: int = DP_WS_PER_EXAMPLE_GRAD) -> str:
    return load_library().dp_kernel_variant(C.byref(desc), use).decode()


def dp_per_example_grad(desc, x, dy, g_w, g_b, sqnorm, ws, g_stride: int = 0, ws_bytes: Optional[int] = None,
                        stream=None):
    _check(load_library().dp_per_example_grad(C.byref(desc), _ptr(x), _ptr(dy), _ptr(g_w), _ptr(g_b), g_stride,
                                              _ptr(sqnorm), _ptr(ws),
                                              _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream)))


def dp_static_scratch_bytes() -> int:
    return int(load_library().dp_static_scratch_bytes())


def dp_per_example_grad_static(desc, x, dy, g_w, g_b, sqnorm, g_stride: int = 0, stream=None):
    _check(load_library().dp_per_example_grad_static(C.byref(desc), _ptr(x), _ptr(dy), _ptr(g_w), _ptr(g_b), g_stride,
                                                     _ptr(sqnorm), _stream(stream)))


def dp_norm_partial_count(desc, materialise: bool) -> int:
    return int(load_library().dp_norm_partial_count(C.byref(desc), 1 if materialise else 0))


def dp_per_example_grad_partials(desc, x, dy, g_w, g_b, ws, g_stride: int = 0, ws_bytes: Optional[int] = None,
                                 stream=None):
    _check(load_library().dp_per_example_grad_partials(C.byref(desc), _ptr(x), _ptr(dy), _ptr(g_w), _ptr(g_b),
                                                       g_stride, _ptr(ws),
                                                       _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream)))


class PartialTable:
    """Host arrays for dp_norms_from_partials, built once: device pointers of every layer's partial
    sums (the start of its workspace), their per-example counts and the layer -> group map."""

    def __init__(self, pointers, counts, groups):
        n = len(pointers)
        self.n_layers = n
        self.ptrs = (C.c_void_p * n)(*[int(p) for p in pointers])
        self.counts = (C.c_int32 * n)(*[int(c) for c in counts])
        self.groups = (C.c_int32 * n)(*[int(g) for g in groups])


def dp_norms_from_partials(table: "PartialTable", n: int, n_groups: int, group_sqnorm, stream=None):
    _check(load_library().dp_norms_from_partials(C.cast(table.ptrs, C.c_void_p), C.cast(table.counts, C.c_void_p),
                                                 C.cast(table.groups, C.c_void_p), table.n_layers, n, n_groups,
                                                 _ptr(group_sqnorm), _stream(stream)))


def dp_unit_workspace_bytes(desc: LayerDesc, clip_unit: int) -> int:
    return int(load_library().dp_unit_workspace_bytes(C.byref(desc), clip_unit))


def dp_unit_grad(desc: LayerDesc, clip_unit: int, x, dy, g_w, g_b, sqnorm, ws, g_stride: int = 0, stream=None):
    """Sums of the per-example gradients over clipping units of clip_unit consecutive examples, and the squared
    norms of the sums ([n / clip_unit])."""
    _check(load_library().dp_unit_grad(C.byref(desc), clip_unit, _ptr(x), _ptr(dy), _ptr(g_w), _ptr(g_b), g_stride,
                                       _ptr(sqnorm), _ptr(ws), _nbytes(ws), _stream(stream)))


class LayerBatch:
    """Host arrays for the batch calls over a fixed set of layers: descriptors, workspaces, and (re)settable
    pointer arrays.  Pointers are plain integers (device addresses); None becomes NULL."""

    def __init__(self, descs, ws_ptrs, ws_bytes):
        k = len(descs)
        self.n_layers = k
        self.descs = (LayerDesc * k)(*descs)
        self.ws = (C.c_void_p * k)(*[int(p) for p in ws_ptrs])
        self.ws_bytes = (C.c_size_t * k)(*[int(b) for b in ws_bytes])
        self.partial_counts = (C.c_int32 * k)()          # written by dp_per_example_grad_batch

    def ptrs(self, values):
        assert len(values) == self.n_layers
        return (C.c_void_p * self.n_layers)(*[(None if v is None else int(v)) for v in values])

    def floats(self, values):
        assert len(values) == self.n_layers
        return (C.c_float * self.n_layers)(*[float(v) for v in values])


def dp_per_example_grad_batch(batch: "LayerBatch", x, dy, g_w, g_b, sqnorm, g_stride: int = 0, stream=None):
    """x, dy: ctypes pointer arrays from batch.ptrs(); g_w, g_b, sqnorm: the same or None (sqnorm None: the
    per-layer reduction is left to dp_layer_norms_from_partials).  batch.partial_counts receives the number of
    partial sums per example each layer left at the start of its workspace."""
    _check(load_library().dp_per_example_grad_batch(C.cast(batch.descs, C.c_void_p), C.cast(x, C.c_void_p),
                                                    C.cast(dy, C.c_void_p),
                                                    None if g_w is None else C.cast(g_w, C.c_void_p),
                                                    None if g_b is None else C.cast(g_b, C.c_void_p), g_stride,
                                                    None if sqnorm is None else C.cast(sqnorm, C.c_void_p),
                                                    C.cast(batch.ws, C.c_void_p), C.cast(batch.ws_bytes, C.c_void_p),
                                                    C.cast(batch.partial_counts, C.c_void_p), batch.n_layers,
                                                    _stream(stream)))


def dp_unit_grad_batch(batch: "LayerBatch", clip_unit: int, x, dy, g_w, g_b, sqnorm, g_stride: int = 0, stream=None):
    """dp_unit_grad for the layers of a LayerBatch; x, dy, sqnorm: ctypes pointer arrays from batch.ptrs()."""
    _check(load_library().dp_unit_grad_batch(C.cast(batch.descs, C.c_void_p), clip_unit, C.cast(x, C.c_void_p),
                                             C.cast(dy, C.c_void_p),
                                             None if g_w is None else C.cast(g_w, C.c_void_p),
                                             None if g_b is None else C.cast(g_b, C.c_void_p), g_stride,
                                             C.cast(sqnorm, C.c_void_p), C.cast(batch.ws, C.c_void_p),
                                             C.cast(batch.ws_bytes, C.c_void_p), batch.n_layers, _stream(stream)))


def dp_layer_norms_from_partials(partials, counts, sqnorm, n_layers: int, n: int, stream=None):
    """partials, sqnorm: ctypes arrays of n_layers device pointers; counts: ctypes int32 array."""
    _check(load_library().dp_layer_norms_from_partials(C.cast(partials, C.c_void_p), C.cast(counts, C.c_void_p),
                                                       C.cast(sqnorm, C.c_void_p), n_layers, n, _stream(stream)))


def dp_clip_accumulate_recompute_batch(batch: "LayerBatch", x, dy, sqnorm, clip_c, acc_w, acc_b, stream=None):
    _check(load_library().dp_clip_accumulate_recompute_batch(C.cast(batch.descs, C.c_void_p), C.cast(x, C.c_void_p),
                                                             C.cast(dy, C.c_void_p), C.cast(sqnorm, C.c_void_p),
                                                             C.cast(clip_c, C.c_void_p), C.cast(acc_w, C.c_void_p),
                                                             None if acc_b is None else C.cast(acc_b, C.c_void_p),
                                                             C.cast(batch.ws, C.c_void_p), C.cast(batch.ws_bytes, C.c_void_p),
                                                             batch.n_layers, _stream(stream)))


def dp_norms(layer_sqnorm, group_of_layer, n_layers: int, n: int, n_groups: int, group_sqnorm, stream=None):
    _check(load_library().dp_norms(_ptr(layer_sqnorm), _ptr(group_of_layer), n_layers, n, n_groups,
                                   _ptr(group_sqnorm), _stream(stream)))


def dp_clip_factors(sqnorm, clip_c: float, n: int, f, stream=None):
    _check(load_library().dp_clip_factors(_ptr(sqnorm), clip_c, n, _ptr(f), _stream(stream)))


def dp_clip_accumulate(g, sqnorm, clip_c: float, n: int, p: int, acc, g_stride: int = 0, stream=None):
    _check(load_library().dp_clip_accumulate(_ptr(g), g_stride, _ptr(sqnorm), clip_c, n, p, _ptr(acc),
                                             _stream(stream)))


class SegmentTable:
    """Host arrays for dp_clip_accumulate_segments: column where each segment starts, its clipping group and bound."""

    def __init__(self, begins, groups, clips):
        k = len(begins)
        self.n_seg = k
        self.begin = (C.c_size_t * k)(*[int(b) for b in begins])
        self.group = (C.c_int32 * k)(*[int(g) for g in groups])
        self.clip = (C.c_float * k)(*[float(c) for c in clips])


def dp_clip_accumulate_segments(g, group_sqnorm, n_groups: int, table: "SegmentTable", n: int, p: int, acc,
                                g_stride: int = 0, stream=None):
    _check(load_library().dp_clip_accumulate_segments(_ptr(g), g_stride, _ptr(group_sqnorm), n_groups,
                                                      C.cast(table.begin, C.c_void_p), C.cast(table.group, C.c_void_p),
                                                      C.cast(table.clip, C.c_void_p), table.n_seg, n, p, _ptr(acc),
                                                      _stream(stream)))


def dp_clip_accumulate_recompute(desc, x, dy, sqnorm, clip_c: float, acc_w, acc_b, ws,
                                 ws_bytes: Optional[int] = None, stream=None):
    _check(load_library().dp_clip_accumulate_recompute(C.byref(desc), _ptr(x), _ptr(dy), _ptr(sqnorm), clip_c,
                                                       _ptr(acc_w), _ptr(acc_b), _ptr(ws),
                                                       _nbytes(ws) if ws_bytes is None else ws_bytes,
                                                       _stream(stream)))


def dp_add_noise_finalize(acc, out, p: int, sigma: float, clip_total: float, total_batch: int, seed: int,
                          step: int, tensor_id: int, stream=None):
    _check(load_library().dp_add_noise_finalize(_ptr(acc), _ptr(out), p, sigma, clip_total, total_batch, seed,
                                                step, tensor_id, _stream(stream)))


def dp_add_example_noise(acc, p: int, sigma: float, clip_total: float, total_batch: int, seed: int, step: int,
                         tensor_id: int, first_example: int, n_examples: int, step_dev=None, stream=None):
    _check(load_library().dp_add_example_noise(_ptr(acc), p, sigma, clip_total, total_batch, seed, step, tensor_id,
                                               first_example, n_examples, _ptr(step_dev), _stream(stream)))


def dp_add_noise_finalize_update(acc, theta, velocity, out, p: int, sigma: float, clip_total: float, total_batch: int,
                                 seed: int, step: int, tensor_id: int, lr: float, momentum: float, stream=None):
    _check(load_library().dp_add_noise_finalize_update(_ptr(acc), _ptr(theta), _ptr(velocity), _ptr(out), p, sigma,
                                                       clip_total, total_batch, seed, step, tensor_id, lr, momentum,
                                                       _stream(stream)))


class TensorTable:
    """Host arrays for dp_add_noise_finalize_flat: where each tensor starts in the flat parameter vector,
    its size and its Philox tensor id."""

    def __init__(self, begins, sizes, tensor_ids):
        k = len(begins)
        self.n_seg = k
        self.begin = (C.c_uint64 * k)(*[int(b) for b in begins])
        self.size = (C.c_uint64 * k)(*[int(v) for v in sizes])
        self.tensor_id = (C.c_uint32 * k)(*[int(t) for t in tensor_ids])


def dp_add_noise_finalize_flat(acc, out, table: "TensorTable", sigma: float, clip_total: float, total_batch: int,
                               seed: int, step: int = 0, step_dev=None, theta=None, velocity=None, lr: float = 0.0,
                               momentum: float = 0.0, stream=None):
    _check(load_library().dp_add_noise_finalize_flat(_ptr(acc), _ptr(out), _ptr(theta), _ptr(velocity),
                                                     C.cast(table.begin, C.c_void_p), C.cast(table.size, C.c_void_p),
                                                     C.cast(table.tensor_id, C.c_void_p), table.n_seg, sigma, clip_total,
                                                     total_batch, seed, step, _ptr(step_dev), lr, momentum,
                                                     _stream(stream)))


def dp_profile_next_contraction(start_event, stop_event):
    """Arm (or, with None, cancel) event bracketing of the next contraction kernel.  The arguments are
    torch.cuda.Event objects that have been recorded once (that creates their HIP handles)."""
    a = start_event.cuda_event if start_event is not None else None
    b = stop_event.cuda_event if stop_event is not None else None
    _check(load_library().dp_profile_next_contraction(a, b))


def dp_philox_raw(raw, p: int, seed: int, step: int, tensor_id: int, stream=None):
    _check(load_library().dp_philox_raw(_ptr(raw), p, seed, step, tensor_id, _stream(stream)))
