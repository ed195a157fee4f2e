"""ctypes front-end of the fp64 CPU oracle (TEST INFRASTRUCTURE, not part of the product).

Only tests, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import
this package.  It never touches the HIP library and the HIP library never touches it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdp_oracle.so")
_SRC = os.path.join(_HERE, "dp_oracle.c")
_lib = None

_KIND = {"dense": 0, "conv": 1, "gn": 2}


class _Layer(C.Structure):
    _fields_ = [("kind", C.c_int), ("cin", C.c_int), ("cout", C.c_int), ("h", C.c_int), ("w", C.c_int),
                ("kh", C.c_int), ("kw", C.c_int), ("stride", C.c_int), ("pad", C.c_int),
                ("has_bias", C.c_int), ("gn_groups", C.c_int), ("gn_eps", C.c_double), ("group", C.c_int)]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "dp_oracle.h"))):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = C.CDLL(_SO)
    dp, fp = C.POINTER(C.c_double), C.POINTER(C.c_float)
    lp = C.POINTER(_Layer)
    lib.orc_weight_grad_elem.restype = C.c_double
    lib.orc_weight_grad_elem.argtypes = [lp, fp, fp, C.c_size_t]
    lib.orc_bias_grad_elem.restype = C.c_double
    lib.orc_bias_grad_elem.argtypes = [lp, fp, fp, C.c_size_t]
    lib.orc_example_grad.restype = None
    lib.orc_example_grad.argtypes = [lp, fp, fp, dp, dp]
    lib.orc_sqnorm.restype = C.c_double
    lib.orc_sqnorm.argtypes = [dp, C.c_size_t]
    lib.orc_clip_factor.restype = C.c_double
    lib.orc_clip_factor.argtypes = [C.c_double, C.c_double]
    lib.orc_group_bounds.restype = None
    lib.orc_group_bounds.argtypes = [C.c_double, C.c_int, dp, dp]
    lib.orc_clip_accumulate.restype = C.c_int
    lib.orc_clip_accumulate.argtypes = [lp, C.c_int, C.POINTER(fp), C.POINTER(fp), C.c_int, C.c_int, dp,
                                        C.POINTER(dp), C.POINTER(dp), dp, dp, C.c_int]
    lib.orc_clip_accumulate_units.restype = C.c_int
    lib.orc_clip_accumulate_units.argtypes = [lp, C.c_int, C.POINTER(fp), C.POINTER(fp), C.c_int, C.c_int, C.c_int, dp,
                                              C.POINTER(dp), C.POINTER(dp), dp, dp, C.c_int]
    lib.orc_weighted_sum_elems.restype = None
    lib.orc_weighted_sum_elems.argtypes = [lp, fp, fp, C.c_int, dp, C.POINTER(C.c_size_t), C.c_size_t,
                                           C.c_int, dp]
    lib.orc_philox4x32_10.restype = None
    lib.orc_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
    lib.orc_noise_raw.restype = None
    lib.orc_noise_raw.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_size_t, C.c_size_t,
                                  C.POINTER(C.c_uint32)]
    lib.orc_noise_normal.restype = None
    lib.orc_noise_normal.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_size_t, C.c_size_t, dp]
    lib.orc_noise_finalize.restype = None
    lib.orc_noise_finalize.argtypes = [dp, dp, C.c_size_t, C.c_double, C.c_double, C.c_uint64, C.c_uint64,
                                       C.c_uint64, C.c_uint32]
    lib.orc_add_example_noise.restype = None
    lib.orc_add_example_noise.argtypes = [dp, C.c_size_t, C.c_double, C.c_double, C.c_uint64, C.c_uint64, C.c_uint64,
                                          C.c_uint32, C.c_uint64, C.c_int]
    lib.orc_sgd_update.restype = None
    lib.orc_sgd_update.argtypes = [dp, dp, dp, C.c_size_t, C.c_double, C.c_double]
    lib.orc_max_threads.restype = C.c_int
    for name in ("orc_x_elems", "orc_dy_elems", "orc_w_elems", "orc_b_elems"):
        getattr(lib, name).restype = C.c_size_t
        getattr(lib, name).argtypes = [lp]
    _lib = lib
    return lib


def _c_layer(layer, group: int = 0) -> _Layer:
    return _Layer(_KIND[layer.kind], layer.cin, layer.cout, layer.h, layer.w, layer.kh, layer.kw,
                  layer.stride, layer.pad, int(bool(layer.has_bias)), layer.gn_groups,
                  float(layer.gn_eps), group)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _fp(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _dp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_double))


def max_threads() -> int:
    return int(_load().orc_max_threads())


def example_grad(layer, x, dy):
    """Per-example gradient of one layer for ONE example: (gw, gb) fp64, gb None without bias."""
    lib = _load()
    cl = _c_layer(layer)
    x, dy = _f32(x), _f32(dy)
    assert x.size == lib.orc_x_elems(C.byref(cl)) and dy.size == lib.orc_dy_elems(C.byref(cl))
    gw = np.empty(layer.pw, dtype=np.float64)
    gb = np.empty(layer.pb, dtype=np.float64) if layer.pb else None
    lib.orc_example_grad(C.byref(cl), _fp(x), _fp(dy), _dp(gw), _dp(gb))
    return gw.reshape(layer.w_shape), gb


def grad_elem(layer, x, dy, e: int, bias: bool = False) -> float:
    lib = _load()
    cl = _c_layer(layer)
    x, dy = _f32(x), _f32(dy)
    fn = lib.orc_bias_grad_elem if bias else lib.orc_weight_grad_elem
    return float(fn(C.byref(cl), _fp(x), _fp(dy), e))


def sqnorm(g) -> float:
    g = np.ascontiguousarray(g, dtype=np.float64)
    return float(_load().orc_sqnorm(_dp(g), g.size))


def clip_factor(n2: float, clip_c: float) -> float:
    return float(_load().orc_clip_factor(float(n2), float(clip_c)))


def group_bounds(clip_c: float, n_groups: int):
    """(per-group bounds C / sqrt(M), bound on the whole clipped gradient) for M clipping groups (Section 3.5)."""
    gc = np.empty(n_groups, dtype=np.float64)
    tot = np.empty(1, dtype=np.float64)
    _load().orc_group_bounds(float(clip_c), int(n_groups), _dp(gc), _dp(tot))
    return [float(c) for c in gc], float(tot[0])


def new_accumulators(layers):
    acc_w = [np.zeros(l.pw, dtype=np.float64) for l in layers]
    acc_b = [np.zeros(l.pb, dtype=np.float64) if l.pb else None for l in layers]
    return acc_w, acc_b


def clip_accumulate(layers, inputs, group_of_layer: Sequence[int], group_clip: Sequence[float],
                    acc_w: List[np.ndarray], acc_b: List[Optional[np.ndarray]], threads: int = 0):
    """One micro-step: adds sum_i clip(g_i) into acc_w / acc_b (fp64, in place).
    inputs: list over layers of (x [n,...], dy [n,...]).  Returns (n2 [n,G], f [n,G])."""
    lib = _load()
    nl = len(layers)
    n = int(inputs[0][0].shape[0])
    ng = len(group_clip)
    arr = (_Layer * nl)(*[_c_layer(l, g) for l, g in zip(layers, group_of_layer)])
    xs = [_f32(x) for x, _ in inputs]
    dys = [_f32(dy) for _, dy in inputs]
    fpp = C.POINTER(C.c_float)
    dpp = C.POINTER(C.c_double)
    xp = (fpp * nl)(*[_fp(a) for a in xs])
    dyp = (fpp * nl)(*[_fp(a) for a in dys])
    awp = (dpp * nl)(*[_dp(a) for a in acc_w])
    abp = (dpp * nl)(*[(_dp(a) if a is not None else C.cast(None, dpp)) for a in acc_b])
    gc = np.asarray(group_clip, dtype=np.float64)
    n2 = np.empty((n, ng), dtype=np.float64)
    f = np.empty((n, ng), dtype=np.float64)
    rc = lib.orc_clip_accumulate(arr, nl, xp, dyp, n, ng, _dp(gc), awp, abp, _dp(n2), _dp(f), threads)
    if rc != 0:
        raise RuntimeError("orc_clip_accumulate failed")
    return n2, f


def clip_accumulate_units(layers, inputs, unit: int, group_of_layer: Sequence[int], group_clip: Sequence[float],
                          acc_w: List[np.ndarray], acc_b: List[Optional[np.ndarray]], threads: int = 0):
    """One micro-step with clipping units of `unit` consecutive examples (the micro-batching of the GPU baseline,
    Abstract and Table 1): adds sum_u clip(mean of unit u's gradients) into acc_w / acc_b.
    Returns (n2 [n/unit, G], f [n/unit, G])."""
    lib = _load()
    nl = len(layers)
    n = int(inputs[0][0].shape[0])
    ng = len(group_clip)
    arr = (_Layer * nl)(*[_c_layer(l, g) for l, g in zip(layers, group_of_layer)])
    xs = [_f32(x) for x, _ in inputs]
    dys = [_f32(dy) for _, dy in inputs]
    fpp = C.POINTER(C.c_float)
    dpp = C.POINTER(C.c_double)
    xp = (fpp * nl)(*[_fp(a) for a in xs])
    dyp = (fpp * nl)(*[_fp(a) for a in dys])
    awp = (dpp * nl)(*[_dp(a) for a in acc_w])
    abp = (dpp * nl)(*[(_dp(a) if a is not None else C.cast(None, dpp)) for a in acc_b])
    gc = np.asarray(group_clip, dtype=np.float64)
    if unit < 1 or n % unit:
        raise ValueError("n must be a multiple of the clipping unit")
    n2 = np.empty((n // unit, ng), dtype=np.float64)
    f = np.empty((n // unit, ng), dtype=np.float64)
    rc = lib.orc_clip_accumulate_units(arr, nl, xp, dyp, n, int(unit), ng, _dp(gc), awp, abp, _dp(n2), _dp(f), threads)
    if rc != 0:
        raise RuntimeError("orc_clip_accumulate_units failed")
    return n2, f


def unit_mean_grad(layer, x, dy, unit: int):
    """Mean of the per-example gradients of each clipping unit: ([n/unit, pw], [n/unit, pb] or None)."""
    n = int(x.shape[0])
    rows_w, rows_b = [], []
    for u in range(n // unit):
        gs = [example_grad(layer, x[i], dy[i]) for i in range(u * unit, (u + 1) * unit)]
        rows_w.append(sum(g[0] for g in gs) / unit)
        rows_b.append(sum(g[1] for g in gs) / unit if layer.pb else None)
    return np.stack(rows_w).reshape(n // unit, -1), (np.stack(rows_b) if layer.pb else None)


def privatise_units(wl, inputs_per_micro_step, unit: int, threads: int = 0):
    """Whole optimiser step with clipping units of `unit` examples: sum over units of the clipped unit means, noise
    N(0, sigma^2 C^2) once, divided by the NUMBER OF UNITS in the step (each unit is one clipped contribution of
    norm at most C, as an example is in Section 2's first equation).  Same tensor ids as privatise()."""
    layers = list(wl.layers)
    group_clip, clip_total = group_bounds(wl.clip_c, wl.n_groups)
    acc_w, acc_b = new_accumulators(layers)
    n2s, fs = [], []
    for inputs in inputs_per_micro_step:
        n2, f = clip_accumulate_units(layers, inputs, unit, wl.group_of_layer, group_clip, acc_w, acc_b, threads)
        n2s.append(n2)
        fs.append(f)
    n_units = wl.total_batch // unit
    out_w, out_b = [], []
    for li, l in enumerate(layers):
        out_w.append(noise_finalize(acc_w[li], wl.sigma, clip_total, n_units, wl.philox_seed, wl.step, 2 * li))
        out_b.append(noise_finalize(acc_b[li], wl.sigma, clip_total, n_units, wl.philox_seed, wl.step, 2 * li + 1)
                     if acc_b[li] is not None else None)
    return dict(acc_w=acc_w, acc_b=acc_b, out_w=out_w, out_b=out_b, n2=n2s, f=fs)


def weighted_sum_elems(layer, x, dy, f, idx, bias: bool = False) -> np.ndarray:
    """sum_i f[i] * g_i[e] for the flat parameter indices in idx."""
    lib = _load()
    cl = _c_layer(layer)
    x, dy = _f32(x), _f32(dy)
    f = np.ascontiguousarray(f, dtype=np.float64)
    idx = np.ascontiguousarray(idx, dtype=np.uint64)
    out = np.empty(idx.size, dtype=np.float64)
    lib.orc_weighted_sum_elems(C.byref(cl), _fp(x), _fp(dy), int(x.shape[0]), _dp(f),
                               idx.ctypes.data_as(C.POINTER(C.c_size_t)), idx.size, int(bias), _dp(out))
    return out


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (C.c_uint32 * 4)()
    _load().orc_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def noise_raw(seed: int, step: int, tensor_id: int, count: int, first: int = 0) -> np.ndarray:
    out = np.empty(count, dtype=np.uint32)
    _load().orc_noise_raw(seed, step, tensor_id, first, count, out.ctypes.data_as(C.POINTER(C.c_uint32)))
    return out


def noise_normal(seed: int, step: int, tensor_id: int, count: int, first: int = 0) -> np.ndarray:
    out = np.empty(count, dtype=np.float64)
    _load().orc_noise_normal(seed, step, tensor_id, first, count, _dp(out))
    return out


def noise_finalize(acc, sigma: float, clip_total: float, total_batch: int, seed: int, step: int,
                   tensor_id: int) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.float64)
    out = np.empty(acc.size, dtype=np.float64)
    _load().orc_noise_finalize(_dp(acc), _dp(out), acc.size, sigma, clip_total, total_batch, seed, step,
                               tensor_id)
    return out.reshape(acc.shape)


def add_example_noise(acc, sigma: float, clip_total: float, total_batch: int, seed: int, step: int, tensor_id: int,
                      first_example: int, count: int) -> np.ndarray:
    """acc + the per-example noise draws of `count` examples (per-example form of the noise)."""
    out = np.array(acc, dtype=np.float64).reshape(-1).copy()
    _load().orc_add_example_noise(_dp(out), out.size, sigma, clip_total, total_batch, seed, step, tensor_id,
                                  first_example, count)
    return out.reshape(np.shape(acc))


def sgd_update(g, theta, v, lr: float, momentum: float):
    """One SGD step on a finalized gradient: returns (theta', v').  v None = no momentum buffer."""
    g = np.ascontiguousarray(g, dtype=np.float64)
    theta = np.array(theta, dtype=np.float64).reshape(-1).copy()
    vv = None if v is None else np.array(v, dtype=np.float64).reshape(-1).copy()
    _load().orc_sgd_update(_dp(g.reshape(-1)), _dp(theta), _dp(vv) if vv is not None else None, theta.size, lr, momentum)
    return theta, vv


def privatise(wl, inputs_per_micro_step, threads: int = 0, noise_form: str = "once"):
    """Whole optimiser step of a workload: clip-accumulate over its micro-steps, then noise and
    divide.  Tensor ids: 2*layer for the weight, 2*layer+1 for the bias.
    Returns dict(acc_w, acc_b, out_w, out_b, n2, f) (lists over layers; n2, f over micro-steps)."""
    layers = list(wl.layers)
    group_clip, clip_total = group_bounds(wl.clip_c, wl.n_groups)
    acc_w, acc_b = new_accumulators(layers)
    n2s, fs = [], []
    for m, inputs in enumerate(inputs_per_micro_step):
        n2, f = clip_accumulate(layers, inputs, wl.group_of_layer, group_clip, acc_w, acc_b, threads)
        n2s.append(n2)
        fs.append(f)
        if noise_form == "per_example":
            # every clipped example brings its own N(0, sigma^2 C^2 / |B|) draw
            for li in range(len(layers)):
                acc_w[li][...] = add_example_noise(acc_w[li], wl.sigma, clip_total, wl.total_batch, wl.philox_seed,
                                                   wl.step, 2 * li, m * wl.n, wl.n)
                if acc_b[li] is not None:
                    acc_b[li][...] = add_example_noise(acc_b[li], wl.sigma, clip_total, wl.total_batch,
                                                       wl.philox_seed, wl.step, 2 * li + 1, m * wl.n, wl.n)
    sigma_end = 0.0 if noise_form == "per_example" else wl.sigma
    out_w, out_b = [], []
    for li, l in enumerate(layers):
        out_w.append(noise_finalize(acc_w[li], sigma_end, clip_total, wl.total_batch, wl.philox_seed,
                                    wl.step, 2 * li))
        out_b.append(noise_finalize(acc_b[li], sigma_end, clip_total, wl.total_batch, wl.philox_seed,
                                    wl.step, 2 * li + 1) if acc_b[li] is not None else None)
    return dict(acc_w=acc_w, acc_b=acc_b, out_w=out_w, out_b=out_b, n2=n2s, f=fs)
