"""ctypes binding of libripple.so: argument marshalling only.

Module-level functions carry the names of the C entry points (include/ripple.h)
and take/return plain numpy arrays or raw device pointers (integers, e.g. a
torch tensor's data_ptr()). Every step of the computation runs inside the
library's GPU kernels; there is no CPU fallback: loading fails loudly when the
shared library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libripple.so")

RIPPLE_OK, RIPPLE_EINVAL, RIPPLE_ESTATE, RIPPLE_ECAPACITY, RIPPLE_ENOMEM, RIPPLE_EDEVICE, RIPPLE_ERANGE = range(7)
STATUS_NAMES = ["RIPPLE_OK", "RIPPLE_EINVAL", "RIPPLE_ESTATE", "RIPPLE_ECAPACITY", "RIPPLE_ENOMEM",
                "RIPPLE_EDEVICE", "RIPPLE_ERANGE"]
RIPPLE_MAX_LAYERS = 8
RIPPLE_N_PHASES = 8
PHASES = ["ingest", "struct", "frontier", "scatter", "compact", "transform", "other", "total"]
OPT_TIMING, OPT_SCATTER_MODE, OPT_PULL_RATIO, OPT_PROJECT_FIRST, OPT_BF16_MFMA, OPT_SELF_CACHE, OPT_DETERMINISTIC = 0, 1, 2, 3, 4, 5, 6
OPT_SPLIT_MFMA = 7
OPT_SPARSE_FRONTIER = 8
OPT_ROW_SEGMENTS = 9
OPT_PACKED_MESSAGES = 10
OPT_STREAM_TRANSFORM = 11
OPT_SORTED_MESSAGES = 12
AGG = {"sum": 0, "mean": 1, "wsum": 2, "max": 3, "min": 4, "attn": 5}
SELF = {"none": 0, "concat": 1, "add": 2}
ACT = {"none": 0, "relu": 1}
STORE = {"f32": 0, "bf16": 1}

EXPORTS = ["ripple_init_graph", "ripple_init_graph_weighted", "ripple_load_model", "ripple_full_infer", "ripple_apply_updates",
           "ripple_get_embeddings", "ripple_get_aggregates", "ripple_get_layer_info", "ripple_get_affected", "ripple_get_affected_static",
           "ripple_export_edges",
           "ripple_get_degrees", "ripple_compact", "ripple_set_option", "ripple_get_stats", "ripple_plan_batch",
           "ripple_measure_peaks", "ripple_destroy", "ripple_last_error"]


class RippleError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {text}")
        self.status = status


class LayerDesc(C.Structure):
    _fields_ = [("d_in", C.c_uint32), ("d_hidden", C.c_uint32), ("d_out", C.c_uint32),
                ("agg", C.c_uint32), ("self_mode", C.c_uint32), ("eps", C.c_float),
                ("act_inner", C.c_uint32), ("act_out", C.c_uint32),
                ("W0", C.c_void_p), ("b0", C.c_void_p), ("W1", C.c_void_p), ("b1", C.c_void_p),
                ("att", C.c_void_p)]


class BatchResult(C.Structure):
    _fields_ = [("n_ops", C.c_uint32), ("n_applied", C.c_uint32), ("n_rejected", C.c_uint32),
                ("n_sub_batches", C.c_uint32), ("n_compactions", C.c_uint32), ("n_alive", C.c_uint32),
                ("n_edges", C.c_uint64),
                ("affected", C.c_uint32 * (RIPPLE_MAX_LAYERS + 1)),
                ("messages", C.c_uint64 * (RIPPLE_MAX_LAYERS + 1)),
                ("n_structural", C.c_uint32),
                ("mono_unchanged", C.c_uint32 * (RIPPLE_MAX_LAYERS + 1)),
                ("mono_incremental", C.c_uint32 * (RIPPLE_MAX_LAYERS + 1)),
                ("mono_recomputed", C.c_uint32 * (RIPPLE_MAX_LAYERS + 1)),
                ("hop_mode", C.c_uint32 * (RIPPLE_MAX_LAYERS + 1)),
                ("n_ops_done", C.c_uint32)]


class Stats(C.Structure):
    _fields_ = [("batches", C.c_uint64),
                ("ms", (C.c_double * (RIPPLE_MAX_LAYERS + 1)) * RIPPLE_N_PHASES),
                ("launches", (C.c_uint64 * (RIPPLE_MAX_LAYERS + 1)) * RIPPLE_N_PHASES),
                ("rows", C.c_uint64 * (RIPPLE_MAX_LAYERS + 1)),
                ("msgs", C.c_uint64 * (RIPPLE_MAX_LAYERS + 1)),
                ("touched", C.c_uint64 * (RIPPLE_MAX_LAYERS + 1))]


class Peaks(C.Structure):
    _fields_ = [("hbm_copy_gbps", C.c_double), ("hbm_read_gbps", C.c_double), ("gather_glines", C.c_double), ("atomic_gops", C.c_double),
                ("mfma_f32_tflops", C.c_double), ("mfma_bf16_tflops", C.c_double),
                ("compute_units", C.c_uint32), ("reserved", C.c_uint32)]


_lib = None


def load_library():
    """dlopen libripple.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           "`python -m paper_2601_12347_amd.build` (needs hipcc)")
    # PyTorch (the caller's device-memory and stream provider) bundles its own HIP runtime.
    # Two HIP runtimes in one process do not share the GPU, so torch is imported first and
    # libripple.so then binds to the runtime that is already loaded.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
    lib.ripple_init_graph.argtypes = [C.POINTER(vp), u32, u32, u64, u64, vp, vp, vp, u32, C.c_int, vp]
    lib.ripple_init_graph_weighted.argtypes = [C.POINTER(vp), u32, u32, u64, u64, vp, vp, vp, vp, u32, C.c_int, vp]
    lib.ripple_load_model.argtypes = [vp, u32, C.POINTER(LayerDesc)]
    lib.ripple_full_infer.argtypes = [vp]
    lib.ripple_apply_updates.argtypes = [vp, vp, u32, vp, u32, C.POINTER(BatchResult)]
    lib.ripple_get_embeddings.argtypes = [vp, u32, vp, u32, vp]
    lib.ripple_get_aggregates.argtypes = [vp, u32, vp, u32, vp]
    lib.ripple_get_layer_info.argtypes = [vp, u32, C.POINTER(u32), C.POINTER(C.c_int)]
    lib.ripple_get_affected.argtypes = [vp, u32, vp, u32, C.POINTER(u32)]
    lib.ripple_get_affected_static.argtypes = [vp, u32, vp, u32, vp]
    lib.ripple_export_edges.argtypes = [vp, C.c_int, vp, vp, u64, C.POINTER(u64)]
    lib.ripple_get_degrees.argtypes = [vp, C.c_int, vp, vp]
    lib.ripple_compact.argtypes = [vp]
    lib.ripple_set_option.argtypes = [vp, C.c_int, C.c_int64]
    lib.ripple_get_stats.argtypes = [vp, C.POINTER(Stats), C.c_int]
    lib.ripple_plan_batch.argtypes = [vp, u32, u32, u32, vp, u32, C.POINTER(u32)]
    lib.ripple_measure_peaks.argtypes = [C.POINTER(Peaks), vp]
    lib.ripple_destroy.argtypes = [vp]
    lib.ripple_destroy.restype = None
    lib.ripple_last_error.argtypes = [vp]
    lib.ripple_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("ripple_destroy", "ripple_last_error"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _ptr(x):
    """numpy array -> host pointer; int -> raw (device) pointer; None -> NULL."""
    if x is None:
        return None
    if isinstance(x, (int, np.integer)):
        return C.c_void_p(int(x))
    return C.c_void_p(x.ctypes.data)


def _check(ctx, rc):
    if rc != RIPPLE_OK:
        text = load_library().ripple_last_error(ctx).decode() if ctx else ""
        raise RippleError(rc, text)


def ripple_init_graph(n_vertices, vertex_capacity, src, dst, features, store="f32", edge_capacity=None,
                      hip_stream=0):
    lib = load_library()
    src = np.ascontiguousarray(src, dtype=np.uint32)
    dst = np.ascontiguousarray(dst, dtype=np.uint32)
    features = np.ascontiguousarray(features, dtype=np.float32)
    if features.ndim != 2 or features.shape[0] != n_vertices or src.shape != dst.shape:
        raise ValueError("features must be [n_vertices x d0]; src and dst must have equal length")
    if edge_capacity is None:
        edge_capacity = int(src.size * 1.25) + 4096
    ctx = C.c_void_p()
    rc = lib.ripple_init_graph(C.byref(ctx), n_vertices, vertex_capacity, src.size, edge_capacity,
                               _ptr(src), _ptr(dst), _ptr(features), features.shape[1],
                               STORE[store] if isinstance(store, str) else int(store),
                               C.c_void_p(int(hip_stream)))
    return _checked_ctx(lib, ctx, rc)


def _checked_ctx(lib, ctx, rc):
    if rc != RIPPLE_OK:
        text = lib.ripple_last_error(ctx).decode() if ctx else "invalid argument"
        if ctx:
            lib.ripple_destroy(ctx)
        raise RippleError(rc, text)
    return ctx


def ripple_init_graph_weighted(n_vertices, vertex_capacity, src, dst, edge_weights, features, store="f32",
                               edge_capacity=None, hip_stream=0):
    lib = load_library()
    src = np.ascontiguousarray(src, dtype=np.uint32)
    dst = np.ascontiguousarray(dst, dtype=np.uint32)
    edge_weights = np.ascontiguousarray(edge_weights, dtype=np.float32)
    features = np.ascontiguousarray(features, dtype=np.float32)
    if (features.ndim != 2 or features.shape[0] != n_vertices or src.shape != dst.shape
            or edge_weights.shape != src.shape):
        raise ValueError("features must be [n_vertices x d0]; src, dst and edge_weights must have equal length")
    if edge_capacity is None:
        edge_capacity = int(src.size * 1.25) + 4096
    ctx = C.c_void_p()
    rc = lib.ripple_init_graph_weighted(C.byref(ctx), n_vertices, vertex_capacity, src.size, edge_capacity,
                                        _ptr(src), _ptr(dst), _ptr(edge_weights), _ptr(features), features.shape[1],
                                        STORE[store] if isinstance(store, str) else int(store),
                                        C.c_void_p(int(hip_stream)))
    return _checked_ctx(lib, ctx, rc)


def ripple_load_model(ctx, model):
    """model: list of layer dicts as produced by ripple_inputs.make_model."""
    lib = load_library()
    descs = (LayerDesc * len(model))()
    keep = []
    for i, lay in enumerate(model):
        w0 = np.ascontiguousarray(lay["W0"], dtype=np.float32)
        b0 = np.ascontiguousarray(lay["b0"], dtype=np.float32)
        keep += [w0, b0]
        d = descs[i]
        d.d_in, d.d_hidden, d.d_out = lay["d_in"], lay["d_hidden"], lay["d_out"]
        d.agg, d.self_mode, d.eps = AGG[lay["agg"]], SELF[lay["self"]], float(lay["eps"])
        d.act_inner, d.act_out = ACT[lay["act_inner"]], ACT[lay["act_out"]]
        d.W0, d.b0 = w0.ctypes.data, b0.ctypes.data
        if lay["d_hidden"]:
            w1 = np.ascontiguousarray(lay["W1"], dtype=np.float32)
            b1 = np.ascontiguousarray(lay["b1"], dtype=np.float32)
            keep += [w1, b1]
            d.W1, d.b1 = w1.ctypes.data, b1.ctypes.data
        if lay["agg"] == "attn":
            att = np.ascontiguousarray(lay["att"], dtype=np.float32)
            if att.shape != (2 * lay["d_out"],):
                raise ValueError("att must hold a_src followed by a_dst, d_out numbers each")
            keep.append(att)
            d.att = att.ctypes.data
    _check(ctx, lib.ripple_load_model(ctx, len(model), descs))


def ripple_full_infer(ctx):
    _check(ctx, load_library().ripple_full_infer(ctx))


def ripple_apply_updates(ctx, ops, payload, n_ops=None, n_feat_rows=None):
    """ops: uint32 [n x 4] numpy array, or a device pointer (then pass n_ops);
    payload: float32 [rows x d0] numpy array, or a device pointer (then pass n_feat_rows)."""
    lib = load_library()
    if not isinstance(ops, (int, np.integer)):
        ops = np.ascontiguousarray(ops, dtype=np.uint32).reshape(-1, 4)
        n_ops = ops.shape[0]
    if payload is not None and not isinstance(payload, (int, np.integer)):
        payload = np.ascontiguousarray(payload, dtype=np.float32)
        n_feat_rows = payload.shape[0] if payload.ndim == 2 else 0
        if n_feat_rows == 0:
            payload = None
    res = BatchResult()
    try:
        _check(ctx, lib.ripple_apply_updates(ctx, _ptr(ops) if n_ops else None, n_ops or 0,
                                             _ptr(payload) if n_feat_rows else None, n_feat_rows or 0,
                                             C.byref(res)))
    except RippleError as err:
        err.result = res            # how far the batch got (n_ops_done and the counts of that prefix)
        raise
    return res


def _get_rows(fn, ctx, layer, ids, n_rows, width, out):
    if ids is not None and not isinstance(ids, (int, np.integer)):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        n_rows = ids.size
    if out is None:
        out = np.empty((n_rows, width), dtype=np.float32)
    _check(ctx, fn(ctx, layer, _ptr(ids), n_rows, _ptr(out)))
    return out


def ripple_get_embeddings(ctx, layer, width, ids=None, n_rows=None, out=None):
    return _get_rows(load_library().ripple_get_embeddings, ctx, layer, ids, n_rows, width, out)


def ripple_get_aggregates(ctx, layer, width, ids=None, n_rows=None, out=None):
    return _get_rows(load_library().ripple_get_aggregates, ctx, layer, ids, n_rows, width, out)


def ripple_get_layer_info(ctx, layer):
    """(width of the cached aggregate rows, handled project-first?, self term cached?)"""
    w, p = C.c_uint32(), C.c_int()
    _check(ctx, load_library().ripple_get_layer_info(ctx, layer, C.byref(w), C.byref(p)))
    return w.value, bool(p.value & 1), bool(p.value & 2)


def ripple_layer_packs_messages(ctx, layer):
    """True when the layer's messages travel as packed 128-byte rows (flag bit 2 of ripple_get_layer_info)."""
    p = C.c_int()
    _check(ctx, load_library().ripple_get_layer_info(ctx, layer, None, C.byref(p)))
    return bool(p.value & 4)


def ripple_get_affected(ctx, layer, cap):
    out = np.empty(max(int(cap), 1), dtype=np.uint32)
    n = C.c_uint32()
    _check(ctx, load_library().ripple_get_affected(ctx, layer, _ptr(out), int(cap), C.byref(n)))
    return out[:min(n.value, int(cap))].copy(), n.value


def ripple_get_affected_static(ctx, layer, ids_ptr, cap, n_ptr):
    """ids_ptr, n_ptr: device pointers (integers) owned by the caller; nothing is allocated by the call."""
    _check(ctx, load_library().ripple_get_affected_static(ctx, layer, _ptr(int(ids_ptr)) if ids_ptr else None, int(cap),
                                                          _ptr(int(n_ptr)) if n_ptr else None))


def ripple_export_edges(ctx, direction, cap):
    src = np.empty(max(int(cap), 1), dtype=np.uint32)
    dst = np.empty(max(int(cap), 1), dtype=np.uint32)
    n = C.c_uint64()
    _check(ctx, load_library().ripple_export_edges(ctx, direction, _ptr(src), _ptr(dst), int(cap), C.byref(n)))
    k = min(n.value, int(cap))
    return src[:k].copy(), dst[:k].copy(), n.value


def ripple_get_degrees(ctx, direction, vertex_capacity):
    deg = np.empty(vertex_capacity, dtype=np.uint32)
    alive = np.empty(vertex_capacity, dtype=np.uint8)
    _check(ctx, load_library().ripple_get_degrees(ctx, direction, _ptr(deg), _ptr(alive)))
    return deg, alive.astype(bool)


def ripple_compact(ctx):
    _check(ctx, load_library().ripple_compact(ctx))


def ripple_set_option(ctx, option, value):
    _check(ctx, load_library().ripple_set_option(ctx, option, int(value)))


def ripple_get_stats(ctx, reset=False):
    st = Stats()
    _check(ctx, load_library().ripple_get_stats(ctx, C.byref(st), 1 if reset else 0))
    return st


def ripple_plan_batch(ops, vertex_capacity, n_feat_rows):
    """Ends (exclusive) of the conflict-free pieces ripple_apply_updates would cut `ops` into; host only."""
    ops = np.ascontiguousarray(ops, dtype=np.uint32).reshape(-1, 4)
    ends = np.zeros(max(len(ops), 1), dtype=np.uint32)
    n = C.c_uint32(0)
    rc = load_library().ripple_plan_batch(_ptr(ops) if len(ops) else None, len(ops), int(vertex_capacity),
                                          int(n_feat_rows), _ptr(ends), len(ends), C.byref(n))
    if rc != RIPPLE_OK:
        raise RippleError(rc, "ripple_plan_batch")
    return ends[: n.value].tolist()


def ripple_measure_peaks(stream=None):
    """Measured rates of the current GPU as a dict (see ripple_peaks in include/ripple.h)."""
    p = Peaks()
    rc = load_library().ripple_measure_peaks(C.byref(p), C.c_void_p(int(stream)) if stream else None)
    if rc != RIPPLE_OK:
        raise RippleError(rc, "ripple_measure_peaks")
    return {name: getattr(p, name) for name, _ in Peaks._fields_ if name != "reserved"}


def ripple_destroy(ctx):
    if ctx:
        load_library().ripple_destroy(ctx)


def ripple_last_error(ctx):
    return load_library().ripple_last_error(ctx).decode()
