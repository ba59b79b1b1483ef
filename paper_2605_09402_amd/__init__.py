"""Python binding of libatlas.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/atlas.h).
Tensors are used for their device / pinned-host addresses; streams are raw
hipStream_t handles (torch.cuda.Stream().cuda_stream).  There is no fallback:
if the HIP library has not been built the import of any entry point raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libatlas.so")

OK = 0
E_NULL, E_BAD_DIMS, E_RANGE, E_ORDER, E_INCOMPLETE, E_OVERFLOW, E_HIP, E_NOMEM, E_STATE, E_TOO_LARGE = range(-1, -11, -1)
NOALLOC_MAX_VERTICES = 1 << 20
RESIDENT_DEVICE, RESIDENT_PINNED_HOST = 0, 1
MODEL_SAGE_MEAN, MODEL_GCN_SYM, MODEL_GAT, MODEL_GIN, MODEL_SGC_HOP = 0, 1, 2, 3, 4
DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
ACT_NONE, ACT_RELU, ACT_ELU = 0, 1, 2
FLAG_TIMING = 1
FLAG_EMB_RESIDENT = 2
FLAG_PLANNED_ONLY = 4
FLAG_TRANSFORM_FIRST = 8
FLAG_CSR_STREAM = 16
FLAG_NO_HANDOVER = 32
FLAG_NO_DENSE = 64
EVICT_MIN_PENDING, EVICT_MAX_PENDING = 0, 1
DBG_INDEG, DBG_PENDING, DBG_READY, DBG_READY_COUNT, DBG_ACC = range(5)

EXPORTS = [
    "atlas_layer_init", "atlas_attention_prepass", "atlas_broadcast_chunk", "atlas_flush_ready",
    "atlas_layer_finish", "atlas_in_degree", "atlas_reorder_indegree_desc", "atlas_debug_copy",
    "atlas_release_cache", "atlas_strerror", "atlas_last_hip_error", "atlas_plan_create", "atlas_plan_destroy",
    "atlas_reorder_score_desc", "atlas_sample_in_edges", "atlas_plan_create_blocked", "atlas_plan_create_dense",
    "atlas_reorder_indegree_desc_noalloc", "atlas_plan_info", "atlas_plan_in_degree", "atlas_probe_copy", "atlas_probe_row_gather",
    "atlas_probe_dense_rows", "atlas_probe_gather_sink_bytes", "atlas_probe_mix21", "atlas_probe_mfma",
]


class atlas_graph_t(ctypes.Structure):
    _fields_ = [("num_vertices", ctypes.c_int64), ("num_edges", ctypes.c_int64),
                ("row_offsets", ctypes.c_void_p), ("col_indices", ctypes.c_void_p),
                ("in_degree", ctypes.c_void_p), ("residency", ctypes.c_int32),
                ("plan", ctypes.c_void_p)]


class atlas_dims_t(ctypes.Structure):
    _fields_ = [("model", ctypes.c_int32), ("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32),
                ("heads", ctypes.c_int32), ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("activation", ctypes.c_int32), ("neg_slope", ctypes.c_float),
                ("max_chunk_sources", ctypes.c_int64), ("flags", ctypes.c_int32), ("gin_eps", ctypes.c_float),
                ("hot_slots", ctypes.c_int64), ("evict_policy", ctypes.c_int32),
                ("tiles_per_run", ctypes.c_int32), ("piece_tiles", ctypes.c_int64)]


class atlas_weights_t(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("attn_src", ctypes.c_void_p),
                ("attn_dst", ctypes.c_void_p), ("dtype", ctypes.c_int32)]


class atlas_layer_stats_t(ctypes.Structure):
    _fields_ = [("edges_processed", ctypes.c_int64), ("sources_processed", ctypes.c_int64),
                ("vertices_completed", ctypes.c_int64), ("vertices_flushed", ctypes.c_int64),
                ("num_chunks", ctypes.c_int64), ("num_flushes", ctypes.c_int64),
                ("bytes_copied_h2d", ctypes.c_int64), ("ms_aggregate", ctypes.c_float),
                ("ms_self", ctypes.c_float), ("ms_update", ctypes.c_float), ("ms_copy", ctypes.c_float),
                ("ms_init", ctypes.c_float), ("hot_evictions", ctypes.c_int64), ("hot_reloads", ctypes.c_int64),
                ("hot_peak_slots", ctypes.c_int64), ("chunks_planned", ctypes.c_int64),
                ("chunks_csr_stream", ctypes.c_int64), ("chunks_regrouped", ctypes.c_int64),
                ("ms_regroup", ctypes.c_float), ("ms_dense", ctypes.c_float), ("rows_handed_over", ctypes.c_int64),
                ("edges_contracted", ctypes.c_int64), ("ms_contract", ctypes.c_float)]


class atlas_plan_info_t(ctypes.Structure):
    _fields_ = [("num_chunks", ctypes.c_int64), ("num_edges", ctypes.c_int64), ("num_groups", ctypes.c_int64),
                ("num_first_groups", ctypes.c_int64), ("bytes_device", ctypes.c_int64),
                ("bytes_pinned_host", ctypes.c_int64), ("dense_edges", ctypes.c_int64), ("dense_groups", ctypes.c_int64), ("dense_cells", ctypes.c_int64),
                ("dense_rows", ctypes.c_int64), ("dense_max_sources", ctypes.c_int64)]


class AtlasError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = ""
        if status in (E_HIP, E_NOMEM):
            detail = " [" + lib().atlas_last_hip_error().decode() + "]"
        super().__init__("%s: %s (%d)%s" % (where, lib().atlas_strerror(status).decode(), status, detail))


_lib = None


def lib() -> ctypes.CDLL:
    """Load libatlas.so; raises if it has not been built (no CPU fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libatlas.so is missing: run `python -m paper_2605_09402_amd.build` "
                              "(hipcc, gfx950) first; there is no fallback path")
        # torch ships its own HIP runtime: load it first so that the library binds to the runtime the
        # caller's tensors and streams live in (two runtimes in one process do not share devices)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        L.atlas_layer_init.argtypes = [ctypes.POINTER(atlas_graph_t), ctypes.POINTER(atlas_dims_t),
                                       ctypes.POINTER(atlas_weights_t), vp, ctypes.POINTER(vp)]
        L.atlas_attention_prepass.argtypes = [vp, i64, i64, vp, vp]
        L.atlas_broadcast_chunk.argtypes = [vp, i64, i64, vp, vp]
        L.atlas_flush_ready.argtypes = [vp, vp, ctypes.POINTER(i64), vp]
        L.atlas_layer_finish.argtypes = [vp, ctypes.POINTER(atlas_layer_stats_t)]
        L.atlas_in_degree.argtypes = [ctypes.POINTER(atlas_graph_t), vp, vp]
        L.atlas_reorder_indegree_desc.argtypes = [ctypes.POINTER(atlas_graph_t), vp, vp]
        L.atlas_reorder_indegree_desc_noalloc.argtypes = [ctypes.POINTER(atlas_graph_t), vp, vp, vp]
        L.atlas_reorder_score_desc.argtypes = [ctypes.POINTER(atlas_graph_t), vp, vp]
        L.atlas_sample_in_edges.argtypes = [ctypes.POINTER(atlas_graph_t), vp, i32, vp, vp, ctypes.POINTER(i64)]
        L.atlas_debug_copy.argtypes = [vp, i32, vp, i64]
        L.atlas_release_cache.argtypes = []
        L.atlas_plan_create.argtypes = [ctypes.POINTER(atlas_graph_t), i64, ctypes.POINTER(vp)]
        L.atlas_plan_create_blocked.argtypes = [ctypes.POINTER(atlas_graph_t), i64, i64, i64, ctypes.POINTER(vp)]
        L.atlas_plan_create_dense.argtypes = [ctypes.POINTER(atlas_graph_t), i64, i64, i64, i64, i64, ctypes.POINTER(vp)]
        L.atlas_plan_destroy.argtypes = [vp]
        L.atlas_plan_info.argtypes = [vp, ctypes.POINTER(atlas_plan_info_t)]
        L.atlas_plan_in_degree.argtypes = [vp, vp, vp]
        L.atlas_probe_copy.argtypes = [vp, vp, i64, vp]
        L.atlas_probe_mix21.argtypes = [vp, vp, vp, i64, vp]
        L.atlas_probe_mfma.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.atlas_probe_gather_sink_bytes.argtypes = []
        L.atlas_probe_row_gather.argtypes = [vp, i64, vp, i64, vp, vp]
        L.atlas_probe_dense_rows.argtypes = [i32, vp, i64, i32, i32, vp, vp, i32, vp]
        for name in EXPORTS:
            getattr(L, name).restype = ctypes.c_int      # raises AttributeError on a missing export
        L.atlas_probe_gather_sink_bytes.restype = ctypes.c_int64
        L.atlas_strerror.argtypes = [i32]
        L.atlas_strerror.restype = ctypes.c_char_p
        L.atlas_last_hip_error.argtypes = []
        L.atlas_last_hip_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    """Address of a tensor's storage (or an int / None passed through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str):
    if status != OK:
        raise AtlasError(status, where)


def make_graph(num_vertices: int, num_edges: int, row_offsets, col_indices, in_degree=None,
               residency: int = RESIDENT_DEVICE, plan: Optional[int] = None) -> atlas_graph_t:
    """Fill an atlas_graph_t from tensors (int64 offsets, int32 columns / degrees).
    The caller keeps the tensors (and the plan) alive."""
    return atlas_graph_t(num_vertices, num_edges, _ptr(row_offsets), _ptr(col_indices), _ptr(in_degree),
                         residency, plan)


def make_dims(model: int, d_in: int, d_out: int, in_dtype: int, out_dtype: int, activation: int,
              max_chunk_sources: int, heads: int = 1, neg_slope: float = 0.2, flags: int = 0,
              gin_eps: float = 0.0, hot_slots: int = 0, evict_policy: int = 0, tiles_per_run: int = 0,
              piece_tiles: int = 0) -> atlas_dims_t:
    return atlas_dims_t(model, d_in, d_out, heads, in_dtype, out_dtype, activation, neg_slope,
                        max_chunk_sources, flags, gin_eps, hot_slots, evict_policy, tiles_per_run, piece_tiles)


def make_weights(W, bias, dtype: int, attn_src=None, attn_dst=None) -> atlas_weights_t:
    return atlas_weights_t(_ptr(W), _ptr(bias), _ptr(attn_src), _ptr(attn_dst), dtype)


def atlas_layer_init(graph: atlas_graph_t, dims: atlas_dims_t, weights: atlas_weights_t, stream=None) -> int:
    h = ctypes.c_void_p()
    _check(lib().atlas_layer_init(ctypes.byref(graph), ctypes.byref(dims), ctypes.byref(weights),
                                  _stream(stream), ctypes.byref(h)), "atlas_layer_init")
    return h.value


def atlas_attention_prepass(layer: int, src_begin: int, src_end: int, emb, stream=None) -> None:
    _check(lib().atlas_attention_prepass(layer, src_begin, src_end, _ptr(emb), _stream(stream)),
           "atlas_attention_prepass")


def atlas_broadcast_chunk(layer: int, src_begin: int, src_end: int, emb, stream=None) -> None:
    _check(lib().atlas_broadcast_chunk(layer, src_begin, src_end, _ptr(emb), _stream(stream)),
           "atlas_broadcast_chunk")


def atlas_flush_ready(layer: int, out, stream=None, count: bool = False) -> Optional[int]:
    """count=True waits for the stream and returns the number of rows written."""
    n = ctypes.c_int64(0)
    _check(lib().atlas_flush_ready(layer, _ptr(out), ctypes.byref(n) if count else None, _stream(stream)),
           "atlas_flush_ready")
    return n.value if count else None


def atlas_layer_finish(layer: int) -> dict:
    st = atlas_layer_stats_t()
    status = lib().atlas_layer_finish(layer, ctypes.byref(st))
    stats = {name: getattr(st, name) for name, _ in atlas_layer_stats_t._fields_}
    if status != OK:
        err = AtlasError(status, "atlas_layer_finish")
        err.stats = stats
        raise err
    return stats


def atlas_plan_create(graph: atlas_graph_t, chunk_sources: int) -> int:
    h = ctypes.c_void_p()
    _check(lib().atlas_plan_create(ctypes.byref(graph), chunk_sources, ctypes.byref(h)), "atlas_plan_create")
    return h.value


def atlas_plan_create_blocked(graph: atlas_graph_t, chunk_sources: int, block_sources: int, hot_min_edges: int) -> int:
    h = ctypes.c_void_p()
    _check(lib().atlas_plan_create_blocked(ctypes.byref(graph), chunk_sources, block_sources, hot_min_edges,
                                           ctypes.byref(h)), "atlas_plan_create_blocked")
    return h.value


def atlas_plan_create_dense(graph: atlas_graph_t, chunk_sources: int, block_sources: int, hot_min_edges: int,
                            dense_max_bytes: int, dense_cells_per_edge: int = 0) -> int:
    h = ctypes.c_void_p()
    _check(lib().atlas_plan_create_dense(ctypes.byref(graph), chunk_sources, block_sources, hot_min_edges,
                                         dense_max_bytes, dense_cells_per_edge, ctypes.byref(h)),
           "atlas_plan_create_dense")
    return h.value


def atlas_plan_info(plan: int) -> dict:
    info = atlas_plan_info_t()
    _check(lib().atlas_plan_info(plan, ctypes.byref(info)), "atlas_plan_info")
    return {name: getattr(info, name) for name, _ in atlas_plan_info_t._fields_}


def atlas_plan_in_degree(plan: int, in_degree, stream=None) -> None:
    _check(lib().atlas_plan_in_degree(plan, _ptr(in_degree), _stream(stream)), "atlas_plan_in_degree")


def atlas_probe_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(lib().atlas_probe_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "atlas_probe_copy")


def atlas_probe_mfma(waves_per_simd: int, iters: int, sink, stream=None) -> float:
    """Enqueues the bare matrix-instruction loop; returns the launch's flop count."""
    fl = ctypes.c_double()
    _check(lib().atlas_probe_mfma(waves_per_simd, iters, _ptr(sink), ctypes.byref(fl), _stream(stream)), "atlas_probe_mfma")
    return fl.value


def atlas_probe_mix21(dst, a, b, nbytes: int, stream=None) -> None:
    _check(lib().atlas_probe_mix21(_ptr(dst), _ptr(a), _ptr(b), nbytes, _stream(stream)), "atlas_probe_mix21")


def atlas_probe_gather_sink_bytes() -> int:
    return int(lib().atlas_probe_gather_sink_bytes())


def atlas_probe_row_gather(table, table_rows: int, ids, n_ids: int, sink, stream=None) -> None:
    _check(lib().atlas_probe_row_gather(_ptr(table), table_rows, _ptr(ids), n_ids, _ptr(sink), _stream(stream)),
           "atlas_probe_row_gather")


def atlas_probe_dense_rows(dtype: int, rows, n_rows: int, K: int, d_out: int, W, out, repeat: int = 1,
                           stream=None) -> None:
    _check(lib().atlas_probe_dense_rows(dtype, _ptr(rows), n_rows, K, d_out, _ptr(W), _ptr(out), repeat,
                                        _stream(stream)), "atlas_probe_dense_rows")


def atlas_plan_destroy(plan: int) -> None:
    _check(lib().atlas_plan_destroy(plan), "atlas_plan_destroy")


def atlas_in_degree(graph: atlas_graph_t, in_degree, stream=None) -> None:
    _check(lib().atlas_in_degree(ctypes.byref(graph), _ptr(in_degree), _stream(stream)), "atlas_in_degree")


def atlas_reorder_indegree_desc(graph: atlas_graph_t, new_of_old, old_of_new) -> None:
    _check(lib().atlas_reorder_indegree_desc(ctypes.byref(graph), _ptr(new_of_old), _ptr(old_of_new)),
           "atlas_reorder_indegree_desc")


def atlas_reorder_indegree_desc_noalloc(graph: atlas_graph_t, new_of_old, old_of_new, stream=None) -> None:
    _check(lib().atlas_reorder_indegree_desc_noalloc(ctypes.byref(graph), _ptr(new_of_old), _ptr(old_of_new),
                                                     _stream(stream)), "atlas_reorder_indegree_desc_noalloc")


def atlas_reorder_score_desc(graph: atlas_graph_t, new_of_old, old_of_new) -> None:
    _check(lib().atlas_reorder_score_desc(ctypes.byref(graph), _ptr(new_of_old), _ptr(old_of_new)),
           "atlas_reorder_score_desc")


def atlas_sample_in_edges(graph: atlas_graph_t, edge_key, fanout: int, out_row_offsets, out_col_indices) -> int:
    """Returns the number of kept edges."""
    kept = ctypes.c_int64(0)
    _check(lib().atlas_sample_in_edges(ctypes.byref(graph), _ptr(edge_key), fanout, _ptr(out_row_offsets),
                                       _ptr(out_col_indices), ctypes.byref(kept)), "atlas_sample_in_edges")
    return kept.value


def atlas_debug_copy(layer: int, what: int, host_array) -> None:
    """host_array: a numpy array (contiguous) that receives the bytes."""
    _check(lib().atlas_debug_copy(layer, what, host_array.ctypes.data, host_array.nbytes), "atlas_debug_copy")


def atlas_release_cache() -> None:
    _check(lib().atlas_release_cache(), "atlas_release_cache")
