"""CPU oracle (test infrastructure only): ctypes front end of atlas_oracle.c.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It never imports the GPU package and the GPU package never
imports it.  Arrays are numpy; all floating point is fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "atlas_oracle.c")
_LIB = os.path.join(_HERE, "libatlas_oracle.so")

ACT_NONE, ACT_RELU, ACT_ELU = 0, 1, 2
FMT_F32, FMT_BF16, FMT_F16 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.ao_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().ao_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


_i64 = ctypes.c_int64


def in_degree(n: int, col: np.ndarray) -> np.ndarray:
    col = _c(col, np.int32)
    out = np.empty(n, dtype=np.int64)
    lib().ao_in_degree(_i64(n), _i64(col.size), _p(col), _p(out))
    return out


class InLists:
    """In-neighbour lists of `n_dst` destinations (vertex ids `dst_ids`, or
    0..n_dst-1 when None)."""

    def __init__(self, in_off: np.ndarray, in_src: np.ndarray, dst_ids: Optional[np.ndarray] = None):
        self.in_off = _c(in_off, np.int64)
        self.in_src = _c(in_src, np.int32)
        self.dst_ids = None if dst_ids is None else _c(dst_ids, np.int64)
        self.n_dst = self.in_off.size - 1

    @staticmethod
    def from_csr(off: np.ndarray, col: np.ndarray) -> "InLists":
        off = _c(off, np.int64)
        col = _c(col, np.int32)
        n = off.size - 1
        in_off = np.empty(n + 1, dtype=np.int64)
        in_src = np.empty(col.size, dtype=np.int32)
        lib().ao_build_in_lists(_i64(n), _p(off), _p(col), _p(in_off), _p(in_src))
        return InLists(in_off, in_src)


def neighbor_sum(il: InLists, X: np.ndarray, scale: Optional[np.ndarray] = None) -> np.ndarray:
    X = _c(X, np.float32)
    d = X.shape[1]
    scale = None if scale is None else _c(scale, np.float64)
    S = np.empty((il.n_dst, d), dtype=np.float64)
    lib().ao_neighbor_sum(_i64(il.n_dst), _p(il.in_off), _p(il.in_src), _p(X), _i64(d), _p(scale), _p(S))
    return S


def sage_mean(il: InLists, X: np.ndarray, W: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    X = _c(X, np.float32)
    W = _c(W, np.float64)
    b = None if b is None else _c(b, np.float64)
    d, dout = X.shape[1], W.shape[1]
    assert W.shape[0] == 2 * d
    Y = np.empty((il.n_dst, dout), dtype=np.float64)
    lib().ao_sage_mean(_i64(il.n_dst), _p(il.dst_ids), _p(il.in_off), _p(il.in_src), _p(X), _i64(d),
                       _p(W), _p(b), _i64(dout), _p(Y))
    return Y


def gcn(il: InLists, indeg: np.ndarray, X: np.ndarray, W: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    X = _c(X, np.float32)
    W = _c(W, np.float64)
    b = None if b is None else _c(b, np.float64)
    indeg = _c(indeg, np.int64)
    d, dout = X.shape[1], W.shape[1]
    assert W.shape[0] == d and indeg.size == X.shape[0]
    Y = np.empty((il.n_dst, dout), dtype=np.float64)
    lib().ao_gcn(_i64(il.n_dst), _p(il.dst_ids), _p(il.in_off), _p(il.in_src), _i64(X.shape[0]), _p(indeg),
                 _p(X), _i64(d), _p(W), _p(b), _i64(dout), _p(Y))
    return Y


def gin(il: InLists, X: np.ndarray, W: np.ndarray, b: Optional[np.ndarray], eps: float = 0.0) -> np.ndarray:
    """GIN layer with one linear map: ((1 + eps) x_v + sum of in-neighbours) W + b."""
    X = _c(X, np.float32)
    W = _c(W, np.float64)
    b = None if b is None else _c(b, np.float64)
    d, dout = X.shape[1], W.shape[1]
    assert W.shape[0] == d
    Y = np.empty((il.n_dst, dout), dtype=np.float64)
    lib().ao_gin(_i64(il.n_dst), _p(il.dst_ids), _p(il.in_off), _p(il.in_src), _p(X), _i64(d),
                 ctypes.c_double(eps), _p(W), _p(b), _i64(dout), _p(Y))
    return Y


def sgc_hop(il: InLists, indeg: np.ndarray, X: np.ndarray) -> np.ndarray:
    """One SGC propagation step: the symmetric-normalised neighbour sum, no weights."""
    X = _c(X, np.float32)
    indeg = _c(indeg, np.int64)
    assert indeg.size == X.shape[0]
    Y = np.empty((il.n_dst, X.shape[1]), dtype=np.float64)
    lib().ao_sym_propagate(_i64(il.n_dst), _p(il.dst_ids), _p(il.in_off), _p(il.in_src), _p(indeg), _p(X),
                           _i64(X.shape[1]), _p(Y))
    return Y


def gat(il: InLists, X: np.ndarray, W: np.ndarray, b: Optional[np.ndarray], a_src: np.ndarray,
        a_dst: np.ndarray, slope: float = 0.2) -> np.ndarray:
    X = _c(X, np.float32)
    W = _c(W, np.float64)
    b = None if b is None else _c(b, np.float64)
    a_src = _c(a_src, np.float64)
    a_dst = _c(a_dst, np.float64)
    heads, dh = a_src.shape
    d, dout = X.shape[1], W.shape[1]
    assert dout == heads * dh and W.shape[0] == d
    n = X.shape[0]
    Z = np.zeros((n, dout), dtype=np.float64)
    if il.dst_ids is None and il.n_dst == n:
        rows = None
        n_rows = n
    else:
        dst = il.dst_ids if il.dst_ids is not None else np.arange(il.n_dst, dtype=np.int64)
        rows = np.unique(np.concatenate([il.in_src.astype(np.int64), dst]))
        n_rows = rows.size
    lib().ao_linear_rows(_i64(n_rows), _p(rows), _p(X), _i64(d), _p(W), _i64(dout), _p(Z))
    Y = np.empty((il.n_dst, dout), dtype=np.float64)
    lib().ao_gat_attend(_i64(il.n_dst), _p(il.dst_ids), _p(il.in_off), _p(il.in_src), _p(Z), _p(a_src),
                        _p(a_dst), _i64(heads), _i64(dh), ctypes.c_double(slope), _p(b), _p(Y))
    return Y


def activation(Y: np.ndarray, kind: int) -> np.ndarray:
    Y = _c(Y, np.float64).copy()
    lib().ao_activation(_i64(Y.size), _p(Y), ctypes.c_int(kind))
    return Y


def round_storage(Y: np.ndarray, fmt: int) -> np.ndarray:
    Y = _c(Y, np.float64).copy()
    lib().ao_round_storage(_i64(Y.size), _p(Y), ctypes.c_int(fmt))
    return Y


def completion_chunk(il: InLists, selfmsg: bool, C: int) -> np.ndarray:
    """Chunk (of C sources) whose broadcast completes each destination of `il`, -1: complete at layer
    start.  With il.dst_ids the lists belong to those vertices and in_src holds streaming ids."""
    cc = np.empty(il.n_dst, dtype=np.int64)
    lib().ao_completion_chunk(_i64(il.n_dst), _p(il.dst_ids), _p(il.in_off), _p(il.in_src),
                              ctypes.c_int(int(selfmsg)), _i64(C), _p(cc))
    return cc


def pending_after(il: InLists, selfmsg: bool, bound: int) -> np.ndarray:
    out = np.empty(il.n_dst, dtype=np.int64)
    lib().ao_pending_after(_i64(il.n_dst), _p(il.dst_ids), _p(il.in_off), _p(il.in_src),
                           ctypes.c_int(int(selfmsg)), _i64(bound), _p(out))
    return out


def reorder_indegree_desc(indeg: np.ndarray):
    indeg = _c(indeg, np.int64)
    n = indeg.size
    new_of_old = np.empty(n, dtype=np.int32)
    old_of_new = np.empty(n, dtype=np.int32)
    lib().ao_reorder_indegree_desc(_i64(n), _p(indeg), _p(new_of_old), _p(old_of_new))
    return new_of_old, old_of_new


def order_score(off: np.ndarray, col: np.ndarray, indeg: np.ndarray) -> np.ndarray:
    off = _c(off, np.int64)
    col = _c(col, np.int32)
    indeg = _c(indeg, np.int64)
    n = off.size - 1
    s = np.empty(n, dtype=np.float64)
    lib().ao_order_score(_i64(n), _p(off), _p(col), _p(indeg), _p(s))
    return s


def reorder_score_desc(off: np.ndarray, col: np.ndarray, indeg: np.ndarray):
    """The paper's greedy order (Sec. 3.8): vertices by decreasing Score, ties by
    smaller id first (a stable library sort on the negated score)."""
    score = order_score(off, col, indeg)
    old_of_new = np.argsort(-score, kind="stable").astype(np.int32)
    new_of_old = np.empty_like(old_of_new)
    new_of_old[old_of_new] = np.arange(old_of_new.size, dtype=np.int32)
    return new_of_old, old_of_new


def message_span(il: "InLists", selfmsg: bool = False) -> np.ndarray:
    """Span of every vertex (Sec. 4.5): ids between its first and last
    in-neighbour in streaming order (0 for fewer than two messages)."""
    span = np.zeros(il.n_dst, dtype=np.int64)
    for v in range(il.n_dst):
        a, b = il.in_off[v], il.in_off[v + 1]
        if b > a:
            lo, hi = int(il.in_src[a]), int(il.in_src[b - 1])   # lists are ascending
            if selfmsg:
                lo, hi = min(lo, v), max(hi, v)
            span[v] = hi - lo
    return span


# --------------------------------------------------------------------------
# neighbourhood sampling by disabling edges (Sec. 3.9)
# --------------------------------------------------------------------------

def sample_in_edges(off: np.ndarray, col: np.ndarray, edge_key: np.ndarray, fanout: int):
    """The preprocessing pass the paper sketches for sampled inference (Sec.
    3.9): every destination keeps at most `fanout` of its in-edges and the rest
    are disabled.  Which ones is decided by the caller's random key per edge:
    the `fanout` smallest keys of each destination, ties by the edge's position
    in the CSR.  Returns the CSR (by source, original edge order) of the kept
    edges.  Plain per-destination selection."""
    off = np.asarray(off, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    key = np.asarray(edge_key, dtype=np.uint32)
    n, e = off.size - 1, col.size
    assert key.size == e and fanout >= 0
    keep = np.zeros(e, dtype=bool)
    order = np.lexsort((np.arange(e), key, col))     # by destination, then key, then position
    dst_sorted = col[order]
    start = np.searchsorted(dst_sorted, dst_sorted, side="left")
    keep[order[np.arange(e) - start < fanout]] = True
    src = np.repeat(np.arange(n), np.diff(off))
    new_off = np.zeros(n + 1, dtype=np.int64)
    np.add.at(new_off, src[keep] + 1, 1)
    return np.cumsum(new_off), col[keep].astype(np.int32)


# --------------------------------------------------------------------------
# bounded hot store (Sec. 3.5): which partial states are evicted and reloaded
# --------------------------------------------------------------------------

EVICT_MIN_PENDING, EVICT_MAX_PENDING = 0, 1


def hot_store_trace(off: np.ndarray, col: np.ndarray, chunk: int, slots: int, selfmsg: bool,
                    policy: int = EVICT_MIN_PENDING):
    """Replay of the memory manager of Sec. 3.5 for one layer streamed in
    chunks of `chunk` sources with `slots` hot-store slots, written as plain
    set bookkeeping (small graphs only).

    A vertex holds a slot from its first message until it has completed (all
    d_in messages, plus its own with `selfmsg`) and been flushed, which happens
    at the end of every chunk.  The self message carries no data: it never
    starts a state, but it needs the state in the hot store once one exists.
    Before a chunk's messages are applied, every destination of the chunk
    without a slot needs one; if the free slots do not suffice, the shortfall
    is evicted from the vertices that are hot, are not addressed by this chunk
    and are still incomplete -- fewest pending messages first (most, with
    EVICT_MAX_PENDING), ties by vertex id.  An evicted vertex that is addressed
    again is reloaded.  Returns (evictions, reloads, peak_hot) with per-chunk
    lists for the first two; raises ValueError if a chunk does not fit."""
    off = np.asarray(off, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    n = off.size - 1
    pending = np.bincount(col, minlength=n).astype(np.int64) + (1 if selfmsg else 0)
    hot, cold = set(), set()
    evictions, reloads, peak = [], [], 0
    for b0 in range(0, n, chunk):
        b1 = min(n, b0 + chunk)
        dst = col[off[b0]:off[b1]]
        addressed = set(int(v) for v in np.unique(dst))
        if selfmsg:
            addressed |= {v for v in range(b0, b1) if v in hot or v in cold}
        need = sorted(v for v in addressed if v not in hot)
        free = slots - len(hot)
        ev = 0
        if len(need) > free:
            ev = len(need) - free
            cands = [v for v in hot if v not in addressed and pending[v] > 0]
            if len(cands) < ev:
                raise ValueError("chunk [%d, %d) does not fit %d slots" % (b0, b1, slots))
            sign = 1 if policy == EVICT_MIN_PENDING else -1
            cands.sort(key=lambda v: (sign * int(pending[v]), v))
            for v in cands[:ev]:
                hot.remove(v)
                cold.add(v)
        rl = 0
        for v in need:
            if v in cold:
                cold.remove(v)
                rl += 1
            hot.add(v)
        peak = max(peak, len(hot))
        np.subtract.at(pending, dst, 1)
        if selfmsg:
            pending[b0:b1] -= 1
        for v in [v for v in hot if pending[v] == 0]:   # completed: flushed, slot released
            hot.remove(v)
        evictions.append(ev)
        reloads.append(rl)
    assert not hot and not cold and (pending == 0).all()
    return evictions, reloads, peak


# --------------------------------------------------------------------------
# whole-model chain
# --------------------------------------------------------------------------

def run_layer(model: str, il: InLists, indeg: Optional[np.ndarray], X: np.ndarray, params, act: int,
              out_fmt: int, slope: float = 0.2, eps: float = 0.0) -> np.ndarray:
    """One layer: aggregate + update (fp64), activation, round to storage.

    `params` has fp64 arrays W, bias (and attn_src / attn_dst for GAT) that
    already hold the rounded storage values.  Returns fp64 holding storage
    values (n_dst x d_out)."""
    if model == "sage":
        Y = sage_mean(il, X, params.W, params.bias)
    elif model == "gcn":
        Y = gcn(il, indeg, X, params.W, params.bias)
    elif model == "gat":
        Y = gat(il, X, params.W, params.bias, params.attn_src, params.attn_dst, slope)
    elif model == "gin":
        Y = gin(il, X, params.W, params.bias, eps)
    elif model == "sgc":   # propagation-only hops (no weights), then one GCN layer
        Y = sgc_hop(il, indeg, X) if params.W is None else gcn(il, indeg, X, params.W, params.bias)
    else:
        raise ValueError(model)
    return round_storage(activation(Y, act), out_fmt)


def run_model(model: str, off: np.ndarray, col: np.ndarray, X: np.ndarray, layers: Sequence,
              between_act: int, store_fmt: int, slope: float = 0.2, eps: float = 0.0) -> List[np.ndarray]:
    """All layers over the full graph; the activation applies between layers
    only, every layer's output is rounded to the storage format.  Returns the
    list of per-layer outputs."""
    il = InLists.from_csr(off, col)
    indeg = in_degree(off.size - 1, col)
    outs = []
    cur = np.asarray(X, dtype=np.float32)
    for li, p in enumerate(layers):
        act = between_act if li + 1 < len(layers) else ACT_NONE
        if model == "sgc":
            act = ACT_NONE   # SGC has no non-linearity between its hops
        Y = run_layer(model, il, indeg, cur, p, act, store_fmt, slope, eps)
        outs.append(Y)
        cur = Y.astype(np.float32)
    return outs
