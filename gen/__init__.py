"""Seeded synthetic inputs: graphs, features and layer parameters.

Everything here is *input data*: a counter-based 64-bit hash, the graph
generators (uniform multigraph, R-MAT), a seeded id bijection, a relabelling
helper that applies a permutation somebody else computed, a CSR-by-source
builder, feature matrices and Xavier-style weights.  None of the layer
arithmetic (aggregation, normalisation, degree counting for the method,
reordering decisions) lives here, so both the CPU oracle's tests and the GPU
path's tests can consume the same arrays without sharing any method code.

All integer work is written with torch int64 tensor ops only, so the very same
code produces bit-identical graphs on CPU tensors and on GPU tensors; large
graphs are generated batch by batch on whatever device is asked for.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, Iterator, Optional, Tuple

import torch

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit constant."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)
_STREAM_MUL = _s64(0xD6E8FEB86659FD93)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on int64 lanes (wrapping arithmetic)."""
    z = x + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _mix64_int(x: int) -> int:
    z = (x + 0x9E3779B97F4A7C15) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """Per-(seed, stream) key; counters are added to it before mixing."""
    return _s64(_mix64_int((seed & _MASK64) ^ ((stream * 0xD6E8FEB86659FD93) & _MASK64)))


def hash_counter(seed: int, stream: int, ctr: torch.Tensor) -> torch.Tensor:
    """64 pseudo-random bits per counter value (int64 tensor in, int64 out)."""
    return mix64(ctr + stream_key(seed, stream))


# Stream ids (one independent sequence each).
STREAM_GRAPH = 0
STREAM_IDPERM = 1
STREAM_FEATURES = 2
STREAM_WEIGHTS = 3  # + layer index * 4 + {0: W, 1: bias, 2: attn_src, 3: attn_dst}
STREAM_SAMPLING = 1000


# --------------------------------------------------------------------------
# graphs
# --------------------------------------------------------------------------

def uniform_edges(seed: int, n: int, lo: int, hi: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Edges [lo, hi) of a uniform directed multigraph without self-edges.

    src = r1 mod n and dst = (src + 1 + r2 mod (n-1)) mod n, so dst != src
    without a rejection loop; duplicate edges are kept.
    """
    e = torch.arange(lo, hi, dtype=torch.int64, device=device)
    r1 = _lsr(hash_counter(seed, STREAM_GRAPH, 2 * e), 1)
    r2 = _lsr(hash_counter(seed, STREAM_GRAPH, 2 * e + 1), 1)
    src = r1 % n
    dst = (src + 1 + r2 % (n - 1)) % n
    return src, dst


_RMAT_BITS = 16


def rmat_edges(seed: int, scale: int, lo: int, hi: int, a=0.57, b=0.19, c=0.19,
               device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Edges [lo, hi) of a plain R-MAT graph on 2**scale vertices (no noise).

    Each edge index owns a private hash sequence; every bit level draws 16
    bits and picks the quadrant a=(0,0), b=(0,1), c=(1,0), d=(1,1) of
    (src bit, dst bit).  Levels run from the most significant bit down.
    """
    one = 1 << _RMAT_BITS
    ta = int(round(a * one))
    tb = ta + int(round(b * one))
    tc = tb + int(round(c * one))
    e = torch.arange(lo, hi, dtype=torch.int64, device=device)
    src = torch.zeros_like(e)
    dst = torch.zeros_like(e)
    per_word = 64 // _RMAT_BITS
    words = (scale + per_word - 1) // per_word
    level = 0
    for w in range(words):
        bits = hash_counter(seed, STREAM_GRAPH, e * words + w)
        for k in range(per_word):
            if level == scale:
                break
            r = _lsr(bits, k * _RMAT_BITS) & (one - 1)
            sbit = (r >= tb).to(torch.int64)
            dbit = (((r >= ta) & (r < tb)) | (r >= tc)).to(torch.int64)
            src = (src << 1) | sbit
            dst = (dst << 1) | dbit
            level += 1
    return src, dst


def id_bijection(seed: int, n: int, device="cpu") -> torch.Tensor:
    """A seeded bijection on [0, n): raw id -> scrambled id (int64[n]).

    Raw R-MAT ids correlate degree with bit pattern; this removes that.
    """
    i = torch.arange(n, dtype=torch.int64, device=device)
    key = _lsr(hash_counter(seed, STREAM_IDPERM, i), 1)
    order = torch.sort(key, stable=True).indices  # order[rank] = raw id
    out = torch.empty_like(order)
    out[order] = i
    return out


EdgeBatchFn = Callable[[int], Tuple[torch.Tensor, torch.Tensor]]


@dataclass
class EdgeSource:
    """A graph as a sequence of edge batches that can be replayed.

    `batch(k)` returns (src, dst) int64 tensors of batch k, already passed
    through `relabel` (a raw-id -> id map, or None).  Replaying gives the
    same edges, so a CSR can be built in two passes without holding an edge
    list.
    """
    n: int
    num_batches: int
    raw_batch: EdgeBatchFn
    relabel: Optional[torch.Tensor] = None

    def batch(self, k: int) -> Tuple[torch.Tensor, torch.Tensor]:
        s, d = self.raw_batch(k)
        if self.relabel is not None:
            s, d = self.relabel[s], self.relabel[d]
        return s, d

    def with_relabel(self, new_of_old: torch.Tensor) -> "EdgeSource":
        """Compose a further relabelling (old id -> new id) on top."""
        m = new_of_old.to(torch.int64)
        if self.relabel is not None:
            m = m[self.relabel]
        return EdgeSource(self.n, self.num_batches, self.raw_batch, m)


def uniform_graph(seed: int, n: int, e: int, device="cpu", batch_edges: int = 1 << 26) -> EdgeSource:
    nb = max(1, (e + batch_edges - 1) // batch_edges)

    def raw(k):
        return uniform_edges(seed, n, k * batch_edges, min(e, (k + 1) * batch_edges), device)

    return EdgeSource(n, nb, raw)


def rmat_graph(seed: int, scale: int, edge_factor: int, *, random_ids: bool = False,
               self_loops: bool = False, device="cpu", batch_edges: int = 1 << 26,
               a=0.57, b=0.19, c=0.19) -> EdgeSource:
    """R-MAT graph with 2**scale vertices and edge_factor * 2**scale edges.

    random_ids scrambles vertex ids with `id_bijection`; self_loops appends
    exactly one (v, v) edge per vertex after the generated edges (generated
    self-edges and multi-edges are kept as they are).
    """
    n = 1 << scale
    e = n * edge_factor
    nb_gen = max(1, (e + batch_edges - 1) // batch_edges)
    nb_loop = max(1, (n + batch_edges - 1) // batch_edges) if self_loops else 0

    def raw(k):
        if k < nb_gen:
            return rmat_edges(seed, scale, k * batch_edges, min(e, (k + 1) * batch_edges), a, b, c, device)
        j = k - nb_gen
        v = torch.arange(j * batch_edges, min(n, (j + 1) * batch_edges), dtype=torch.int64, device=device)
        return v, v

    relabel = id_bijection(seed, n, device) if random_ids else None
    if self_loops and relabel is not None:
        # self-loop batches are id-symmetric; relabelling them is harmless
        pass
    return EdgeSource(n, nb_gen + nb_loop, raw, relabel)


def build_csr(g: EdgeSource, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """CSR by source: (row_offsets int64[n+1], col_indices int32[E]).

    Within a row, destinations keep edge-generation order.  Two passes over
    the replayable batches: out-degree count, then placement.
    """
    n = g.n
    deg = torch.zeros(n, dtype=torch.int64, device=device)
    for k in range(g.num_batches):
        s, _ = g.batch(k)
        deg += torch.bincount(s, minlength=n)
    off = torch.zeros(n + 1, dtype=torch.int64, device=device)
    torch.cumsum(deg, 0, out=off[1:])
    e_total = int(off[-1].item())
    col = torch.empty(e_total, dtype=torch.int32, device=device)
    cursor = off[:-1].clone()
    for k in range(g.num_batches):
        s, d = g.batch(k)
        ss, idx = torch.sort(s, stable=True)
        ds = d[idx].to(torch.int32)
        del idx, d, s
        cnt = torch.bincount(ss, minlength=n)
        run_start = torch.cumsum(cnt, 0) - cnt
        pos = cursor[ss] + (torch.arange(ss.numel(), dtype=torch.int64, device=device) - run_start[ss])
        col[pos] = ds
        cursor += cnt
        del ss, ds, cnt, run_start, pos
    return off, col


# --------------------------------------------------------------------------
# features and parameters
# --------------------------------------------------------------------------

def _u01_open(bits: torch.Tensor) -> torch.Tensor:
    """Top 24 bits -> (2k+1)/2**25 in (0,1), exact in fp32 and fp64."""
    k = _lsr(bits, 40)
    return (2 * k + 1).to(torch.float64) / float(1 << 25)


def features(seed: int, n: int, d: int, dist: str, dtype: torch.dtype, device="cpu",
             rows: Optional[Tuple[int, int]] = None, row_batch: int = 1 << 20,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Feature rows [rows) of the n x d matrix.

    dist: "uniform" (U[-1,1], 24-bit grid) or "normal" (N(0,1), Box-Muller
    in fp64).  Element (i, j) depends only on (seed, i, j).  The result is
    rounded to `dtype` (fp32 or bf16, round-to-nearest-even); for bf16
    configs those rounded values are the inputs of every implementation.
    """
    lo, hi = rows if rows is not None else (0, n)
    if out is None:
        out = torch.empty((hi - lo, d), dtype=dtype, device=device)
    for r0 in range(lo, hi, row_batch):
        r1 = min(hi, r0 + row_batch)
        ctr = torch.arange(r0 * d, r1 * d, dtype=torch.int64, device=device)
        if dist == "uniform":
            v = 2.0 * _u01_open(hash_counter(seed, STREAM_FEATURES, ctr)) - 1.0
        elif dist == "normal":
            u1 = _u01_open(hash_counter(seed, STREAM_FEATURES, 2 * ctr))
            u2 = _u01_open(hash_counter(seed, STREAM_FEATURES, 2 * ctr + 1))
            v = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)
        else:
            raise ValueError(dist)
        out[r0 - lo:r1 - lo] = v.view(r1 - r0, d).to(dtype)
    return out


def _uniform_param(seed: int, stream: int, shape, bound: float) -> torch.Tensor:
    numel = 1
    for s in shape:
        numel *= s
    ctr = torch.arange(numel, dtype=torch.int64)
    v = (2.0 * _u01_open(hash_counter(seed, stream, ctr)) - 1.0) * bound
    return v.view(*shape)


@dataclass
class LayerParams:
    """Parameters of one layer, fp64 master copies (round before use).

    W is row-major [K, d_out]: K = 2*d_in for SAGE (rows 0..d_in-1 multiply
    the vertex's own embedding, rows d_in.. multiply the neighbour mean),
    K = d_in otherwise.  GAT: column block k*(d_out/heads).. belongs to head
    k; attn_src / attn_dst are [heads, d_out/heads].
    """
    W: Optional[torch.Tensor]        # None: a layer without parameters (SGC propagation hop)
    bias: Optional[torch.Tensor]
    attn_src: Optional[torch.Tensor] = None
    attn_dst: Optional[torch.Tensor] = None

    def rounded(self, dtype: torch.dtype) -> "LayerParams":
        r = lambda t: None if t is None else t.to(dtype).to(torch.float64)
        return LayerParams(r(self.W), r(self.bias), r(self.attn_src), r(self.attn_dst))


def layer_params(seed: int, layer: int, model: str, d_in: int, d_out: int, heads: int = 1) -> LayerParams:
    """Xavier-uniform weights, bias U(-0.1, 0.1)."""
    base = STREAM_WEIGHTS + 4 * layer
    bias = _uniform_param(seed, base + 1, (d_out,), 0.1)
    if model == "sage":
        a = math.sqrt(6.0 / (d_in + d_out))
        W = _uniform_param(seed, base, (2 * d_in, d_out), a)
        return LayerParams(W, bias)
    if model in ("gcn", "gin"):
        a = math.sqrt(6.0 / (d_in + d_out))
        return LayerParams(_uniform_param(seed, base, (d_in, d_out), a), bias)
    if model == "sgc_hop":   # propagation only: no parameters
        return LayerParams(None, None)
    if model == "gat":
        dh = d_out // heads
        a = math.sqrt(6.0 / (d_in + dh))
        W = _uniform_param(seed, base, (d_in, d_out), a)
        aa = math.sqrt(6.0 / (dh + 1))
        return LayerParams(W, bias, _uniform_param(seed, base + 2, (heads, dh), aa),
                           _uniform_param(seed, base + 3, (heads, dh), aa))
    raise ValueError(model)


def edge_keys(seed: int, num_edges: int, device="cpu", bits: int = 32) -> torch.Tensor:
    """One random key per edge (uint32 values held in an int32 tensor, edge e's
    key is a function of (seed, e) only), for neighbourhood sampling.  `bits`
    < 32 leaves few distinct values, i.e. many ties."""
    e = torch.arange(num_edges, dtype=torch.int64, device=device)
    k = _lsr(hash_counter(seed, STREAM_SAMPLING, e), 64 - bits)
    return (k & 0xFFFFFFFF).to(torch.int32) if bits < 32 else ((k ^ 0x80000000) - 0x80000000).to(torch.int32)


# --------------------------------------------------------------------------
# small helpers that only move data
# --------------------------------------------------------------------------

def permute_rows(x: torch.Tensor, new_of_old: torch.Tensor) -> torch.Tensor:
    """X'[new_of_old[v]] = X[v]."""
    out = torch.empty_like(x)
    out[new_of_old.to(torch.int64)] = x
    return out


def in_edges_of(off: torch.Tensor, col: torch.Tensor, dst_ids: torch.Tensor,
                batch_edges: int = 1 << 27) -> Tuple[torch.Tensor, torch.Tensor]:
    """In-neighbour lists of a few destinations, extracted from a CSR by source.

    Returns (in_off int64[len(dst_ids)+1], in_src int32[...]) with sources in
    ascending order (duplicates kept) for each destination in `dst_ids` order.
    Pure data movement: a filter over the edge array, used to hand a sample of
    a very large graph to a checker that cannot hold all of it.
    """
    dev = col.device
    n = off.numel() - 1
    dst_ids = dst_ids.to(device=dev, dtype=torch.int64)
    slot = torch.full((n,), -1, dtype=torch.int64, device=dev)
    slot[dst_ids] = torch.arange(dst_ids.numel(), dtype=torch.int64, device=dev)
    srcs, slots = [], []
    e_total = col.numel()
    for e0 in range(0, e_total, batch_edges):
        e1 = min(e_total, e0 + batch_edges)
        sl = slot[col[e0:e1].to(torch.int64)]
        hit = torch.nonzero(sl >= 0).squeeze(1)
        if hit.numel():
            eid = hit + e0
            srcs.append(torch.searchsorted(off, eid, right=True) - 1)
            slots.append(sl[hit])
    if srcs:
        src = torch.cat(srcs)
        sl = torch.cat(slots)
    else:
        src = torch.zeros(0, dtype=torch.int64, device=dev)
        sl = torch.zeros(0, dtype=torch.int64, device=dev)
    key = sl * n + src
    order = torch.sort(key, stable=True).indices
    src, sl = src[order], sl[order]
    cnt = torch.bincount(sl, minlength=dst_ids.numel())
    in_off = torch.zeros(dst_ids.numel() + 1, dtype=torch.int64, device=dev)
    torch.cumsum(cnt, 0, out=in_off[1:])
    return in_off, src.to(torch.int32)


def sample_subgraph(off: torch.Tensor, col: torch.Tensor, dst_ids: torch.Tensor):
    """The in-edges of a few destinations as a small self-contained problem.

    Returns (in_off, in_src_local, need, dst_local): `need` lists, ascending, the
    vertices that occur as a picked destination or as one of their in-neighbours;
    rows of per-vertex arrays are taken at `need` (X[need], indeg[need]) and every
    id is renumbered to its position in `need`: in_src_local holds the sources of
    in_edges_of(off, col, dst_ids) in that numbering, dst_local the destinations.
    Pure data movement, like in_edges_of: no degree, sum or normalisation is
    computed here.
    """
    dev = col.device
    n = off.numel() - 1
    dst_ids = dst_ids.to(device=dev, dtype=torch.int64)
    in_off, in_src = in_edges_of(off, col, dst_ids)
    need = torch.unique(torch.cat([in_src.to(torch.int64), dst_ids]))
    local = torch.full((n,), -1, dtype=torch.int64, device=dev)
    local[need] = torch.arange(need.numel(), dtype=torch.int64, device=dev)
    return in_off, local[in_src.to(torch.int64)].to(torch.int32), need, local[dst_ids]
