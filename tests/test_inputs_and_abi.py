"""CPU checks of the seeded input generators and of the C-ABI library's
exports (no compute calls: there is no GPU here)."""
import ctypes
import os
import re

import numpy as np
import torch

import gen
from gen import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_hash_is_counter_based_and_batch_independent():
    a = gen.rmat_edges(7, 12, 0, 5000)
    b0 = gen.rmat_edges(7, 12, 0, 1234)
    b1 = gen.rmat_edges(7, 12, 1234, 5000)
    assert torch.equal(a[0], torch.cat([b0[0], b1[0]])) and torch.equal(a[1], torch.cat([b0[1], b1[1]]))
    x = gen.features(3, 100, 64, "uniform", torch.float32)
    y = gen.features(3, 100, 64, "uniform", torch.float32, rows=(40, 60))
    assert torch.equal(x[40:60], y)
    assert gen.mix64(torch.tensor([0], dtype=torch.int64)).item() == gen._s64(gen._mix64_int(0))


def test_uniform_graph_has_no_self_edges():
    g = gen.uniform_graph(1, 1000, 20000)
    s, d = g.batch(0)
    assert (s != d).all() and s.min() >= 0 and s.max() < 1000 and d.min() >= 0 and d.max() < 1000


def test_rmat_quadrant_probabilities():
    s, d = gen.rmat_edges(11, 1, 0, 400000)      # one level: src bit, dst bit
    n = float(s.numel())
    pa = ((s == 0) & (d == 0)).sum().item() / n
    pb = ((s == 0) & (d == 1)).sum().item() / n
    pc = ((s == 1) & (d == 0)).sum().item() / n
    assert abs(pa - 0.57) < 5e-3 and abs(pb - 0.19) < 5e-3 and abs(pc - 0.19) < 5e-3


def test_csr_matches_edge_list_and_batches():
    g = gen.rmat_graph(5, 10, 8, random_ids=True, self_loops=True, batch_edges=1000)
    off, col = gen.build_csr(g)
    n = g.n
    assert off[0] == 0 and off[-1] == col.numel() == n * 8 + n
    src = torch.cat([g.batch(k)[0] for k in range(g.num_batches)])
    dst = torch.cat([g.batch(k)[1] for k in range(g.num_batches)])
    order = torch.sort(src, stable=True).indices          # stable: keeps generation order inside a row
    assert torch.equal(col.long(), dst[order])
    assert torch.equal(off[1:] - off[:-1], torch.bincount(src, minlength=n))
    # every vertex got exactly one extra self edge
    loops = (src == dst).long()
    assert int(loops.sum()) >= n
    g1 = gen.rmat_graph(5, 10, 8, random_ids=True, self_loops=True, batch_edges=1 << 20)
    off1, col1 = gen.build_csr(g1)
    assert torch.equal(off, off1) and torch.equal(col, col1)


def test_id_bijection_and_relabel():
    p = gen.id_bijection(9, 4096)
    assert torch.equal(torch.sort(p).values, torch.arange(4096))
    g = gen.rmat_graph(5, 8, 4)
    perm = torch.randperm(256, generator=torch.Generator().manual_seed(1))
    off, col = gen.build_csr(g)
    off2, col2 = gen.build_csr(g.with_relabel(perm))
    src = torch.repeat_interleave(torch.arange(256), off[1:] - off[:-1])
    a = sorted(zip(perm[src].tolist(), perm[col.long()].tolist()))
    src2 = torch.repeat_interleave(torch.arange(256), off2[1:] - off2[:-1])
    b = sorted(zip(src2.tolist(), col2.tolist()))
    assert a == b


def test_in_edges_of_matches_direct_scan():
    g = gen.rmat_graph(6, 9, 8)
    off, col = gen.build_csr(g)
    pick = torch.tensor([0, 3, 77, 511, 200])
    in_off, in_src = gen.in_edges_of(off, col, pick, batch_edges=700)
    src = torch.repeat_interleave(torch.arange(g.n), off[1:] - off[:-1])
    for i, v in enumerate(pick.tolist()):
        ref = torch.sort(src[col.long() == v]).values
        assert torch.equal(in_src[in_off[i]:in_off[i + 1]].long(), ref)


def test_features_and_params_distributions():
    x = gen.features(3, 4000, 64, "uniform", torch.float32)
    assert x.abs().max() < 1 and abs(x.mean()) < 0.01
    z = gen.features(3, 4000, 64, "normal", torch.float32)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    xb = gen.features(3, 100, 64, "uniform", torch.bfloat16)
    assert torch.equal(xb, x[:100].to(torch.bfloat16))
    p = gen.layer_params(1, 0, "sage", 64, 32)
    assert p.W.shape == (128, 32) and p.W.abs().max() <= (6 / 96) ** 0.5 and p.bias.abs().max() <= 0.1
    q = gen.layer_params(1, 0, "gat", 128, 128, 4)
    assert q.attn_src.shape == (4, 32) and q.attn_dst.shape == (4, 32)
    r = p.rounded(torch.bfloat16)
    assert torch.equal(r.W, p.W.to(torch.bfloat16).double())


def test_config1_shape():
    wl = workloads.config1()
    assert wl.n == 10_000 and wl.e == 100_000 and wl.chunk == 1024 and wl.dims == [64, 64, 16]
    assert (wl.n + wl.chunk - 1) // wl.chunk == 10 and wl.n - 9 * wl.chunk == 784


def test_small_config5_with_oracle_ordering(oracle):
    def reorder(off, col):
        new_of_old, _ = oracle.reorder_indegree_desc(oracle.in_degree(off.numel() - 1, col.numpy()))
        return torch.from_numpy(new_of_old.astype(np.int64))
    wl = workloads.config5(scale=10, reorder=reorder)
    indeg = oracle.in_degree(wl.n, wl.col.numpy())
    assert np.all(indeg[:-1] >= indeg[1:])            # ids are in-degree descending
    assert wl.e == 32 * 1024 and wl.X.dtype == torch.bfloat16


def test_library_exports_every_declared_symbol():
    """Every function declared in include/atlas.h is exported by libatlas.so
    (load + symbol lookup only)."""
    import paper_2605_09402_amd as atlas
    header = open(os.path.join(ROOT, "include", "atlas.h")).read()
    declared = set(re.findall(r"\b(atlas_[a-z_0-9]+)\s*\(", header))
    declared -= {"atlas_plan_create on"}  # prose
    assert {"atlas_layer_init", "atlas_broadcast_chunk", "atlas_flush_ready", "atlas_layer_finish"} <= declared
    lib = ctypes.CDLL(atlas.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert set(atlas.EXPORTS) == declared
    lib.atlas_strerror.restype = ctypes.c_char_p
    assert b"ascending" in lib.atlas_strerror(atlas.E_ORDER)
    # struct sizes the binding assumes (LP64)
    assert ctypes.sizeof(atlas.atlas_graph_t) == 56 and ctypes.sizeof(atlas.atlas_weights_t) == 40
    assert ctypes.sizeof(atlas.atlas_dims_t) == 72 and ctypes.sizeof(atlas.atlas_layer_stats_t) == 160
