"""Pins for the oracle's subset mode and for the placement of the activation in a
chain of layers.  No GPU.

Every check of a full-size workload hands the oracle a SAMPLE of destinations
with all their in-edges and renumbered vertex ids (`InLists(..., dst_ids)`).
Here that mode is compared with something that is not the oracle: a dense
adjacency brute force over the WHOLE graph, read at the sampled rows.  The
samples always hold isolated vertices and the vertex of highest in-degree, come
in no particular order, and their renumbered ids differ from the original ones,
so that taking a destination's own row, degree or attention term at its
position in the sample instead of at its vertex id cannot pass.  The last tests
plant exactly such slips in a copy of the oracle's source and require the pins
to catch them.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest
import torch

import gen
from test_oracle_pins import dense_adjacency, dense_gat, tiny_graph, with_self_loops


class Params:
    W = bias = attn_src = attn_dst = None


def _graph(model, seed=41, n=120, e=700):
    """(off, col, src, A) of a tiny multigraph; GCN-like models get one self-edge per vertex."""
    if model in ("gcn", "sgc"):
        off, col, src = tiny_graph(seed, n, e, isolated=0)
        off, src, dst = with_self_loops(n, src, col)
        col = dst.astype(np.int32)
    else:
        off, col, src = tiny_graph(seed, n, e, isolated=4)
    return off, col, src, dense_adjacency(n, src, col)


def _sample(n, A, rng, k=23):
    """Destinations in arbitrary order: random ones, the isolated ones, the heaviest one."""
    deg = A.sum(1)
    pick = set(rng.choice(n, size=k, replace=False).tolist())
    pick |= set(np.nonzero(deg == 0)[0].tolist())
    pick.add(int(np.argmax(deg)))
    pick = np.array(sorted(pick), dtype=np.int64)
    return pick[rng.permutation(pick.size)]


def _subset(oracle, off, col, pick):
    in_off, in_src, need, dst_local = gen.sample_subgraph(torch.from_numpy(off), torch.from_numpy(col),
                                                          torch.from_numpy(pick))
    need = need.numpy()
    il = oracle.InLists(in_off.numpy(), in_src.numpy(), dst_local.numpy())
    # the renumbering must move ids, or the test could not tell a vertex id from a position
    assert need.size < off.size - 1 and (need != np.arange(need.size)).any()
    assert (dst_local.numpy() != np.arange(pick.size)).any()
    return il, need


def dense_layer(model, A, X, p, eps=0.0, slope=0.2):
    """The layer over the whole graph from the dense adjacency, fp64, explicit formulas."""
    n = A.shape[0]
    X = X.astype(np.float64)
    deg = A.sum(1)
    if model == "sage":
        d = X.shape[1]
        mean = np.zeros_like(X)
        for v in range(n):
            if deg[v] > 0:
                mean[v] = (A[v] @ X) / deg[v]
        return X @ p.W[:d] + mean @ p.W[d:] + p.bias
    if model in ("gcn", "sgc"):
        S = np.zeros_like(X)
        for v in range(n):
            for u in range(n):
                if A[v, u]:
                    S[v] += A[v, u] * X[u] / np.sqrt(deg[u] * deg[v])
        return S if p.W is None else S @ p.W + p.bias
    if model == "gin":
        return ((1.0 + eps) * X + A @ X) @ p.W + p.bias
    if model == "gat":
        return dense_gat(n, A, X, p.W, p.bias, p.attn_src, p.attn_dst, slope)
    raise ValueError(model)


def _params(model, rng, d, dout, heads=2):
    p = Params()
    if model == "sgc":
        return p
    p.W = rng.standard_normal((2 * d if model == "sage" else d, dout))
    p.bias = rng.standard_normal(dout)
    if model == "gat":
        p.attn_src = rng.standard_normal((heads, dout // heads))
        p.attn_dst = rng.standard_normal((heads, dout // heads))
    return p


def check_subset_layer(oracle, model, seed=41):
    """The assertion body shared by the pin and by the planted-slip tests."""
    rng = np.random.default_rng(seed)
    off, col, src, A = _graph(model, seed)
    n, d, dout = off.size - 1, 6, 8
    X = rng.standard_normal((n, d)).astype(np.float32)
    p = _params(model, rng, d, dout)
    eps = 0.3 if model == "gin" else 0.0
    pick = _sample(n, A, rng)
    il, need = _subset(oracle, off, col, pick)
    indeg = A.sum(1).astype(np.int64)
    got = oracle.run_layer(model, il, indeg[need], X[need], p, oracle.ACT_NONE, oracle.FMT_F32, 0.2, eps)
    ref = dense_layer(model, A, X, p, eps)[pick]
    # outputs are rounded once to fp32 storage
    assert np.allclose(got, ref.astype(np.float32).astype(np.float64), rtol=1e-6, atol=1e-7), model
    # and the unrounded layer functions agree with the brute force to fp64 accuracy
    if model == "sage":
        raw = oracle.sage_mean(il, X[need], p.W, p.bias)
    elif model == "gcn":
        raw = oracle.gcn(il, indeg[need], X[need], p.W, p.bias)
    elif model == "sgc":
        raw = oracle.sgc_hop(il, indeg[need], X[need])
    elif model == "gin":
        raw = oracle.gin(il, X[need], p.W, p.bias, eps)
    else:
        raw = oracle.gat(il, X[need], p.W, p.bias, p.attn_src, p.attn_dst, 0.2)
    assert np.allclose(raw, ref, rtol=1e-11, atol=1e-11), model
    # the whole-graph mode at the same rows
    full = oracle.run_layer(model, oracle.InLists.from_csr(off, col), indeg, X, p, oracle.ACT_NONE,
                            oracle.FMT_F32, 0.2, eps)
    assert np.allclose(got, full[pick], rtol=1e-12, atol=1e-12), model


@pytest.mark.parametrize("model", ["sage", "gcn", "gin", "sgc", "gat"])
def test_subset_mode_vs_dense(oracle, model):
    check_subset_layer(oracle, model)
    check_subset_layer(oracle, model, seed=43)


def check_subset_counters(oracle, selfmsg, seed=47):
    """Completion chunk and pending counts of sampled destinations (source ids stay the
    streaming ids) against an explicit replay of the message stream over the whole graph."""
    rng = np.random.default_rng(seed)
    n, C = 150, 16
    off, col, src = tiny_graph(seed, n, 900, isolated=5)
    A = dense_adjacency(n, src, col)
    pick = _sample(n, A, rng, k=31)
    in_off, in_src = gen.in_edges_of(torch.from_numpy(off), torch.from_numpy(col), torch.from_numpy(pick))
    il = oracle.InLists(in_off.numpy(), in_src.numpy(), pick)
    pend = A.sum(1).astype(np.int64) + int(selfmsg)
    done_at = np.full(n, -1, dtype=np.int64)
    nchunks = (n + C - 1) // C
    for c in range(nchunks):
        for u in range(c * C, min(n, (c + 1) * C)):
            for e in range(off[u], off[u + 1]):
                pend[col[e]] -= 1
                if pend[col[e]] == 0:
                    done_at[col[e]] = c
            if selfmsg:
                pend[u] -= 1
                if pend[u] == 0:
                    done_at[u] = c
        assert np.array_equal(oracle.pending_after(il, selfmsg, min(n, (c + 1) * C)), pend[pick])
    assert np.array_equal(oracle.completion_chunk(il, selfmsg, C), done_at[pick])


@pytest.mark.parametrize("selfmsg", [False, True])
def test_subset_counters_vs_stream_replay(oracle, selfmsg):
    check_subset_counters(oracle, selfmsg)


# --------------------------------------------------------------------------
# a chain of layers: the activation sits between layers and nowhere else
# --------------------------------------------------------------------------

@pytest.mark.parametrize("model,act", [("sage", "relu"), ("gcn", "relu"), ("gin", "relu"), ("gat", "elu")])
def test_run_model_activation_placement(oracle, model, act):
    rng = np.random.default_rng(53)
    off, col, src, A = _graph(model, 53, n=90, e=500)
    n, dims = off.size - 1, [6, 8, 8, 4]
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    layers = [_params(model, rng, dims[i], dims[i + 1]) for i in range(3)]
    kind = {"relu": oracle.ACT_RELU, "elu": oracle.ACT_ELU}[act]
    outs = oracle.run_model(model, off, col, X, layers, kind, oracle.FMT_F32)
    cur = X
    for li, p in enumerate(layers):
        y = dense_layer(model, A, cur, p)
        if li + 1 < len(layers):                       # between layers only
            y = np.maximum(y, 0.0) if act == "relu" else np.where(y > 0, y, np.expm1(y))
        y = y.astype(np.float32)                       # stored in fp32 between layers
        assert np.allclose(outs[li], y.astype(np.float64), rtol=2e-6, atol=1e-6), (model, li)
        cur = y
    # the check can tell: hidden layers are clipped, the last one is not
    assert outs[0].min() >= (0.0 if act == "relu" else -1.0) and outs[1].min() >= (0.0 if act == "relu" else -1.0)
    assert outs[2].min() < (-1e-3 if act == "relu" else -1.0)


# --------------------------------------------------------------------------
# planted slips: a copy of the oracle with one index wrong must fail the pins
# --------------------------------------------------------------------------

SLIPS = [
    # (what, text in the source, replacement, pin that must fail)
    ("SAGE own row taken at the sample position", "A[i * 2 * d + k] = (double)X[v * d + k];",
     "A[i * 2 * d + k] = (double)X[i * d + k];", lambda o: check_subset_layer(o, "sage")),
    ("GCN / SGC destination degree taken at the sample position", "(double)indeg[u] * (double)indeg[v]",
     "(double)indeg[u] * (double)indeg[i]", lambda o: (check_subset_layer(o, "gcn"))),
    ("SGC destination degree taken at the sample position", "(double)indeg[u] * (double)indeg[v]",
     "(double)indeg[u] * (double)indeg[i]", lambda o: (check_subset_layer(o, "sgc"))),
    ("GIN own row taken at the sample position", "(1.0 + eps) * (double)X[v * d + k]",
     "(1.0 + eps) * (double)X[i * d + k]", lambda o: check_subset_layer(o, "gin")),
    ("GAT destination term taken at the sample position", "er += ad[k] * Z[v * dout + h * dh + k]",
     "er += ad[k] * Z[i * dout + h * dh + k]", lambda o: check_subset_layer(o, "gat")),
    ("self message compared at the sample position", "int64_t last = selfmsg ? v : -1;",
     "int64_t last = selfmsg ? i : -1;", lambda o: check_subset_counters(o, True)),
    ("own chunk of a pending count taken at the sample position", "if (selfmsg && v < bound) got += 1;",
     "if (selfmsg && i < bound) got += 1;", lambda o: check_subset_counters(o, True)),
    ("mean divides by a wrong count", "deg > 0 ? S[i * d + k] / (double)deg : 0.0",
     "deg > 0 ? S[i * d + k] / (double)(deg + 1) : 0.0", lambda o: check_subset_layer(o, "sage")),
]


@pytest.mark.parametrize("what,old,new,pin", SLIPS, ids=[s[0] for s in SLIPS])
def test_planted_slip_is_caught(oracle, tmp_path, monkeypatch, what, old, new, pin):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "atlas_oracle.c")).read()
    assert src.count(old) >= 1, "the oracle no longer contains the statement this test mutates"
    mutant_c = tmp_path / "mutant.c"
    mutant_c.write_text(src.replace(old, new))
    mutant_so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off", "-o",
                           str(mutant_so), str(mutant_c), "-lm"])
    pin(oracle)                                   # the oracle as it stands passes
    bad = ctypes.CDLL(str(mutant_so))
    bad.ao_num_threads.restype = ctypes.c_int
    monkeypatch.setattr(oracle, "_lib", bad)
    with pytest.raises(AssertionError):
        pin(oracle)
