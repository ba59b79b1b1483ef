"""Seeded random combinations of graph shape, layer type, storage type, chunk
size and the library's options (plan kind, residency, zero-fill-free start,
flush cadence, run length, piece size, transform-first, bounded store, dense part of the first chunk), each
checked against the oracle: outputs to the storage type's tolerance and the
layer counters exactly.  The single-option cases live in the other files; this
one looks for interactions."""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu

SEED = 0x5EED0300


@pytest.fixture(scope="module")
def H():
    import harness
    return harness


def _degree_ordered(oracle, g):
    off, col = gen.build_csr(g)
    new_of_old, _ = oracle.reorder_indegree_desc(oracle.in_degree(g.n, col.numpy()))
    return g.with_relabel(torch.from_numpy(new_of_old.astype(np.int64)))


def _draw_gat(rng, oracle, H, idx):
    """GAT: plain plan or none, graph in HBM or in pinned host memory."""
    g = gen.rmat_graph(SEED + idx, int(rng.integers(8, 12)), int(rng.integers(4, 20)), random_ids=bool(rng.random() < 0.5))
    if rng.random() < 0.5:
        g = _degree_ordered(oracle, g)
    heads = int(rng.choice([1, 2, 4]))
    dims = [int(rng.choice([64, 128])), int(rng.choice([64, 128])), int(rng.choice([64, 128]))]
    store = [torch.float32, torch.float32, torch.bfloat16, torch.float16][int(rng.integers(4))]
    case = H.make_case("gat", g, SEED + idx, dims, int(rng.integers(37, max(38, g.n // 2))), store=store,
                       feat="normal" if store == torch.float32 else "uniform", act="elu", heads=heads)
    opts = {"flush_every": int(rng.choice([1, 2, 5]))}
    if rng.random() < 0.6:
        opts["plan"] = True
    if rng.random() < 0.4:
        opts["pinned_host"] = True
        opts["device_later"] = bool(rng.random() < 0.5)
    return case, opts, {"run": int(rng.choice([0, 2, 5, 8])), "piece": 0}


def _draw_sgc(rng, oracle, H, idx, store):
    """SGC: two propagation-only hops and a final GCN layer on a graph with self loops."""
    if store == torch.float16:
        store = torch.bfloat16
    g = gen.rmat_graph(SEED + idx, int(rng.integers(8, 12)), int(rng.integers(4, 20)), random_ids=True, self_loops=True)
    d = int(rng.choice([64, 128, 256]))
    case = H.make_case("sgc", g, SEED + idx, [d, d, d, int(rng.choice([16, 48, 64]))],
                       int(rng.integers(37, max(38, g.n // 2))), store=store,
                       feat="normal" if store == torch.float32 else "uniform")
    opts = {"flush_every": int(rng.choice([1, 2, 5]))}
    if rng.random() < 0.6:
        opts["plan"] = True
        if rng.random() < 0.5:
            opts["planned_only"] = True
    return case, opts, {"run": int(rng.choice([0, 2, 5, 8])), "piece": 0}


def _draw(rng, oracle, H, idx, handed=False):
    """handed: only the combinations in which the flush may leave finished rows to the update as its 16-bit
    operand (SAGE or GCN, 16-bit storage, 128 input features, a plan), drawn with the same other options."""
    model = ["sage", "gcn", "gin", "gat", "sgc"][int(rng.integers(5))]
    store = [torch.float32, torch.bfloat16, torch.float16][int(rng.integers(3))]
    if handed:
        model = ["sage", "gcn"][int(rng.integers(2))]
        store = [torch.bfloat16, torch.float16][int(rng.integers(2))]
    if model == "gat":
        return _draw_gat(rng, oracle, H, idx)
    if model == "sgc":
        return _draw_sgc(rng, oracle, H, idx, store)
    scale = int(rng.integers(8, 12))
    if rng.random() < 0.3 and model != "gcn":   # (GCN is defined on graphs where every vertex has an in-edge)
        n = int(rng.integers(200, 3000))
        g = gen.uniform_graph(SEED + idx, n, int(n * rng.integers(2, 20)))
    else:
        g = gen.rmat_graph(SEED + idx, scale, int(rng.integers(4, 24)), random_ids=bool(rng.random() < 0.4),
                           self_loops=(model == "gcn"))
    if rng.random() < 0.5:   # degree order: hubs first, long groups
        off, col = gen.build_csr(g)
        new_of_old, _ = oracle.reorder_indegree_desc(oracle.in_degree(g.n, col.numpy()))
        g = g.with_relabel(torch.from_numpy(new_of_old.astype(np.int64)))
    d_in = 128 if handed else int(rng.choice([64, 128, 192, 256]))
    if model == "sage" and store == torch.float32:
        d_in = min(d_in, 256)
    dims = [d_in, int(rng.choice([64, 128])), int(rng.choice([16, 48, 64]))]
    chunk = int(rng.integers(37, max(38, g.n // 2)))
    opts = {}
    plan_kind = int(rng.integers(3))          # 0 none, 1 plain, 2 source-blocked
    pinned = bool(rng.random() < 0.4)
    tf = bool(rng.random() < 0.25)
    if handed:
        plan_kind, tf = max(1, plan_kind), False
    if model == "gin" and store == torch.float16:
        tf = True                             # half-precision GIN runs transform-first only
    if tf:
        dims[1] = 64 if dims[1] not in (64, 128) else dims[1]
        dims[2] = 64                          # transform-first needs output widths that are multiples of 64
        opts["transform_first"] = True
    if plan_kind:
        opts["plan"] = True
        if plan_kind == 2:
            opts["plan_block"] = (int(rng.choice([16, 64, 128])), int(rng.choice([4, 8, 24])))
        if rng.random() < 0.5:
            opts["planned_only"] = True
    if pinned:
        opts["pinned_host"] = True
        if plan_kind and rng.random() < 0.5:
            opts["device_later"] = True
    opts["flush_every"] = int(rng.choice([1, 1, 2, 5]))
    case = H.make_case(model, g, SEED + idx, dims, chunk, store=store,
                       feat="normal" if store == torch.float32 else "uniform", eps=0.5 if model == "gin" else 0.0)
    knobs = {"run": int(rng.choice([0, 0, 2, 5, 8, 16])), "piece": int(rng.choice([0, 1, 4]))}
    if plan_kind == 1 and not tf and rng.random() < 0.4:   # bounded store where the chunks fit
        started = int((np.bincount(case.col.numpy(), minlength=case.n) > 0).sum())
        slots = max(1, int(started * rng.uniform(0.6, 0.95)))
        try:
            oracle.hot_store_trace(case.off.numpy(), case.col.numpy(), chunk, slots, model in ("sage", "gin"))
            opts["hot_slots"] = slots
            opts["flush_every"] = 1       # the replay flushes after every chunk; later flushes hold rows longer
        except ValueError:
            pass
    if handed and rng.random() < 0.25:
        opts["no_handover"] = True
    if not plan_kind and rng.random() < 0.3:
        opts["csr_stream"] = True
    if plan_kind and "hot_slots" not in opts and rng.random() < 0.4:
        # the first chunk's dense corner as matrices of 4-bit counts (contracted on the matrix cores where the layer's rows
        # allow it, pushed as a planned chunk otherwise), at three densities
        opts["plan_dense"] = (1 << 30, int(rng.choice([64, 512, 1 << 20])))
        if rng.random() < 0.25:
            opts["no_dense"] = True
    return case, opts, knobs


@pytest.mark.parametrize("idx", range(64))
def test_random_configuration(oracle, H, idx):
    import paper_2605_09402_amd as atlas
    rng = np.random.default_rng(SEED + 1000 + idx)
    case, opts, knobs = _draw(rng, oracle, H, idx, handed=idx >= 48)
    print("config %d: %s %s n=%d e=%d dims=%s chunk=%d %s %s" % (idx, case.model, case.store, case.n, case.e, case.dims,
                                                                case.chunk, opts, knobs), flush=True)
    run = H.run_gpu(case, tiles_per_run=knobs["run"], piece_tiles=knobs["piece"], **opts)
    print("  errors", H.check_outputs(oracle, case, run), flush=True)
    for st in run.stats:
        assert st["edges_processed"] == case.e and st["vertices_flushed"] == case.n
        assert st["vertices_completed"] == case.n and st["sources_processed"] == case.n
        assert st["chunks_planned"] + st["chunks_csr_stream"] == st["num_chunks"]
