"""GPU edge cases: degenerate graphs, width sweep, residency and API errors.
All through the C ABI, all against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu
SEED = 0x5EED0100


@pytest.fixture(scope="module")
def H():
    import harness
    return harness


@pytest.fixture(scope="module")
def atlas():
    import paper_2605_09402_amd as a
    a.lib()
    return a


def both_paths(H, oracle, case, ints=True, **kw):
    for plan, lazy in ((False, False), (True, False), (True, True)):
        if lazy and case.model == "gat":
            continue
        run = H.run_gpu(case, snapshots=ints, plan=plan, planned_only=lazy, **kw)
        if ints:
            for li in range(len(case.layers)):
                H.check_integers(oracle, case, run, layer=li)
        H.check_outputs(oracle, case, run)
        for st in run.stats:
            assert st["edges_processed"] == case.e and st["vertices_flushed"] == case.n


@pytest.mark.parametrize("model", ["sage", "gcn", "gin"])
def test_no_edges(oracle, H, model):
    """N vertices, E = 0: SAGE and GIN complete by self messages, GCN at layer start."""
    case = H.case_from_edges(model, 300, [], [], SEED, [64, 32], 128)
    both_paths(H, oracle, case)


def test_hot_source_and_hot_destination(oracle, H):
    """One source with 70,000 out-edges and one destination with 70,000
    in-edges (groups spanning >1,000 tiles; multi-edges), plus a sparse rest."""
    n = 50_000
    rng = np.random.default_rng(3)
    hub_out = rng.integers(0, n, 70_000)
    hub_in = rng.integers(0, n, 70_000)
    rest_s = rng.integers(0, n, 30_000)
    rest_d = rng.integers(0, n, 30_000)
    src = np.concatenate([np.full(70_000, 17), hub_in, rest_s, np.full(500, 4242)])
    dst = np.concatenate([hub_out, np.full(70_000, 31_000), rest_d, np.full(500, 99)])   # 500 copies of 4242 -> 99
    case = H.case_from_edges("sage", n, src, dst, SEED + 1, [128, 64], 4096)
    both_paths(H, oracle, case)


@pytest.mark.parametrize("model", ["gat", "sage", "gcn"])
def test_group_starting_on_a_tile_boundary(oracle, H, model):
    """Per chunk, destination 5 gets exactly 64 messages (one full 64-edge tile
    of the destination-ordered list), destination 6 the next 100 (its group
    starts on the first edge of a tile and is cut by the next boundary) and
    destination 7 another 28; three chunks, so the running softmax state of the
    cut destination is rescaled twice.  GCN gets its self loops at the end."""
    n, chunk = 600, 200
    src, dst = [], []
    for c in range(3):
        base = c * chunk
        src += list(range(base, base + 64)) + list(range(base + 10, base + 110)) + list(range(base + 150, base + 178))
        dst += [5] * 64 + [6] * 100 + [7] * 28
    if model == "gcn":
        src += list(range(n))
        dst += list(range(n))
    kw = dict(feat="normal", act="elu", heads=2) if model == "gat" else {}
    case = H.case_from_edges(model, n, src, dst, SEED + 31, [64, 64, 64] if model == "gat" else [64, 32], chunk, **kw)
    both_paths(H, oracle, case)


def test_long_runs_of_sources_without_edges(oracle, H):
    """Every 150th source has one out-edge: a 64-edge tile spans ~9,600 sources."""
    n = 40_000
    src = np.arange(0, n, 150)
    dst = (src * 7 + 3) % n
    case = H.case_from_edges("gcn", n, np.concatenate([src, np.arange(n)]), np.concatenate([dst, np.arange(n)]),
                             SEED + 2, [64, 16], 16_384)
    both_paths(H, oracle, case)


@pytest.mark.parametrize("store", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("d_in,d_out", [(64, 16), (192, 48), (256, 160), (512, 256), (128, 96)])
def test_width_sweep(oracle, H, d_in, d_out, store):
    if store == torch.float32 and d_in == 512:
        d_in = 256   # fp32 SAGE tile of K = 1024 does not fit LDS; K = 512 is the fp32 limit
    g = gen.rmat_graph(SEED + d_in + d_out, 11, 8)
    for model in ("sage", "gcn"):
        case = H.make_case(model, g, SEED + d_in, [d_in, d_out], 600, store=store,
                           feat="normal" if store == torch.float32 else "uniform")
        if model == "gcn":   # GCN needs D > 0 everywhere: add the self loops
            case = H.make_case(model, gen.rmat_graph(SEED + d_in + d_out, 11, 8, self_loops=True), SEED + d_in,
                               [d_in, d_out], 600, store=store)
        both_paths(H, oracle, case, ints=False)


def test_unaligned_chunks_fall_back_to_csr_stream(oracle, H):
    """Plan built for 1,000-source chunks, layer streamed in 768-source chunks."""
    case = H.make_case("sage", gen.rmat_graph(SEED + 9, 12, 16), SEED + 9, [128, 64], 768)
    run = H.run_gpu(case, snapshots=True, plan=True, plan_chunk=1000)
    H.check_integers(oracle, case, run)
    H.check_outputs(oracle, case, run)


@pytest.mark.parametrize("model,store", [("sage", torch.bfloat16), ("gcn", torch.float32)])
def test_pinned_host_residency(oracle, H, model, store):
    """Graph and layer-0 features in pinned host memory, staged chunk by chunk
    on the library's copy stream (a ring of staging slots)."""
    g = gen.rmat_graph(SEED + 11, 12, 16, self_loops=(model == "gcn"))
    case = H.make_case(model, g, SEED + 11, [128, 128, 64], 500, store=store)
    run = H.run_gpu(case, snapshots=True, pinned_host=True)
    H.check_integers(oracle, case, run)
    H.check_outputs(oracle, case, run)
    row = 128 * (2 if store == torch.bfloat16 else 4)
    assert run.stats[0]["bytes_copied_h2d"] == case.n * row + case.e * 4 + (case.n + 1) * 8
    run2 = H.run_gpu(case, pinned_host=True, flush_every=3)     # no host sync between chunks
    H.check_outputs(oracle, case, run2)
    # with a plan the regrouped chunks are what is streamed (the plan itself sits in pinned host memory)
    run3 = H.run_gpu(case, snapshots=True, pinned_host=True, plan=True)
    H.check_integers(oracle, case, run3)
    H.check_outputs(oracle, case, run3)
    # rows + 3 bytes per edge + group and tile arrays; the row offsets came over once, with the plan
    assert case.n * row + case.e * 3 < run3.stats[0]["bytes_copied_h2d"] < case.n * row + case.e * 4 + (case.n + 1) * 8
    run4 = H.run_gpu(case, pinned_host=True, plan=True, flush_every=5, planned_only=True)
    H.check_outputs(oracle, case, run4)
    # graph in pinned host memory, layer 2 reads layer 1's output in device memory: only edges are staged
    run5 = H.run_gpu(case, pinned_host=True, plan=True, device_later=True)
    H.check_outputs(oracle, case, run5)
    assert run5.stats[1]["bytes_copied_h2d"] < case.e * 4 + (case.n + 1) * 8
    run6 = H.run_gpu(case, pinned_host=True, device_later=True, emb_resident=True, flush_every=2)
    H.check_outputs(oracle, case, run6)


def test_api_errors(atlas, H):
    dev = torch.device("cuda:0")
    case = H.make_case("sage", gen.uniform_graph(SEED + 20, 1000, 5000), SEED + 20, [64, 16], 256)
    off, col = case.off.to(dev), case.col.to(dev)
    X = case.X.to(dev)
    W = case.layers[0].W.float().to(dev).contiguous()
    b = case.layers[0].bias.float().to(dev).contiguous()
    g = atlas.make_graph(case.n, case.e, off, col)
    wts = atlas.make_weights(W, b, atlas.DTYPE_F32)
    L = atlas.lib()

    def dims(**kw):
        a = dict(model=atlas.MODEL_SAGE_MEAN, d_in=64, d_out=16, in_dtype=0, out_dtype=0, activation=0,
                 max_chunk_sources=256)
        a.update(kw)
        return atlas.make_dims(**a)

    def status(fn, *args):
        with pytest.raises(atlas.AtlasError) as ei:
            fn(*args)
        return ei.value.status

    assert status(atlas.atlas_layer_init, g, dims(d_in=100), wts) == atlas.E_BAD_DIMS
    assert status(atlas.atlas_layer_init, g, dims(d_out=20), wts) == atlas.E_BAD_DIMS
    assert status(atlas.atlas_layer_init, g, dims(model=7), wts) == atlas.E_BAD_DIMS
    assert status(atlas.atlas_layer_init, g, dims(max_chunk_sources=0), wts) == atlas.E_BAD_DIMS
    assert status(atlas.atlas_layer_init, atlas.make_graph(1 << 31, 0, off, col), dims(), wts) == atlas.E_OVERFLOW
    assert status(atlas.atlas_layer_init, atlas.make_graph(case.n, case.e, None, col), dims(), wts) == atlas.E_NULL
    assert L.atlas_layer_init(None, None, None, None, None) == atlas.E_NULL
    assert L.atlas_broadcast_chunk(None, 0, 1, None, None) == atlas.E_NULL
    assert L.atlas_layer_finish(None, None) == atlas.E_NULL

    h = atlas.atlas_layer_init(g, dims(), wts)
    out = torch.zeros((case.n, 16), device=dev)
    assert status(atlas.atlas_broadcast_chunk, h, 256, 512, X[256:512]) == atlas.E_ORDER     # must start at 0
    assert status(atlas.atlas_broadcast_chunk, h, 0, 300, X[0:300]) == atlas.E_RANGE         # longer than max
    assert status(atlas.atlas_broadcast_chunk, h, 0, 0, X[0:1]) == atlas.E_RANGE
    assert status(atlas.atlas_broadcast_chunk, h, -1, 5, X[0:6]) == atlas.E_RANGE
    assert status(atlas.atlas_attention_prepass, h, 0, 256, X[0:256]) == atlas.E_STATE       # not a GAT layer
    atlas.atlas_broadcast_chunk(h, 0, 256, X[0:256])
    assert status(atlas.atlas_broadcast_chunk, h, 0, 256, X[0:256]) == atlas.E_ORDER         # repeated chunk
    assert status(atlas.atlas_broadcast_chunk, h, 300, 400, X[300:400]) == atlas.E_ORDER     # gap
    assert status(atlas.atlas_broadcast_chunk, h, 256, 1001, X[256:]) == atlas.E_RANGE       # past N
    atlas.atlas_flush_ready(h, out)
    with pytest.raises(atlas.AtlasError) as ei:      # finish with sources still unbroadcast
        atlas.atlas_layer_finish(h)
    assert ei.value.status == atlas.E_INCOMPLETE and ei.value.stats["sources_processed"] == 256

    # all chunks broadcast but the last flush forgotten
    h = atlas.atlas_layer_init(g, dims(), wts)
    for b0 in range(0, case.n, 256):
        atlas.atlas_broadcast_chunk(h, b0, min(case.n, b0 + 256), X[b0:b0 + 256])
    with pytest.raises(atlas.AtlasError) as ei:
        atlas.atlas_layer_finish(h)
    assert ei.value.status == atlas.E_INCOMPLETE
    assert ei.value.stats["vertices_completed"] == case.n and ei.value.stats["vertices_flushed"] == 0

    # resident-embedding promise broken: second chunk comes from another matrix
    h = atlas.atlas_layer_init(g, dims(flags=atlas.FLAG_EMB_RESIDENT), wts)
    atlas.atlas_broadcast_chunk(h, 0, 256, X[0:256])
    other = X.clone()
    assert status(atlas.atlas_broadcast_chunk, h, 256, 512, other[256:512]) == atlas.E_STATE
    with pytest.raises(atlas.AtlasError):
        atlas.atlas_layer_finish(h)
    assert status(atlas.atlas_plan_create, atlas.make_graph(case.n, case.e, off, col), 0) == atlas.E_BAD_DIMS

    # SGC propagation hop: no weights, but the widths must agree and there is no activation
    none = atlas.make_weights(None, None, atlas.DTYPE_F32)
    sgc = dict(model=atlas.MODEL_SGC_HOP, d_in=64, d_out=64)
    assert status(atlas.atlas_layer_init, g, dims(model=atlas.MODEL_SGC_HOP), none) == atlas.E_BAD_DIMS   # 64 -> 16
    assert status(atlas.atlas_layer_init, g, dims(activation=atlas.ACT_RELU, **sgc), none) == atlas.E_BAD_DIMS
    assert status(atlas.atlas_layer_init, g, dims(model=atlas.MODEL_GIN), none) == atlas.E_NULL   # GIN needs W
    h = atlas.atlas_layer_init(g, dims(**sgc), none)
    with pytest.raises(atlas.AtlasError):
        atlas.atlas_layer_finish(h)

    # planned-only promise broken: the plan was built for 256-source chunks, the caller sends 128
    plan_h = atlas.atlas_plan_create(atlas.make_graph(case.n, case.e, off, col), 256)
    gp = atlas.make_graph(case.n, case.e, off, col, None, atlas.RESIDENT_DEVICE, plan_h)
    h = atlas.atlas_layer_init(gp, dims(flags=atlas.FLAG_PLANNED_ONLY), wts)
    assert status(atlas.atlas_broadcast_chunk, h, 0, 128, X[0:128]) == atlas.E_RANGE
    atlas.atlas_broadcast_chunk(h, 0, 256, X[0:256])
    with pytest.raises(atlas.AtlasError):
        atlas.atlas_layer_finish(h)
    atlas.atlas_plan_destroy(plan_h)
    atlas.atlas_release_cache()


def test_zero_vertices(atlas):
    dev = torch.device("cuda:0")
    off = torch.zeros(1, dtype=torch.int64, device=dev)
    col = torch.zeros(1, dtype=torch.int32, device=dev)
    W = torch.zeros((128, 16), device=dev)
    h = atlas.atlas_layer_init(atlas.make_graph(0, 0, off, col),
                               atlas.make_dims(atlas.MODEL_SAGE_MEAN, 64, 16, 0, 0, 0, 64),
                               atlas.make_weights(W, None, atlas.DTYPE_F32))
    out = torch.zeros((1, 16), device=dev)
    assert atlas.atlas_flush_ready(h, out, count=True) == 0
    st = atlas.atlas_layer_finish(h)
    assert st["vertices_flushed"] == 0 and st["edges_processed"] == 0


@pytest.mark.parametrize("model", ["sage", "gcn"])
@pytest.mark.parametrize("plan", [False, True], ids=["csr_stream", "planned"])
def test_accumulators_alone(oracle, H, atlas, model, plan):
    """The scatter-aggregate step on its own: after all chunks (and before any
    update) the fp32 accumulators equal the oracle's neighbour sums."""
    dev = torch.device("cuda:0")
    g = gen.rmat_graph(SEED + 30, 12, 16, self_loops=(model == "gcn"))
    case = H.make_case(model, g, SEED + 30, [128, 64], 500, feat="normal")
    off, col, X = case.off.to(dev), case.col.to(dev), case.X.to(dev)
    n, e = case.n, case.e
    plan_h = atlas.atlas_plan_create(atlas.make_graph(n, e, off, col), 500) if plan else None
    graph = atlas.make_graph(n, e, off, col, None, atlas.RESIDENT_DEVICE, plan_h)
    p = case.layers[0]
    W, b = p.W.float().to(dev).contiguous(), p.bias.float().to(dev).contiguous()
    h = atlas.atlas_layer_init(graph, atlas.make_dims(H.MODEL_ID[model], 128, 64, 0, 0, 0, 500),
                               atlas.make_weights(W, b, atlas.DTYPE_F32))
    for b0 in range(0, n, 500):
        atlas.atlas_broadcast_chunk(h, b0, min(n, b0 + 500), X[b0:b0 + 500])
    acc = np.empty((n, 128), dtype=np.float32)
    atlas.atlas_debug_copy(h, atlas.DBG_ACC, acc)
    out = torch.empty((n, 64), device=dev)
    atlas.atlas_flush_ready(h, out)
    atlas.atlas_layer_finish(h)
    if plan_h:
        atlas.atlas_plan_destroy(plan_h)
    il = oracle.InLists.from_csr(case.off.numpy(), case.col.numpy())
    scale = None
    if model == "gcn":      # the source side of the symmetric normalisation is applied while pushing
        scale = 1.0 / np.sqrt(oracle.in_degree(n, case.col.numpy()).astype(np.float64))
    ref = oracle.neighbor_sum(il, case.X.numpy(), scale)
    assert H.row_rel_err(acc.astype(np.float64), ref) <= 1e-5


def test_non_default_stream(oracle, H):
    """Every layer call on a non-blocking stream of the caller's (not the default
    stream): device and pinned-host residency, GAT, the bounded store.  The plan
    is built (on the default stream, synchronously) from arrays that are complete
    before the call."""
    import gen
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        g = gen.rmat_graph(SEED + 31, 12, 16)
        sage = H.make_case("sage", g, SEED + 31, [128, 128, 64], 300, store=torch.bfloat16)
        print("side stream sage", H.check_outputs(oracle, sage, H.run_gpu(sage, plan=True, planned_only=True)))
        print("side stream sage pinned", H.check_outputs(oracle, sage, H.run_gpu(sage, plan=True, pinned_host=True)))
        print("side stream sage csr", H.check_outputs(oracle, sage, H.run_gpu(sage, pinned_host=True, flush_every=3)))
        gat = H.make_case("gat", g, SEED + 31, [64, 64, 64], 300, feat="normal", act="elu", heads=2)
        print("side stream gat", H.check_outputs(oracle, gat, H.run_gpu(gat, plan=True)))
        rnd = H.make_case("sage", gen.rmat_graph(SEED + 31, 12, 16, random_ids=True), SEED + 31, [128, 64], 64)
        slots = int((np.bincount(rnd.col.numpy(), minlength=rnd.n) > 0).sum()) // 2
        print("side stream bounded", H.check_outputs(oracle, rnd, H.run_gpu(rnd, plan=True, hot_slots=slots)))
    torch.cuda.synchronize()


@pytest.mark.parametrize("model,store", [("sage", torch.bfloat16), ("gcn", torch.float32), ("gin", torch.float32)])
@pytest.mark.parametrize("piece", [1, 3, 16])
def test_pinned_chunk_in_pieces(oracle, H, atlas, model, store, piece):
    """dims.piece_tiles: a planned chunk of a pinned-host graph arrives in
    pieces of a few tiles and is pushed piece by piece (groups cut by a piece
    boundary, first-touch groups cleared once, ragged last piece), with and
    without the zero-fill-free layer start, source-blocked plans included.
    Degree-ordered R-MAT scale 12, so the first chunk's hub groups span pieces."""
    g = gen.rmat_graph(SEED + 41, 12, 16, self_loops=(model == "gcn"))
    off, col = gen.build_csr(g)
    new_of_old, _ = oracle.reorder_indegree_desc(oracle.in_degree(g.n, col.numpy()))
    g = g.with_relabel(torch.from_numpy(new_of_old.astype(np.int64)))
    case = H.make_case(model, g, SEED + 41, [128, 128, 64], 1024, store=store,
                       feat="normal" if store == torch.float32 else "uniform", eps=0.25 if model == "gin" else 0.0)
    run = H.run_gpu(case, snapshots=True, pinned_host=True, plan=True, piece_tiles=piece)
    H.check_integers(oracle, case, run)
    print("pieces of", piece, model, H.check_outputs(oracle, case, run))
    H.check_outputs(oracle, case, H.run_gpu(case, pinned_host=True, plan=True, planned_only=True, device_later=True,
                                            flush_every=3, piece_tiles=piece))
    H.check_outputs(oracle, case, H.run_gpu(case, pinned_host=True, plan=True, planned_only=True, plan_block=(64, 8),
                                            piece_tiles=piece))
    for st in run.stats:
        assert st["edges_processed"] == case.e and st["vertices_flushed"] == case.n
        assert st["chunks_planned"] == st["num_chunks"]
    with pytest.raises(atlas.AtlasError) as ei:
        H.run_gpu(case, pinned_host=True, plan=True, piece_tiles=-1)
    assert ei.value.status == atlas.E_BAD_DIMS


@pytest.mark.parametrize("piece", [0, 3])
def test_pinned_plan_with_four_byte_words(oracle, H, atlas, piece):
    """A plan of a pinned-host graph keeps its edge words in 3 bytes only for
    chunks of at most 2^23 sources; with a larger chunk size (here one chunk over
    the whole graph) the 4-byte words travel and are read where they were
    staged, whole or in pieces."""
    g = gen.rmat_graph(SEED + 43, 12, 16)
    off, col = gen.build_csr(g)
    new_of_old, _ = oracle.reorder_indegree_desc(oracle.in_degree(g.n, col.numpy()))
    g = g.with_relabel(torch.from_numpy(new_of_old.astype(np.int64)))
    case = H.make_case("sage", g, SEED + 43, [128, 64, 64], (1 << 23) + 1, store=torch.bfloat16, feat="uniform")
    run = H.run_gpu(case, snapshots=True, pinned_host=True, plan=True, piece_tiles=piece)
    H.check_integers(oracle, case, run)
    print("4-byte words, pieces of", piece, H.check_outputs(oracle, case, run))
    assert run.stats[0]["bytes_copied_h2d"] >= case.e * 4 + case.n * 256
    H.check_outputs(oracle, case, H.run_gpu(case, pinned_host=True, plan=True, planned_only=True, device_later=True,
                                            piece_tiles=piece))
    H.check_outputs(oracle, case, H.run_gpu(case, pinned_host=True, plan=True, planned_only=True, plan_block=(64, 8),
                                            piece_tiles=piece))



@pytest.mark.parametrize("ids", ["raw", "degree_ordered", "one_hub"])
@pytest.mark.parametrize("residency", ["device", "pinned_host"])
def test_in_degree_of_a_large_graph(oracle, atlas, ids, residency):
    """Graphs above 2^15 vertices and 2^22 edges in device memory are counted bucket by bucket
    in LDS (buckets of 2^15 ids; a heavy bucket is counted in several slices and merged), host
    edge arrays with one atomic per edge: the whole array against the oracle, bit-exact, with a
    vertex count that is no multiple of the bucket size, with degree-ordered ids (first bucket
    far heavier than the rest), and with every edge pointing at one vertex of the last bucket."""
    dev = torch.device("cuda:0")
    g = gen.rmat_graph(SEED + 61, 18, 20)
    off, col = gen.build_csr(g)
    n = g.n - 12_345                                    # ragged last bucket
    col = col[col < n].contiguous()
    if ids == "degree_ordered":
        new_of_old, _ = oracle.reorder_indegree_desc(oracle.in_degree(n, col.numpy()))
        col = torch.from_numpy(new_of_old)[col.to(torch.int64)].contiguous()
    elif ids == "one_hub":
        col = torch.full_like(col, n - 1)
    e = col.numel()
    assert n > (1 << 15) and e >= (1 << 22)
    col_t = col.to(dev) if residency == "device" else col.pin_memory()
    res = atlas.RESIDENT_DEVICE if residency == "device" else atlas.RESIDENT_PINNED_HOST
    indeg = torch.full((n,), -7, dtype=torch.int32, device=dev)
    atlas.atlas_in_degree(atlas.make_graph(n, e, None, col_t, None, res), indeg)
    torch.cuda.synchronize()
    assert np.array_equal(indeg.cpu().numpy().astype(np.int64), oracle.in_degree(n, col.numpy()))
    # twice in a row: the scratch comes back from the library's cache with the first call's contents
    atlas.atlas_in_degree(atlas.make_graph(n, e, None, col_t, None, res), indeg)
    torch.cuda.synchronize()
    assert np.array_equal(indeg.cpu().numpy().astype(np.int64), oracle.in_degree(n, col.numpy()))


@pytest.mark.parametrize("plan_block", [None, (256, 16)])
def test_in_degree_from_the_plan(oracle, H, atlas, plan_block):
    """atlas_plan_in_degree: group sizes summed over the chunks equal the oracle's in-degree, for
    plain and source-blocked plans (several groups per destination and chunk); a layer on a graph
    with a plan and no in_degree counts this way (checked through the layer's own array); plans
    of pinned-host graphs refuse."""
    dev = torch.device("cuda:0")
    g = gen.rmat_graph(SEED + 67, 13, 24)
    off, col = gen.build_csr(g)
    n, e = g.n, col.numel()
    off_d, col_d = off.to(dev), col.to(dev)
    pg = atlas.make_graph(n, e, off_d, col_d)
    plan = atlas.atlas_plan_create_blocked(pg, 1000, *plan_block) if plan_block else atlas.atlas_plan_create(pg, 1000)
    try:
        indeg = torch.full((n,), -3, dtype=torch.int32, device=dev)
        atlas.atlas_plan_in_degree(plan, indeg)
        torch.cuda.synchronize()
        assert np.array_equal(indeg.cpu().numpy().astype(np.int64), oracle.in_degree(n, col.numpy()))
        info = atlas.atlas_plan_info(plan)
        assert info["num_edges"] == e and info["num_chunks"] == (n + 999) // 1000
        assert info["num_first_groups"] == int((oracle.in_degree(n, col.numpy()) > 0).sum())
    finally:
        atlas.atlas_plan_destroy(plan)
    case = H.make_case("sage", g, SEED + 67, [64, 64], 1000)
    run = H.run_gpu(case, snapshots=True, plan=True, plan_block=plan_block)    # in_degree not given: counted at init
    H.check_integers(oracle, case, run)
    H.check_outputs(oracle, case, run)
    hp = atlas.atlas_plan_create(atlas.make_graph(n, e, off.pin_memory(), col.pin_memory(), None,
                                                  atlas.RESIDENT_PINNED_HOST), 1000)
    try:
        with pytest.raises(atlas.AtlasError) as ei:
            atlas.atlas_plan_in_degree(hp, indeg)
        assert ei.value.status == atlas.E_STATE
    finally:
        atlas.atlas_plan_destroy(hp)


def test_measurement_probes(atlas):
    """The benchmark's bare-kernel probes do what they say: the copy copies, the 2:1 stream
    combines its two inputs, the gather runs over ragged id lists without touching anything but
    its sink, and the dense-row contraction equals rows x W (fp64 matmul of the stored 16-bit
    values, library routine) to the 16-bit output's rounding, for the K-sliced kernel (more than
    128 columns), the generic one, a ragged row count and both 16-bit types; the bare loop of matrix
    instructions leaves the sums its operands imply."""
    dev = torch.device("cuda:0")
    a = torch.randint(-2 ** 31, 2 ** 31 - 1, (1 << 20,), dtype=torch.int32, device=dev)
    b = torch.randint(-2 ** 31, 2 ** 31 - 1, (1 << 20,), dtype=torch.int32, device=dev)
    out = torch.zeros_like(a)
    atlas.atlas_probe_copy(out, a, a.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(out, a)
    atlas.atlas_probe_mix21(out, a, b, a.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(out, a ^ b)
    with pytest.raises(atlas.AtlasError):
        atlas.atlas_probe_copy(out, a, 24)          # not a multiple of 16
    table = torch.randint(0, 255, (4096, 256), dtype=torch.uint8, device=dev)
    sink = torch.zeros(atlas.atlas_probe_gather_sink_bytes() // 4, dtype=torch.int32, device=dev)
    for n_ids in (1, 63, 64, 65, 100_003):
        ids = torch.randint(0, 4096, (n_ids,), dtype=torch.int32, device=dev)
        before = table.clone()
        atlas.atlas_probe_row_gather(table, 4096, ids, n_ids, sink)
        torch.cuda.synchronize()
        assert torch.equal(table, before)
    for dt, tdt in ((atlas.DTYPE_BF16, torch.bfloat16), (atlas.DTYPE_F16, torch.float16)):
        for n_rows, K, d_out in ((1000, 1024, 256), (515, 256, 128), (129, 512, 192)):
            rows = (torch.rand((n_rows, K), device=dev) - 0.5).to(tdt)
            W = (torch.rand((K, d_out), device=dev) - 0.5).to(tdt)
            got = torch.full((n_rows, d_out), float("nan"), dtype=tdt, device=dev)
            atlas.atlas_probe_dense_rows(dt, rows, n_rows, K, d_out, W, got, 2)
            ref = rows.double().cpu().numpy() @ W.double().cpu().numpy()
            err = np.abs(got.double().cpu().numpy() - ref).max() / np.abs(ref).max()
            assert err <= (2.0 ** -8 if tdt == torch.bfloat16 else 2.0 ** -11), (tdt, n_rows, K, d_out, err)
    with pytest.raises(atlas.AtlasError) as ei:
        atlas.atlas_probe_dense_rows(atlas.DTYPE_F32, rows, n_rows, K, d_out, W, got, 1)
    assert ei.value.status == atlas.E_BAD_DIMS
    # the bare matrix-instruction loop: ones times a matrix with two ones in every odd column, four accumulators
    # of 16 values per lane, `iters` rounds: every lane of an odd column folds 4 x 16 x 2 x iters, the others 0
    sink.zero_()
    for wps, iters in ((1, 10), (4, 3)):
        flops = atlas.atlas_probe_mfma(wps, iters, sink)
        torch.cuda.synchronize()
        threads = int(flops / (iters * 4 * 2 * 32 * 32 * 16)) * 64
        assert threads > 0 and threads % 256 == 0 and threads * 4 <= atlas.atlas_probe_gather_sink_bytes()
        got = sink.view(torch.float32)[:threads].cpu().numpy()
        want = np.where(np.arange(threads) % 2 == 1, 128.0 * iters, 0.0)
        assert np.array_equal(got, want)
    with pytest.raises(atlas.AtlasError):
        atlas.atlas_probe_mfma(9, 1, sink)
