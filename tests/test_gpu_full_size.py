"""The five workloads at their full sizes, generated on the GPU and run through
the C ABI in the launch configuration the benchmark uses (planned chunks, flush
after every chunk), ALL layers, each layer reading the previous one's output.

What is compared with the CPU oracle, on a sample of destinations it computes
one by one with all their in-edges (a random sample plus the vertices of
highest in-degree):
  * integers, bit-exact: in-degree, the pending count after every chunk, and
    the flush in which each sampled vertex became ready (every layer);
  * every layer's output rows, layer by layer in isolation: the oracle's layer
    l is fed the GPU's layer l-1 rows of the sample's vertices and their
    in-neighbours, so an error is pinned to the layer that makes it;
and, over all vertices, what holds at any size: every edge pushed once, every
vertex completed and flushed exactly once, all pending counts zero.

The large workload also runs in the execution its configuration states:
graph and features in pinned host memory, streamed chunk by chunk (long
chunks in pieces) on the library's copy stream, later layers reading the
previous output in device memory."""
import pytest
import torch

from gen import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import harness
    return harness


def _go(oracle, H, wl, plan=True, n_random=1 << 14, sample=None, indeg=None, contracted=None, **kw):
    if sample is None:
        if indeg is None:
            indeg = torch.empty(wl.n, dtype=torch.int32, device=wl.off.device)
            H.atlas.atlas_in_degree(H.atlas.make_graph(wl.n, wl.e, wl.off, wl.col), indeg)
        sample = H.draw_sample(wl, indeg, n_random=n_random)
    run = H.run_workload(wl, plan=plan, sample=sample, indeg=indeg, **kw)
    assert len(run.outs) == len(wl.layers)
    if contracted is not None:   # a plan with a dense part: it exists, and its edges went the expected way
        assert run.plan_info["dense_edges"] > 0 and run.plan_info["dense_cells"] >= 64 * run.plan_info["dense_rows"]
        for st in run.stats:
            assert st["edges_contracted"] == (run.plan_info["dense_edges"] if contracted else 0)
        print("dense part:", run.plan_info, flush=True)
    H.check_layer_counters(wl, run, planned=plan)
    H.check_sampled_integers(oracle, wl, run, sample)
    errs = H.check_sampled_layers(oracle, wl, run, sample)
    print("%s plan=%s %s: sampled %d destinations / %d in-edges, per-layer errors %s" %
          (wl.name, plan, kw, sample.pick.numel(), sample.edges, ["%.2e" % v for v in errs]), flush=True)
    del run
    torch.cuda.empty_cache()
    H.atlas.atlas_release_cache()
    return sample


def test_config1_full(oracle, H):
    _go(oracle, H, workloads.config1("cuda:0"))


@pytest.mark.parametrize("order", ["random_ids", "indegree_desc"])
def test_config2_gcn_scale20(oracle, H, order):
    wl = workloads.config2("cuda:0", reorder=H.gpu_reorder if order == "indegree_desc" else None)
    assert wl.n == 1 << 20 and wl.e == 17 * (1 << 20) and wl.chunk == 1 << 16
    s = _go(oracle, H, wl)
    _go(oracle, H, wl, plan=False, sample=s)


def test_config3_sage_scale22_bf16(oracle, H):
    wl = workloads.config3("cuda:0")
    assert wl.n == 1 << 22 and wl.e == 25 * (1 << 22) and wl.chunk == 1 << 18 and wl.dims == [256, 256, 256, 128]
    s = _go(oracle, H, wl)
    # the same with a dense part in the plan: the ids are not degree-ordered, so the region is whatever the
    # first chunk happens to hold at one edge per 4,096 cells; rows of 256 features are wider than the
    # contraction takes, so the part is pushed as the planned chunk it also is
    _go(oracle, H, wl, sample=s, planned_only=True, plan_dense=(8 << 30, 4096), contracted=False)


def test_config4_gat_scale22(oracle, H):
    wl = workloads.config4("cuda:0")
    assert wl.n == 1 << 22 and wl.e == 16 * (1 << 22) and wl.heads == 4 and len(wl.layers) == 2
    _go(oracle, H, wl)


def test_config5_sage_scale26_bf16(oracle, H):
    """The benchmark's workload, three layers, in both executions the benchmark times.
    Device-resident: resident embeddings, every chunk planned (no zero fill at the layer
    start), plan in plain destination order with the first chunk's dense corner (up to 32 GB of
    cells at the library's default density) contracted on the matrix cores in all three layers.  As the configuration states it: CSR and
    features in pinned host memory, plan in pinned host memory except the first chunk's dense
    corner (device memory), chunks streamed on the copy stream (the first one in pieces), later
    layers fed from device memory.  The oracle computes
    2^18 random destinations and the 1,024 of highest in-degree, about 1.2e8 in-edges, for each
    of the three layers of both runs."""
    wl = workloads.config5("cuda:0", reorder=H.gpu_reorder)
    assert wl.n == 1 << 26 and wl.e == 1 << 31 and wl.chunk == 1 << 22 and wl.dims == [128, 128, 128, 64]
    s = _go(oracle, H, wl, emb_resident=True, n_random=1 << 18, planned_only=True, plan_dense=(32 * 10 ** 9, 0),
            contracted=True)
    _go(oracle, H, wl, sample=s, emb_resident=True, planned_only=True, pinned=True, plan_dense=(32 * 10 ** 9, 0),
        contracted=True)
