"""The five workloads at their full sizes, generated on the GPU, layer 1 run
through the C ABI in the launch configuration the benchmark uses (planned
chunks, flush after every chunk), checked on sampled destinations the CPU
oracle computes one by one (random sample + the highest in-degree vertices)
and on counters that hold at any size.  Deeper layers are checked on the
mid-size chained cases of test_gpu_parity.py: a sampled check of layer 2
would need the oracle's full layer-1 output."""
import pytest
import torch

from gen import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import harness
    return harness


def _go(oracle, H, wl, plan=True, emb_resident=False, n_random=1 << 14, planned_only=False, plan_block=None):
    out, stats, indeg, pend, ready = H.run_workload_layer1(wl, plan, emb_resident, planned_only, plan_block)
    H.check_layer_counters(wl, stats, pend, ready)
    err, nd, ne = H.sampled_layer1_check(oracle, wl, out, indeg, n_random=n_random)
    print("%s plan=%s: sampled %d destinations / %d in-edges, error %.3e" % (wl.name, plan, nd, ne, err))
    del out
    torch.cuda.empty_cache()
    H.atlas.atlas_release_cache()


def test_config1_full(oracle, H):
    _go(oracle, H, workloads.config1("cuda:0"))


@pytest.mark.parametrize("order", ["random_ids", "indegree_desc"])
def test_config2_gcn_scale20(oracle, H, order):
    wl = workloads.config2("cuda:0", reorder=H.gpu_reorder if order == "indegree_desc" else None)
    assert wl.n == 1 << 20 and wl.e == 17 * (1 << 20) and wl.chunk == 1 << 16
    _go(oracle, H, wl)
    _go(oracle, H, wl, plan=False)


def test_config3_sage_scale22_bf16(oracle, H):
    wl = workloads.config3("cuda:0")
    assert wl.n == 1 << 22 and wl.e == 25 * (1 << 22) and wl.chunk == 1 << 18 and wl.dims[0] == 256
    _go(oracle, H, wl)


def test_config4_gat_scale22(oracle, H):
    wl = workloads.config4("cuda:0")
    assert wl.n == 1 << 22 and wl.e == 16 * (1 << 22) and wl.heads == 4
    _go(oracle, H, wl)


def test_config5_sage_scale26_bf16(oracle, H):
    """The benchmark's workload and launch configuration: resident embeddings,
    every chunk planned (no zero fill at the layer start), source-blocked plan
    with 2 MiB of source rows per block and 32 messages per block as the
    threshold for a blocked destination.  The oracle computes 2^20 random
    destinations and the 1,024 of highest in-degree, about 1.4e8 in-edges."""
    wl = workloads.config5("cuda:0", reorder=H.gpu_reorder)
    assert wl.n == 1 << 26 and wl.e == 1 << 31 and wl.chunk == 1 << 22
    block = (2 << 20) // (wl.dims[0] * 2)
    _go(oracle, H, wl, emb_resident=True, n_random=1 << 20, planned_only=True,
        plan_block=(block, 32 * (wl.chunk // block)))
