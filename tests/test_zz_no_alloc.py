"""The entry point that allocates nothing: atlas_reorder_indegree_desc_noalloc
against atlas_reorder_indegree_desc, bit for bit, on two calls in a row (the
second with a smaller input, so the scratch still holds the first call's
contents), with ties, isolated vertices and a ragged size; sizes beyond the
fixed scratch are refused."""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu


def _degrees(atlas, seed, scale, ef):
    dev = torch.device("cuda:0")
    g = gen.rmat_graph(seed, scale, ef)
    off, col = gen.build_csr(g)
    off, col = off.to(dev), col.to(dev)
    n = off.numel() - 1
    indeg = torch.empty(n, dtype=torch.int32, device=dev)
    atlas.atlas_in_degree(atlas.make_graph(n, col.numel(), off, col), indeg)
    torch.cuda.synchronize()
    return off, col, indeg


def _both(atlas, off, col, indeg, n):
    """Permutations of the first n vertices' degrees from both entry points."""
    dev = indeg.device
    g = atlas.make_graph(n, 0, off, col, indeg)
    ref_new = torch.full((n,), -1, dtype=torch.int32, device=dev)
    ref_old = torch.full((n,), -1, dtype=torch.int32, device=dev)
    atlas.atlas_reorder_indegree_desc(g, ref_new, ref_old)
    got_new = torch.full((n,), -1, dtype=torch.int32, device=dev)
    got_old = torch.full((n,), -1, dtype=torch.int32, device=dev)
    atlas.atlas_reorder_indegree_desc_noalloc(g, got_new, got_old)
    torch.cuda.synchronize()
    return ref_new, ref_old, got_new, got_old


def test_no_alloc_reorder_matches_and_reuses_scratch(oracle):
    import paper_2605_09402_amd as atlas
    off, col, indeg = _degrees(atlas, 0x5EED0101, 17, 8)
    n_big = off.numel() - 1
    for n in (n_big, 40_003, 1, n_big - 1):          # larger, smaller (ragged), one vertex, larger again
        ref_new, ref_old, got_new, got_old = _both(atlas, off, col, indeg, n)
        assert torch.equal(got_old, ref_old), "old_of_new differs at n=%d" % n
        assert torch.equal(got_new, ref_new), "new_of_old differs at n=%d" % n
        # and both are the oracle's stable degree sort
        o_new, o_old = oracle.reorder_indegree_desc(indeg[:n].cpu().numpy().astype(np.int64))
        assert np.array_equal(got_old.cpu().numpy(), o_old) and np.array_equal(got_new.cpu().numpy(), o_new)


def test_no_alloc_reorder_on_a_side_stream_and_limits():
    import paper_2605_09402_amd as atlas
    dev = torch.device("cuda:0")
    off, col, indeg = _degrees(atlas, 0x5EED0102, 12, 4)
    n = off.numel() - 1
    g = atlas.make_graph(n, 0, off, col, indeg)
    ref_new = torch.empty(n, dtype=torch.int32, device=dev)
    ref_old = torch.empty(n, dtype=torch.int32, device=dev)
    atlas.atlas_reorder_indegree_desc(g, ref_new, ref_old)
    s = torch.cuda.Stream()
    got_new = torch.empty(n, dtype=torch.int32, device=dev)
    got_old = torch.empty(n, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    atlas.atlas_reorder_indegree_desc_noalloc(g, got_new, got_old, s)
    s.synchronize()
    assert torch.equal(got_old, ref_old) and torch.equal(got_new, ref_new)
    # empty input: nothing to do; beyond the fixed scratch: refused, nothing launched
    atlas.atlas_reorder_indegree_desc_noalloc(atlas.make_graph(0, 0, off, col, indeg), got_new, got_old)
    too_many = atlas.NOALLOC_MAX_VERTICES + 1
    with pytest.raises(atlas.AtlasError) as ei:
        atlas.atlas_reorder_indegree_desc_noalloc(atlas.make_graph(too_many, 0, off, col, indeg), got_new, got_old)
    assert ei.value.status == atlas.E_TOO_LARGE
    with pytest.raises(atlas.AtlasError) as ei:
        atlas.atlas_reorder_indegree_desc_noalloc(atlas.make_graph(n, 0, off, col, None), got_new, got_old)
    assert ei.value.status == atlas.E_NULL
    # the limit itself fits the scratch
    big = torch.randint(0, 1000, (atlas.NOALLOC_MAX_VERTICES,), dtype=torch.int32, device=dev)
    gb = atlas.make_graph(big.numel(), 0, off, col, big)
    a_new = torch.empty(big.numel(), dtype=torch.int32, device=dev)
    a_old = torch.empty_like(a_new)
    b_new = torch.empty_like(a_new)
    b_old = torch.empty_like(a_new)
    atlas.atlas_reorder_indegree_desc(gb, a_new, a_old)
    atlas.atlas_reorder_indegree_desc_noalloc(gb, b_new, b_old)
    torch.cuda.synchronize()
    assert torch.equal(a_old, b_old) and torch.equal(a_new, b_new)
