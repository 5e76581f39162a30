"""The entry point that allocates nothing (ivfr_search_static) against ivfr_search, through the C ABI."""
import numpy as np
import pytest

from helpers import compare_results, tiny_workload

pytestmark = pytest.mark.gpu


def test_static_workspace_search_matches_the_allocating_entry_point():
    import torch
    import paper_1102_3828_amd as pkg
    from test_gpu_parity import gpu_index_from_oracle, queries_dev
    wl = tiny_workload(d=64, G=16, N=30000, n_train=3000, n_query=48, c=12, m=8, m_refine=8, iters=3)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    xq = queries_dev(X)
    w, kp, k = 5, 120, 12
    # two calls in a row, the second with a smaller input: what the first call left in the array must not leak into it
    for nq in (48, 17):
        q = xq[:nq].contiguous()
        ref_ids, ref_dist = ix.search(q, w, kp, k)
        ids = torch.full((nq, k), -7, dtype=torch.int32, device="cuda")
        dist = torch.full((nq, k), -7.0, dtype=torch.float32, device="cuda")
        free_before = torch.cuda.mem_get_info()[0]
        ix.search_static(q, w, kp, k, ids, dist)
        assert torch.cuda.mem_get_info()[0] == free_before           # nothing allocated, nothing freed
        assert torch.equal(ids, ref_ids) and torch.equal(dist, ref_dist)
        compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X[:nq], index, w, kp, k)
    # the sampled-bound path (a small full_mult makes every query filter) and every list-sharing mode
    ix.set_tuning(full_mult=1)
    for mode in (2, 1, 0):
        ix.set_list_sharing(mode)
        ref_ids, ref_dist = ix.search(xq, w, kp, k)
        ids = torch.empty((48, k), dtype=torch.int32, device="cuda")
        dist = torch.empty((48, k), dtype=torch.float32, device="cuda")
        ix.search_static(xq, w, kp, k, ids, dist)
        assert torch.equal(ids, ref_ids) and torch.equal(dist, ref_dist)
    # on a caller's stream
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ix.search_static(xq, w, kp, k, ids, dist)
    assert torch.equal(ids, ref_ids) and torch.equal(dist, ref_dist)
    # more queries than fit the fixed array at once (96 KB of tables per query at w = 12): the call splits them into
    # internal batches by itself, same bits as the allocating entry point
    big = xq.repeat(80, 1).contiguous()                                # 3840 queries
    ix.set_list_sharing(2)
    ref_ids, ref_dist = ix.search(big, 12, kp, k)
    ids_b = torch.empty((len(big), k), dtype=torch.int32, device="cuda")
    dist_b = torch.empty((len(big), k), dtype=torch.float32, device="cuda")
    ix.search_static(big, 12, kp, k, ids_b, dist_b)
    assert ix.search_stats()["pairs"] == len(big) * 12
    assert torch.equal(ids_b, ref_ids) and torch.equal(dist_b, ref_dist)
    ref_ids, ref_dist = ix.search(xq, w, kp, k)
    ix.search_static(xq, w, kp, k, ids, dist)
    assert torch.equal(ids, ref_ids) and torch.equal(dist, ref_dist)
    # a request whose workspace cannot fit the fixed array even for one query: clear error, nothing done
    with pytest.raises(pkg.IvfrError) as e:
        ix.search_static(xq, 12, 6_000_000, 12, ids, dist)            # 24 k' bytes of short-list per query = 144 MB
    assert e.value.code == pkg.binding.ERR_OOM and "too small" in str(e.value)
    ix.search_static(xq, w, kp, k, ids, dist)                         # still usable
    assert torch.equal(ids, ref_ids)
    ix.close()
    # a second index on the same GPU shares the array; used one after the other both stay correct
    wl2 = tiny_workload(d=32, G=16, N=3000, n_train=2000, n_query=12, c=8, m=4, m_refine=4, iters=4)
    ix2 = gpu_index_from_oracle(wl2["index"])
    q2 = queries_dev(wl2["X"])
    r_ids, r_dist = ix2.search(q2, 3, 50, 10)
    ids2 = torch.empty((12, 10), dtype=torch.int32, device="cuda")
    dist2 = torch.empty((12, 10), dtype=torch.float32, device="cuda")
    ix2.search_static(q2, 3, 50, 10, ids2, dist2)
    assert torch.equal(ids2, r_ids) and torch.equal(dist2, r_dist)
    ix2.close()
