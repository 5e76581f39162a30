"""Shared test fixtures: tiny synthetic workloads and the GPU-vs-oracle comparator."""
from __future__ import annotations

import functools

import numpy as np

import synthdata as sd
from oracle import ivfadcr_oracle as orc


def init_draws(n_train: int, c: int, m: int, m_refine: int, seed: int = sd.BASE_SEED):
    """Initial-centroid row draws for train(): distinct rows per quantizer."""
    ic = sd.draw_without_replacement(seed, sd.STREAM_INIT, n_train, c)
    ip = np.stack([sd.draw_without_replacement(seed, sd.STREAM_INIT + 100 + j, n_train, 256) for j in range(m)])
    ir = (np.stack([sd.draw_without_replacement(seed, sd.STREAM_INIT + 200 + j, n_train, 256)
                    for j in range(m_refine)]) if m_refine else None)
    return ic, ip, ir


@functools.lru_cache(maxsize=None)
def tiny_workload(d=32, G=16, N=3000, n_train=2000, n_query=12, c=8, m=4, m_refine=4, iters=4, zipf=None):
    """A workload small enough for dense float64 checks, trained with the oracle."""
    mix = sd.make_mixture(G, d, zipf)
    T = sd.gen_vectors(mix, sd.STREAM_TRAIN, 0, n_train)
    Y = sd.gen_vectors(mix, sd.STREAM_BASE0, 0, N)
    X = sd.gen_vectors(mix, sd.STREAM_QUERY, 0, n_query)
    ic, ip, ir = init_draws(n_train, c, m, m_refine)
    books = orc.train(T, c, m, m_refine, iters, ic, ip, ir)
    index = orc.build_index(Y, np.arange(N), books)
    return dict(mix=mix, T=T, Y=Y, X=X, books=books, index=index)


def dense_reconstructions(index, refine=True):
    """Every entry's approximation, built with explicit loops (independent of orc.reconstruct)."""
    b = index.books
    N = index.N
    d = b.coarse.shape[1]
    out = np.zeros((N, d))
    for l in range(len(index.list_offsets) - 1):
        for e in range(index.list_offsets[l], index.list_offsets[l + 1]):
            y = b.coarse[l].astype(np.float64).copy()
            m, _, sub = b.pq.shape
            for j in range(m):
                y[j * sub:(j + 1) * sub] += b.pq[j, index.codes[e, j]].astype(np.float64)
            if refine and b.rq is not None:
                mr, _, subr = b.rq.shape
                for j in range(mr):
                    y[j * subr:(j + 1) * subr] += b.rq[j, index.rcodes[e, j]].astype(np.float64)
            out[e] = y
    return out


REL_TOL = 1e-4   # relative distance tolerance between the fp32 GPU path and the float64 oracle


def close(a, b, rel=REL_TOL, floor=0.0):
    return abs(a - b) <= rel * max(abs(b), floor)


def compare_results(gpu_ids, gpu_dist, X, index, w, kprime, k, rel=REL_TOL, abs_floor=1.0):
    """GPU (ids, distances) against the oracle's search on the same index.

    Per query: (1) every returned distance matches the oracle's refined distance (Eq. (10)) of
    the returned id within `rel`, and the GPU's list is ascending; (2) the returned id sets
    agree, except for ids that the oracle's own float64 values place within `rel` of a
    decision boundary: the k-th final distance, the k'-th short-list estimate, or the w-th
    visited-list coarse distance (several results are correct exactly there).  Returns
    (ranks with identical id, excused ids); raises AssertionError on anything else.
    abs_floor keeps the relative test meaningful for near-zero distances.
    """
    exact = excused = 0
    if index.N <= 50_000_000:
        inv = orc.entry_of_id(index)
    else:
        class _Lazy:   # a handful of look-ups in a huge index: search instead of an N-long inverse
            def __getitem__(self, i):
                return int(np.flatnonzero(index.ids == np.int32(i))[0])
        inv = _Lazy()
    offs = index.list_offsets
    for qi, x in enumerate(X):
        o_ids, o_dist, tr = orc.search_one(x, index, w, kprime, k)
        g_ids = np.asarray(gpu_ids[qi]).astype(np.int64)
        g_dist = np.asarray(gpu_dist[qi]).astype(np.float64)
        n_o = int((o_ids >= 0).sum())
        n_g = int((g_ids >= 0).sum())
        assert n_g == n_o, ("result count", qi, n_g, n_o)
        assert (g_ids[n_g:] == -1).all() and np.isinf(g_dist[n_g:]).all(), ("padding", qi)
        assert len(set(g_ids[:n_g].tolist())) == n_g, ("duplicate ids", qi)
        # (1) distances and order
        for r in range(n_g):
            ref = o_dist[r] if g_ids[r] == o_ids[r] else orc.refined_distance(x, index, int(inv[g_ids[r]]))
            assert close(g_dist[r], ref, rel, abs_floor), ("distance", qi, r, int(g_ids[r]), g_dist[r], ref)
            if r:
                assert g_dist[r] >= g_dist[r - 1], ("not ascending", qi, r)
        exact += int((g_ids[:n_g] == o_ids[:n_o]).sum())
        # (2) set differences must sit on a boundary
        kth_final = o_dist[n_o - 1] if n_o else np.inf
        kth_est = tr.short_est[-1] if len(tr.short_est) else np.inf
        wth = tr.probe_d[-1]
        Dc = orc.sqdist(np.asarray(x, dtype=np.float64)[None], index.books.coarse)[0]
        gset = set(g_ids[:n_g].tolist())
        oset = set(o_ids[:n_o].astype(np.int64).tolist())
        short_ids = set(index.ids[tr.short_entries].astype(np.int64).tolist())

        def boundaries(i):
            e = int(inv[i])
            l = int(np.searchsorted(offs, e, side="right") - 1)
            final = close(orc.refined_distance(x, index, e), kth_final, rel, abs_floor)
            upstream = (close(orc.adc_distance(x, index, e), kth_est, rel, abs_floor)
                        or close(Dc[l], wth, rel, abs_floor))
            return final, upstream

        upstream_leavers = 0
        for i in oset - gset:          # in the oracle's answer, missing from the GPU's
            final, upstream = boundaries(i)
            assert final or upstream, ("unexcused missing id", qi, i)
            upstream_leavers += int(upstream and not final)
            excused += 1
        for i in gset - oset:          # in the GPU's answer only
            final, upstream = boundaries(i)
            # an id displaced upstream frees a slot for the next-best short-list member
            ok = final or upstream or (upstream_leavers > 0 and i in short_ids)
            assert ok, ("unexcused extra id", qi, i)
            excused += 1
    return exact, excused
