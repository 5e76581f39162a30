"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs, the same codebooks and the same inverted file."""
import numpy as np
import pytest

import synthdata as sd
from oracle import ivfadcr_oracle as orc
from helpers import REL_TOL, compare_results, init_draws, tiny_workload

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def gpu_index_from_oracle(index, d=None):
    """An ivfadcr Index holding exactly the oracle's codebooks and inverted file."""
    import paper_1102_3828_amd as pkg
    b = index.books
    c, dd = b.coarse.shape
    ix = pkg.Index(dd, c, b.pq.shape[0], b.m_refine)
    ix.set_codebooks(b.coarse, b.pq, b.rq)
    ix.import_(index.list_offsets, index.ids, index.codes, index.rcodes)
    # Left to itself the library scans batches this small pair by pair; the tests want the shared-list scans
    # (units of eight, four, two) exercised on every small case as well, so they ask for them.
    ix.set_list_sharing(2)
    return ix


def queries_dev(X):
    torch = _torch()
    return torch.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).cuda()


def log(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ generator

def test_hip_generator_matches_numpy():
    from synthdata.gpu import DeviceMixture
    for G, d, zipf in ((16, 32, None), (256, 128, None), (1024, 128, 1.1)):
        mix = sd.make_mixture(G, d, zipf)
        dm = DeviceMixture(mix)
        for stream, start, n in ((sd.STREAM_TRAIN, 0, 5000), (sd.STREAM_BASE0 + 3, 123457, 3001)):
            log("generator", G, d, zipf, stream, start, n)
            ref = sd.gen_vectors(mix, stream, start, n)
            got = dm.generate(stream, start, n).cpu().numpy()
            assert np.array_equal(ref, got)


# ------------------------------------------------------------------ stage-level parity

@pytest.mark.parametrize("table_mode", [0, 1])
@pytest.mark.parametrize("kw", [dict(), dict(m_refine=0), dict(d=64, m=8, m_refine=16, c=24, N=5000, n_train=3000)])
def test_stages_against_oracle_trace(kw, table_mode):
    """Visited lists, short-list (ids, ADC estimates) and refined distances of every query; with one look-up table
    per pair and with split tables (per-list and per-query terms summed in the scan)."""
    wl = tiny_workload(**kw)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    ix.set_table_mode(table_mode)
    c = len(index.books.coarse)
    for w, kp, k in ((3, 50, 10), (c, 200, 20), (1, 10 ** 4, 5), (2, 7, 7)):
        log("stages", kw, w, kp, k)
        ids, dist, t = ix.search(queries_dev(X), w, kp, k, trace=True)
        t = {a: b.cpu().numpy() for a, b in t.items()}
        inv = orc.entry_of_id(index)
        for qi, x in enumerate(X):
            o_ids, o_dist, tr = orc.search_one(x, index, w, kp, k)
            # visited lists: identical unless two coarse distances nearly tie
            if not np.array_equal(t["probe"][qi], tr.probe):
                Dc = orc.sqdist(x[None].astype(np.float64), index.books.coarse)[0]
                assert np.allclose(np.sort(Dc[t["probe"][qi]]), np.sort(tr.probe_d), rtol=REL_TOL)
            assert np.allclose(t["probe_dist"][qi], tr.probe_d, rtol=REL_TOL, atol=1e-2)
            # short-list: same members (it is unordered on the GPU side)
            n = int(t["short_count"][qi])
            assert n == len(tr.short_entries) == min(kp, tr.scanned)
            g_ids = t["short_ids"][qi, :n]
            o_short = index.ids[tr.short_entries]
            diff = set(g_ids.tolist()) ^ set(o_short.tolist())
            for i in diff:   # only near-ties of the k'-th estimate may differ
                est = orc.adc_distance(x, index, int(inv[i]))
                assert abs(est - tr.short_est[-1]) <= REL_TOL * tr.short_est[-1]
            est_of = dict(zip(o_short.tolist(), tr.short_est.tolist()))
            ref_of = dict(zip(o_short.tolist(), tr.short_refined.tolist()))
            for s in range(n):
                i = int(g_ids[s])
                if i in est_of:
                    assert abs(t["short_est"][qi, s] - est_of[i]) <= REL_TOL * max(est_of[i], 1.0)
                    assert abs(t["short_ref"][qi, s] - ref_of[i]) <= REL_TOL * max(ref_of[i], 1.0)
            assert (t["short_ids"][qi, n:] == -1).all()
        exact, excused = compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, w, kp, k)
        log("  exact", exact, "excused", excused)
        assert excused <= 2
    ix.close()


@pytest.mark.parametrize("table_mode", [0, 1])
@pytest.mark.parametrize("m,m_refine", [(4, 0), (4, 64), (16, 8), (32, 32), (64, 4)])
def test_other_code_sizes(m, m_refine, table_mode):
    """Code sizes other than the workloads' m = 8 (the paper's Table 2 varies m and m'): every
    sub-vector width from 16 down to 1 dimension, with and without list sharing."""
    wl = tiny_workload(d=64, G=16, N=4000, n_train=2500, n_query=16, c=12, m=m, m_refine=m_refine, iters=3)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    ix.set_table_mode(table_mode)
    xq = queries_dev(X)
    for share in (2, 1, 0):
        ix.set_list_sharing(share)
        for full_mult in (8, 1):
            ix.set_tuning(full_mult=full_mult)
            log("code sizes", m, m_refine, "share", share, "full_mult", full_mult)
            ids, dist = ix.search(xq, 5, 150, 12)
            exact, excused = compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, 5, 150, 12)
            assert excused <= 2
    ix.close()


def test_single_list_is_exhaustive_adc_plus_r():
    """c = 1: no inverted file, every query scans every code (the ADC+R rows of Table 1)."""
    import paper_1102_3828_amd as pkg
    wl = tiny_workload(d=32, G=16, N=6000, n_train=2000, n_query=12, c=1, m=4, m_refine=8, iters=4)
    index, X, Y = wl["index"], wl["X"], wl["Y"]
    ix = gpu_index_from_oracle(index)
    for kp, k, full_mult in ((100, 10, 8), (600, 50, 1), (6000, 20, 8)):
        ix.set_tuning(full_mult=full_mult)
        ids, dist = ix.search(queries_dev(X), 1, kp, k)
        assert ix.search_stats()["codes_scanned"] == len(X) * index.N
        compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, 1, kp, k)
    ix.close()
    # the GPU builds the same single-list index from the vectors
    ix = pkg.Index(32, 1, 4, 8)
    b = index.books
    ix.set_codebooks(b.coarse, b.pq, b.rq)
    ix.add(Y, 0)
    ix.finalize()
    offsets, ids, codes, rcodes = ix.export()
    assert offsets.tolist() == [0, index.N] and np.array_equal(ids, np.arange(index.N))
    assert check_encoding(Y, b, offsets, ids, codes, rcodes) <= 20
    ix.close()


def test_all_lists_full_shortlist_is_exact_over_reconstructions():
    """w = c and k' = N: the GPU result is the exact k-NN among the refined reconstructions."""
    from helpers import dense_reconstructions
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    dense = dense_reconstructions(index, refine=True)
    ids, dist = ix.search(queries_dev(X), len(index.books.coarse), index.N, 25)
    ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
    for qi, x in enumerate(X):
        D = ((dense - x.astype(np.float64)) ** 2).sum(axis=1)
        order = np.lexsort((index.ids, D))[:25]
        assert ids[qi].tolist() == index.ids[order].tolist()
        assert np.allclose(dist[qi], D[order], rtol=REL_TOL)
    assert ix.search_stats()["codes_scanned"] == index.N * len(X)
    ix.close()


def test_lattice_database_returns_exact_neighbours():
    rng = np.random.default_rng(5)
    d, c, m, mr, N = 32, 6, 4, 8, 900
    coarse = (rng.normal(size=(c, d)) * 100).astype(np.float32)
    pq = (rng.normal(size=(m, 256, d // m)) * 2.0).astype(np.float32)
    rq = (rng.normal(size=(mr, 256, d // mr)) * 1e-3).astype(np.float32)
    books = orc.Codebooks(coarse, pq, rq)
    Y = (coarse[rng.integers(0, c, N)].astype(np.float64) + orc.pq_decode(rng.integers(0, 256, (N, m)).astype(np.uint8), pq)
         + orc.pq_decode(rng.integers(0, 256, (N, mr)).astype(np.uint8), rq))
    lists, codes, rcodes = orc.encode(Y, books)
    index = orc.assemble_index(lists, np.arange(N), codes, rcodes, books)
    X = (rng.normal(size=(6, d)) * 100).astype(np.float32)
    true_i, true_d = orc.brute_force(X.astype(np.float64), Y, 5)
    ix = gpu_index_from_oracle(index)
    ids, dist = ix.search(queries_dev(X), c, N, 5)
    assert np.array_equal(ids.cpu().numpy(), true_i)
    assert np.allclose(dist.cpu().numpy(), true_d, rtol=REL_TOL)
    ix.close()


# ------------------------------------------------------------------ end to end on workload-shaped data

def _cfg_workload(cfg, N, n_train, n_query, iters=10):
    mix = cfg.mixture()
    T = sd.gen_vectors(mix, sd.STREAM_TRAIN, 0, n_train)
    Y = sd.gen_base(mix, N)
    X = sd.gen_vectors(mix, sd.STREAM_QUERY, 0, n_query)
    return mix, T, Y, X


def test_config0_end_to_end_gpu_built_index():
    """The first workload (100k x 128-d, c = 256, m = m' = 8, w = 8, k' = 100, k = 10): the GPU trains,
    encodes and searches; the oracle searches the exported index; brute force gives recall."""
    import paper_1102_3828_amd as pkg
    torch = _torch()
    cfg = sd.CONFIGS["cfg0"]
    mix, T, Y, X = _cfg_workload(cfg, cfg.N, cfg.n_train, cfg.n_query)
    ix = pkg.Index(cfg.d, cfg.c, cfg.m, cfg.m_refine)
    log("train")
    ix.train(T, iters=10, seed=1)
    log("add")
    ix.add(torch.from_numpy(Y[:60000]).cuda(), 0)       # device input
    ix.add(Y[60000:], 60000)                              # host input
    ix.finalize()
    assert ix.ntotal == cfg.N
    coarse, pq, rq = ix.get_codebooks()
    offsets, ids, codes, rcodes = ix.export()
    index = orc.Index(orc.Codebooks(coarse, pq, rq), offsets, ids, codes, rcodes)
    assert sorted(ids.tolist()) == list(range(cfg.N))
    for l in range(cfg.c):
        assert np.all(np.diff(ids[offsets[l]:offsets[l + 1]]) > 0)
    log("encode parity")
    sub_n = 20000      # the oracle's encoders on the first 20000 vectors (ids 0..19999)
    keep = ids < sub_n
    sub_off = np.concatenate([[0], np.cumsum([int(keep[offsets[l]:offsets[l + 1]].sum()) for l in range(cfg.c)])])
    subst = check_encoding(Y[:sub_n], index.books, sub_off, ids[keep], codes[keep], rcodes[keep])
    log("near-tie substitutions", subst)
    assert subst <= 0.002 * sub_n * (1 + cfg.m + cfg.m_refine)
    log("search parity")
    g_ids, g_dist = ix.search(queries_dev(X), cfg.w, cfg.kprime, cfg.k)
    g_ids, g_dist = g_ids.cpu().numpy(), g_dist.cpu().numpy()
    exact, excused = compare_results(g_ids, g_dist, X, index, cfg.w, cfg.kprime, cfg.k)
    log("exact", exact, "excused", excused)
    assert exact >= 0.99 * cfg.n_query * cfg.k
    true_i, _ = orc.brute_force(X, Y, 1)
    r1, r10 = (orc.recall_at(g_ids, true_i[:, 0], r) for r in (1, 10))
    log("recall@1", r1, "recall@10", r10)
    o_ids, _, _ = orc.search(X, index, cfg.w, cfg.kprime, cfg.k)
    assert abs(r10 - orc.recall_at(o_ids, true_i[:, 0], 10)) <= 0.02
    assert r10 > 0.5
    st = ix.search_stats()
    assert st["pairs"] == cfg.n_query * cfg.w and st["dense_fallbacks"] == 0
    ix.set_table_mode(1)
    t_ids, t_dist = ix.search(queries_dev(X), cfg.w, cfg.kprime, cfg.k)
    exact, excused = compare_results(t_ids.cpu().numpy(), t_dist.cpu().numpy(), X, index, cfg.w, cfg.kprime, cfg.k)
    log("split tables: exact", exact, "excused", excused)
    assert exact >= 0.99 * cfg.n_query * cfg.k
    ix.close()


def _full_size_case(name, n_check, also=(), **override):
    """One of the five benchmark workloads at its full size, in the launch configuration the benchmark times
    (index built on the GPU from the HIP generator, first batch of 1000 queries searched in one
    call); n_check of those queries are verified one by one against the oracle on the exported index.
    also: further settings (dicts with kprime / k / n_check) searched on the same index and verified the same way."""
    import dataclasses
    import paper_1102_3828_amd as pkg
    from synthdata.gpu import DeviceMixture
    torch = _torch()
    cfg = dataclasses.replace(sd.CONFIGS[name], **override)
    dm = DeviceMixture(cfg.mixture())
    ix = pkg.Index(cfg.d, cfg.c, cfg.m, cfg.m_refine)
    log(name, "train")
    ix.train(dm.generate(sd.STREAM_TRAIN, 0, cfg.n_train), iters=10, seed=1)
    buf = None
    for j, a in enumerate(range(0, cfg.N, sd.BASE_CHUNK)):
        n = min(sd.BASE_CHUNK, cfg.N - a)
        if buf is None or buf.shape[0] != n:
            buf = torch.empty((n, cfg.d), dtype=torch.uint8, device="cuda")
        dm.generate(sd.STREAM_BASE0 + j, 0, n, out=buf)
        ix.add(buf, a)
        if j % 20 == 19:
            log(name, "added", a + n)
    del buf
    ix.finalize()
    B = min(cfg.batch, cfg.n_query)
    q_u8 = dm.generate(sd.STREAM_QUERY, 0, B)
    xq = q_u8.float().contiguous()
    settings = [dict(kprime=cfg.kprime, k=cfg.k, n_check=n_check, whole=True)]
    settings += [dict(kprime=a.get("kprime", cfg.kprime), k=a.get("k", cfg.k), n_check=a.get("n_check", n_check),
                      whole=False) for a in also]
    results = []
    for s in settings:
        kp, k = s["kprime"], s["k"]
        log(name, "search k' =", kp, "k =", k)
        ix.set_list_sharing(2)
        g_ids, g_dist = ix.search(xq, cfg.w, kp, k)
        st = ix.search_stats()
        log(name, st, ix.workspace_info())
        # closed form of section 3.3: a fraction of the order of w/c of the database is visited
        frac = st["codes_scanned"] / float(B) / cfg.N
        assert 0.3 * cfg.w / cfg.c < frac < (30.0 if cfg.zipf else 4.0) * cfg.w / cfg.c
        # properties that hold at any size: ascending distances, distinct valid ids
        gi, gd = g_ids.cpu().numpy(), g_dist.cpu().numpy()
        assert (np.diff(gd, axis=1) >= 0).all() and (gi >= 0).all() and (gi < cfg.N).all()
        assert all(len(set(r.tolist())) == k for r in gi[:50])
        # every (query, list) pair scanned on its own, and the matrix-core units, must give the same bits for the
        # whole batch
        for mode in (0, 3, -1):
            ix.set_list_sharing(mode)
            p_ids, p_dist = ix.search(xq, cfg.w, kp, k)
            log(name, "sharing mode", mode, ix.search_stats())
            assert np.array_equal(p_ids.cpu().numpy(), gi) and np.array_equal(p_dist.cpu().numpy(), gd)
            if mode == -1:   # left to itself the library shares lists when it expects the batch to stream 3e8 codes
                if st["codes_scanned"] >= 1.0e9: assert ix.search_stats()["codes_scanned_shared8"] > 0
                if st["codes_scanned"] <= 1.0e8: assert ix.search_stats()["codes_scanned_shared8"] == 0
        ix.set_list_sharing(2)
        if s["whole"] and cfg.n_query > B:
            # the workload's whole query set in one call (more queries share every list): same bits for the first
            # B queries as when they are searched on their own, and the same bits with the matrix-core units
            qa = dm.generate(sd.STREAM_QUERY, 0, cfg.n_query).float().contiguous()
            ix.set_tuning(batch=cfg.n_query)
            outs = []
            for mode in (2, 3):
                ix.set_list_sharing(mode)
                a_ids, a_dist = ix.search(qa, cfg.w, kp, k)
                log(name, "whole query set, sharing mode", mode, ix.search_stats())
                outs.append((a_ids.cpu().numpy(), a_dist.cpu().numpy()))
            assert np.array_equal(outs[0][0][:B], gi) and np.array_equal(outs[0][1][:B], gd)
            assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
            ix.set_list_sharing(2)
            ix.set_tuning(batch=B)
            del qa
        results.append((s, gi, gd, 0))
        # split look-up tables (per-list and per-query terms summed in the scan's prologue): per-pair and shared scans
        # must agree bit for bit with one another; the oracle comparison below covers the different rounding
        ix.set_table_mode(1)
        t_ids, t_dist = ix.search(xq, cfg.w, kp, k)
        log(name, "split tables", ix.search_stats(), ix.workspace_info())
        ti, td = t_ids.cpu().numpy(), t_dist.cpu().numpy()
        ix.set_list_sharing(0)
        p_ids, p_dist = ix.search(xq, cfg.w, kp, k)
        assert np.array_equal(p_ids.cpu().numpy(), ti) and np.array_equal(p_dist.cpu().numpy(), td)
        ix.set_list_sharing(2)
        ix.set_table_mode(0)
        log(name, "split tables: ids identical to materialised tables", float((ti == gi).mean()))
        assert (ti == gi).mean() > 0.98
        results.append((dict(s, n_check=max(2, s["n_check"] // 2)), ti, td, 1))
    log(name, "export")
    coarse, pq, rq = ix.get_codebooks()
    offsets, ids, codes, rcodes = ix.export()
    ix.close()
    index = orc.Index(orc.Codebooks(coarse, pq, rq), offsets, ids, codes, rcodes)
    assert index.bytes_per_vector() == cfg.m + cfg.m_refine + 4
    for s, gi, gd, table_mode in results:
        n = s["n_check"]
        X = q_u8[:n].cpu().numpy()
        log(name, "oracle on", n, "queries, k' =", s["kprime"], "table mode", table_mode)
        exact, excused = compare_results(gi[:n], gd[:n], X, index, cfg.w, s["kprime"], s["k"])
        log(name, "exact", exact, "excused", excused)
        assert exact >= 0.98 * n * s["k"]


@pytest.mark.timeout(300)
def test_full_size_config1():
    _full_size_case("cfg1", 24)


@pytest.mark.timeout(300)
def test_full_size_config2():
    _full_size_case("cfg2", 16)


@pytest.mark.timeout(600)
def test_full_size_config3():
    _full_size_case("cfg3", 4)


@pytest.mark.timeout(1200)
def test_full_size_config4_one_billion():
    """N = 10^9 with m' = 8: the short-list lengths the workload names, k' = 1000 and k' = 10000, on one index."""
    _full_size_case("cfg4", 16, also=[dict(kprime=10000, n_check=16)])


@pytest.mark.timeout(1200)
def test_full_size_config4_one_billion_32_refinement_bytes():
    """N = 10^9 with m' = 32 (44 bytes per vector resident)."""
    _full_size_case("cfg4", 16, m_refine=32)


def test_gpu_training_quality_matches_oracle():
    """k-means is chaotic, so trained codebooks are compared by their quantization error."""
    import paper_1102_3828_amd as pkg
    wl = tiny_workload(d=32, G=16, N=3000, n_train=4000, c=16, m=4, m_refine=8, iters=8)
    T, Y = wl["T"], wl["Y"]
    ix = pkg.Index(32, 16, 4, 8)
    ix.train(T, iters=8, seed=3)
    coarse, pq, rq = ix.get_codebooks()
    gb = orc.Codebooks(coarse, pq, rq)

    def errors(books):
        lists, codes, rcodes = orc.encode(Y, books)
        r1 = Y.astype(np.float64) - books.coarse[lists]
        r2 = r1 - orc.pq_decode(codes, books.pq)
        r3 = r2 - orc.pq_decode(rcodes, books.rq)
        return [(r ** 2).sum(axis=1).mean() for r in (r1, r2, r3)]
    eg, eo = errors(gb), errors(wl["books"])
    log("gpu", eg, "oracle", eo)
    for a, b in zip(eg, eo):
        assert a < 1.1 * b
    assert eg[0] > eg[1] > eg[2]
    ix.close()


def check_encoding(Y, books, offsets, ids, codes, rcodes, rel=REL_TOL):
    """GPU encoding of vectors Y (row i has id i) against the oracle's encoders: every choice must
    be the oracle's argmin, or a near-tie of it under the oracle's float64 distances (Eq. (8):
    the encoders are argmins).  Returns the number of near-tie substitutions."""
    N = len(Y)
    assert sorted(ids.tolist()) == list(range(N))
    entry = np.empty(N, dtype=np.int64)
    entry[ids] = np.arange(N)
    g_list = np.searchsorted(offsets, entry, side="right") - 1
    for l in range(len(offsets) - 1):
        assert np.all(np.diff(ids[offsets[l]:offsets[l + 1]]) > 0)
    Yf = Y.astype(np.float64)
    o_list = orc.nearest(Yf, books.coarse)
    subst = 0
    bad = np.nonzero(g_list != o_list)[0]
    for i in bad:
        D = orc.sqdist(Yf[i:i + 1], books.coarse)[0]
        assert D[g_list[i]] <= (1 + rel) * D[o_list[i]], ("list", i)
    subst += len(bad)
    # first-stage codes, given the GPU's own list choice
    r1 = Yf - books.coarse[g_list].astype(np.float64)
    g_codes = codes[entry]
    o_codes = orc.pq_encode(r1, books.pq)
    m, _, sub = books.pq.shape
    for i, j in zip(*np.nonzero(g_codes != o_codes)):
        dd = ((r1[i, j * sub:(j + 1) * sub][None] - books.pq[j].astype(np.float64)) ** 2).sum(axis=1)
        assert dd[g_codes[i, j]] <= (1 + rel) * dd[o_codes[i, j]] + 1e-9, ("code", i, j)
        subst += 1
    if books.rq is not None:
        r2 = r1 - orc.pq_decode(g_codes, books.pq)
        g_r = rcodes[entry]
        o_r = orc.pq_encode(r2, books.rq)
        mr, _, subr = books.rq.shape
        for i, j in zip(*np.nonzero(g_r != o_r)):
            dd = ((r2[i, j * subr:(j + 1) * subr][None] - books.rq[j].astype(np.float64)) ** 2).sum(axis=1)
            assert dd[g_r[i, j]] <= (1 + rel) * dd[o_r[i, j]] + 1e-9, ("rcode", i, j)
            subst += 1
    return subst


def test_encode_parity_with_oracle_codebooks():
    import paper_1102_3828_amd as pkg
    wl = tiny_workload(d=64, m=8, m_refine=16, c=24, N=5000, n_train=3000)
    b, Y = wl["books"], wl["Y"]
    ix = pkg.Index(64, 24, 8, 16)
    ix.set_codebooks(b.coarse, b.pq, b.rq)
    ix.add(Y[:1234], 0)
    ix.add(Y[1234:1234], 1234)      # empty add
    ix.add(Y[1234:], 1234)
    ix.finalize()
    offsets, ids, codes, rcodes = ix.export()
    subst = check_encoding(Y, b, offsets, ids, codes, rcodes)
    log("near-tie substitutions", subst)
    assert subst <= 0.002 * Y.shape[0] * (1 + 8 + 16)
    ix.close()


# ------------------------------------------------------------------ edge cases and host logic

def test_automatic_sharing_scans_small_batches_pair_by_pair():
    wl = tiny_workload(d=64, m=8, m_refine=16, c=24, N=5000, n_train=3000)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    xq = queries_dev(X)
    shared = ix.search(xq, 6, 300, 20)
    assert ix.search_stats()["codes_scanned_shared"] > 0
    ix.set_list_sharing(-1)   # the library's default
    auto = ix.search(xq, 6, 300, 20)
    st = ix.search_stats()
    assert st["codes_scanned_shared"] == 0 and st["codes_scanned_shared8"] == 0
    assert st["codes_streamed"] == st["codes_scanned"]
    assert np.array_equal(shared[0].cpu().numpy(), auto[0].cpu().numpy())
    assert np.array_equal(shared[1].cpu().numpy(), auto[1].cpu().numpy())
    ix.close()


def test_edge_cases_and_internal_paths():
    wl = tiny_workload(d=64, m=8, m_refine=16, c=24, N=5000, n_train=3000)
    index, X = wl["index"], wl["X"]
    torch = _torch()
    ix = gpu_index_from_oracle(index)
    xq = queries_dev(X)
    base_ids, base_dist = (t.cpu().numpy() for t in ix.search(xq, 6, 300, 20))
    compare_results(base_ids, base_dist, X, index, 6, 300, 20)
    # run twice: identical bits
    again = ix.search(xq, 6, 300, 20)
    assert np.array_equal(base_ids, again[0].cpu().numpy()) and np.array_equal(base_dist, again[1].cpu().numpy())
    # lists shared between queries are scanned several queries at a time by default; pair by pair gives the same bits
    st = ix.search_stats()
    assert st["codes_scanned_shared"] > 0 and st["codes_streamed"] < st["codes_scanned"]
    ix.set_list_sharing(0)
    pp = ix.search(xq, 6, 300, 20)
    st = ix.search_stats()
    assert st["codes_scanned_shared"] == 0 and st["codes_streamed"] == st["codes_scanned"]
    assert np.array_equal(base_ids, pp[0].cpu().numpy()) and np.array_equal(base_dist, pp[1].cpu().numpy())
    ix.set_tuning(full_mult=1)
    pp = ix.search(xq, 6, 300, 20)
    assert np.array_equal(base_ids, pp[0].cpu().numpy()) and np.array_equal(base_dist, pp[1].cpu().numpy())
    ix.set_tuning(full_mult=8)
    ix.set_list_sharing(2)
    # batches of 5 queries give the same answer
    ix.set_tuning(batch=5)
    b_ids, b_dist = ix.search(xq, 6, 300, 20)
    assert np.array_equal(base_ids, b_ids.cpu().numpy()) and np.array_equal(base_dist, b_dist.cpu().numpy())
    # sampled bound + filtered scan (the path large workloads take), forced by a small full_mult
    ix.set_tuning(full_mult=1, batch=1024)
    p_ids, p_dist = ix.search(xq, 6, 300, 20)
    assert ix.search_stats()["dense_fallbacks"] == 0
    assert np.array_equal(base_ids, p_ids.cpu().numpy()) and np.array_equal(base_dist, p_dist.cpu().numpy())
    # the smallest candidate buffers the plan allows
    ix.set_tuning(full_mult=1, cap_mult=1, min_cap=1)
    f_ids, f_dist = ix.search(xq, 6, 300, 20)
    log("smallest buffers", ix.search_stats())
    assert np.array_equal(base_ids, f_ids.cpu().numpy()) and np.array_equal(base_dist, f_dist.cpu().numpy())
    # every estimate kept (no sample, no filter)
    ix.set_tuning(full_mult=1000, cap_mult=1000, min_cap=8192)
    s_ids, s_dist = ix.search(xq, 6, 300, 20)
    assert np.array_equal(base_ids, s_ids.cpu().numpy()) and np.array_equal(base_dist, s_dist.cpu().numpy())
    ix.set_tuning(full_mult=8, cap_mult=16, scan_groups=3)
    g_ids, _ = ix.search(xq, 6, 300, 20)
    assert np.array_equal(base_ids, g_ids.cpu().numpy())
    ix.set_tuning(full_mult=1, scan_groups=5)
    g_ids, _ = ix.search(xq, 6, 300, 20)
    assert np.array_equal(base_ids, g_ids.cpu().numpy())
    ix.set_tuning(full_mult=8)
    # no queries
    e_ids, e_dist = ix.search(xq[:0], 6, 300, 20)
    assert e_ids.shape == (0, 20)
    # non-default stream
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        t_ids, _ = ix.search(xq, 6, 300, 20)
    assert np.array_equal(base_ids, t_ids.cpu().numpy())
    ix.close()


@pytest.mark.parametrize("table_mode", [0, 1])
@pytest.mark.parametrize("m", [8, 16, 4])
def test_list_sharing_modes_give_identical_bits(m, table_mode):
    """Many queries on few lists: units of eight (half-precision tables + exact re-evaluation), of
    four and of two (fp32 tables) and single pairs must all record the same fp32 estimates, so the
    three sharing modes return identical bits; the trace is checked against the oracle as well."""
    wl = tiny_workload(d=32, G=16, N=600000, n_train=3000, n_query=75, c=4, m=m, m_refine=16, iters=4)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    ix.set_table_mode(table_mode)
    xq = queries_dev(X)
    # sampled bound + filter, as the large workloads run; k' is small against the ~300000 visited entries, so
    # the bound passes well under 1 % of the estimates and the half-precision units are used
    w, kp, k = 2, 64, 5
    outs = {}
    for mode in (2, 1, 0):
        ix.set_list_sharing(mode)
        ids, dist, t = ix.search(xq, w, kp, k, trace=True)
        st = ix.search_stats()
        log("sharing mode", mode, st)
        outs[mode] = (ids.cpu().numpy(), dist.cpu().numpy(),
                      np.sort(t["short_ids"].cpu().numpy(), axis=1), np.sort(t["short_est"].cpu().numpy(), axis=1))
        assert st["dense_fallbacks"] == 0
        assert (st["codes_scanned_shared8"] > 0) == (mode == 2)
        if mode == 1:
            assert st["codes_scanned_shared"] > 0
        if mode == 0:
            assert st["codes_scanned_shared"] == 0 and st["codes_scanned_shared2"] == 0
        assert (st["codes_streamed"] == st["codes_scanned"]) == (mode == 0)
    for mode in (1, 0):
        for a, b in zip(outs[2], outs[mode]):
            assert np.array_equal(a, b)
    exact, excused = compare_results(outs[2][0], outs[2][1], X, index, w, kp, k)
    assert excused <= 3
    # a much larger k' (about 2 % of the visited entries) makes too many estimates pass for the half-precision
    # units: fp32 units only, same answers
    ix.set_list_sharing(2)
    ids, dist = ix.search(xq, w, 6000, 20)
    assert ix.search_stats()["codes_scanned_shared8"] == 0 and ix.search_stats()["codes_scanned_shared"] > 0
    compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, w, 6000, 20)
    ix.close()


@pytest.mark.parametrize("d,m", [(128, 8), (64, 8), (128, 4), (64, 4), (32, 4), (128, 16)])
def test_matrix_core_units_give_identical_bits(d, m):
    """Lists visited by 64 or more queries of the batch: the matrix-core scan (fp16 contraction against the
    decoded entries as a filter, exact fp32 table sums for what passes) must record the same estimates as the
    table look-up scans, so sharing mode 3 returns the bits of modes 2 and 0; checked against the oracle too."""
    wl = tiny_workload(d=d, G=16, N=200000, n_train=3000, n_query=230, c=4, m=m, m_refine=8, iters=4)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    xq = queries_dev(X)
    w, kp, k = 2, 16, 5   # k' small against the ~100000 visited entries: the bound passes a tiny share of them
    outs = {}
    for mode in (3, 2, 0):
        ix.set_list_sharing(mode)
        ids, dist, t = ix.search(xq, w, kp, k, trace=True)
        st = ix.search_stats()
        log("sharing mode", mode, st)
        outs[mode] = (ids.cpu().numpy(), dist.cpu().numpy(),
                      np.sort(t["short_ids"].cpu().numpy(), axis=1), np.sort(t["short_est"].cpu().numpy(), axis=1))
        assert st["dense_fallbacks"] == 0
        assert (st["codes_scanned_shared64"] > 0) == (mode == 3)
        if mode == 3:
            assert st["codes_scanned_shared64"] > st["codes_scanned"] // 2
    for mode in (2, 0):
        for a, b in zip(outs[3], outs[mode]):
            assert np.array_equal(a, b)
    sel = list(range(0, 230, 9))
    compare_results(outs[3][0][sel], outs[3][1][sel], X[sel], index, w, kp, k)
    ix.close()


def test_papers_own_shortlist_setting():
    """Section 4.3 runs k = 10000 with k' = 20000 (k'/k = 2): the largest result lists the library sorts."""
    wl = tiny_workload(d=32, G=16, N=60000, n_train=2000, n_query=3, c=8, m=4, m_refine=8, iters=4)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    for full_mult in (8, 1):
        ix.set_tuning(full_mult=full_mult)
        ids, dist = ix.search(queries_dev(X), 6, 20000, 10000)
        exact, excused = compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, 6, 20000, 10000)
        log("k = 10000, k' = 20000: exact", exact, "excused", excused)
        assert excused <= 20
    import paper_1102_3828_amd as pkg
    with pytest.raises(pkg.IvfrError):
        ix.search(queries_dev(X), 6, 40000, 20000)     # beyond the sortable result length
    ix.close()


def test_duplicate_vectors_are_cut_by_id():
    """Degenerate input: a database of three vectors repeated two thousand times each.  Estimates tie in
    huge groups, so the entries at or below the sampled bound overflow the candidate buffer; the
    rescan's bound is a key (estimate, id), which cuts through the ties, lowest ids first."""
    wl = tiny_workload(d=32, G=16, N=3000, n_train=2000, n_query=12, c=8, m=4, m_refine=4, iters=4)
    books, X = wl["books"], wl["X"]
    distinct = wl["Y"][:3]
    Y = np.repeat(distinct, 2000, axis=0)
    rng = np.random.default_rng(3)
    Y = Y[rng.permutation(len(Y))]
    index = orc.build_index(Y, np.arange(len(Y)), books)
    ix = gpu_index_from_oracle(index)
    ix.set_tuning(full_mult=1, cap_mult=1, min_cap=1)
    ids, dist = ix.search(queries_dev(X), 8, 50, 20)
    st = ix.search_stats()
    log("duplicates", st)
    assert st["bound_retries"] > 0
    o_ids, o_dist, _ = orc.search(X, index, 8, 50, 20)
    assert np.array_equal(ids.cpu().numpy(), o_ids)
    assert np.allclose(dist.cpu().numpy(), o_dist, rtol=REL_TOL)
    ix.close()
    # The same with every estimate kept (no bound): the short-list selection then takes 50 of 15000 records of
    # which thousands share one estimate, so the few-of-many shortcut finds a crowd at its bound, the general
    # narrowing takes over and goes on over the ids.
    Y = np.repeat(distinct, 5000, axis=0)
    Y = Y[rng.permutation(len(Y))]
    index = orc.build_index(Y, np.arange(len(Y)), books)
    ix = gpu_index_from_oracle(index)
    for mode in (2, 0):
        ix.set_list_sharing(mode)
        ix.set_tuning(full_mult=1000)
        ids, dist = ix.search(queries_dev(X), 8, 50, 20)
        st = ix.search_stats()
        assert st["bound_retries"] == 0 and st["dense_fallbacks"] == 0
        o_ids, o_dist, _ = orc.search(X, index, 8, 50, 20)
        assert np.array_equal(ids.cpu().numpy(), o_ids)
        assert np.allclose(dist.cpu().numpy(), o_dist, rtol=REL_TOL)
        # and with a bound: the sample's selection meets the same crowd
        ix.set_tuning(full_mult=1)
        ids, dist = ix.search(queries_dev(X), 8, 50, 20)
        assert np.array_equal(ids.cpu().numpy(), o_ids)
    ix.close()


@pytest.mark.parametrize("mode", [0, 2])
def test_bound_from_a_sample_of_the_nearest_lists(mode):
    """A short-list that is tiny against the visit (k' = 10 of ~30000 visited entries): the bound's sample is drawn
    from the nearest visited lists only.  Also with the nearest lists empty, so that the walk over the lists has to
    go on past them."""
    wl = tiny_workload(d=32, G=64, N=60000, n_train=4000, n_query=16, c=64, m=4, m_refine=4, iters=4)
    index, X = wl["index"], wl["X"]
    w, kp, k = 32, 10, 5
    ix = gpu_index_from_oracle(index)
    ix.set_list_sharing(mode)
    ids, dist = ix.search(queries_dev(X), w, kp, k)
    st = ix.search_stats()
    log("nearest-list sample", st)
    assert st["dense_fallbacks"] == 0
    o_ids, o_dist, traces = orc.search(X, index, w, kp, k)
    assert np.array_equal(ids.cpu().numpy(), o_ids)
    assert np.allclose(dist.cpu().numpy(), o_dist, rtol=REL_TOL)
    ix.close()
    # the same database with every query's three nearest lists emptied
    drop = set()
    for t in traces:
        drop.update(int(l) for l in t.probe[:3])
    keep = np.ones(index.N, dtype=bool)
    for l in drop:
        keep[index.list_offsets[l]:index.list_offsets[l + 1]] = False
    lens = np.array([int(keep[index.list_offsets[l]:index.list_offsets[l + 1]].sum()) for l in range(64)])
    offsets = np.concatenate([[0], np.cumsum(lens)])
    sparse = orc.Index(index.books, offsets, index.ids[keep], index.codes[keep], index.rcodes[keep])
    ix = gpu_index_from_oracle(sparse)
    ix.set_list_sharing(mode)
    ids, dist = ix.search(queries_dev(X), w, kp, k)
    o_ids, o_dist, _ = orc.search(X, sparse, w, kp, k)
    assert np.array_equal(ids.cpu().numpy(), o_ids)
    assert np.allclose(dist.cpu().numpy(), o_dist, rtol=REL_TOL)
    ix.close()


@pytest.mark.parametrize("order", ["far_first", "near_first"])
def test_unrepresentative_sample(order):
    """One list whose sampled prefix misrepresents it.  Far entries first: the bound drawn from the
    prefix lets every near entry through, the candidate buffer overflows, and the query is rescanned
    with the k'-th smallest key of the records that were kept.  The few nearest entries first: the
    bound falls among them, fewer than k' entries pass, and the query is redone without a filter."""
    rng = np.random.default_rng(17)
    d, c, m, mr = 32, 1, 4, 4
    if order == "far_first":
        parts = [rng.normal(60, 12, size=(60000, d)), rng.normal(180, 12, size=(60000, d))]
    else:
        parts = [rng.normal(180, 4, size=(4000, d)), rng.normal(60, 12, size=(116000, d))]
    Y = np.clip(np.concatenate(parts), 0, 255).round()
    T = Y[rng.permutation(len(Y))[:4000]]
    ic, ip, ir = init_draws(len(T), c, m, mr)
    books = orc.train(T, c, m, mr, 4, ic, ip, ir)
    index = orc.build_index(Y, np.arange(len(Y)), books)
    X = np.concatenate([rng.normal(180, 12, size=(6, d)), rng.normal(60, 12, size=(3, d))]).astype(np.float32)
    ix = gpu_index_from_oracle(index)
    ids, dist = ix.search(queries_dev(X), 1, 100, 20)
    st = ix.search_stats()
    log("ordered list", order, st)
    if order == "far_first":
        assert st["bound_retries"] >= 6 and st["dense_fallbacks"] == 0
    else:
        assert st["dense_fallbacks"] >= 6
    compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, 1, 100, 20)
    ix.close()


def test_redo_paths_on_a_callers_stream_and_across_batches():
    """Several queries of one call fail the filter's check (the few nearest entries lead the list): they are
    redone without a filter.  On a non-default stream, and with the call split into internal batches so that
    failing queries sit in batches whose arrays a later batch has overwritten, the results stay exact."""
    torch = _torch()
    rng = np.random.default_rng(17)
    d, c, m, mr = 32, 1, 4, 4
    parts = [rng.normal(180, 4, size=(4000, d)), rng.normal(60, 12, size=(116000, d))]
    Y = np.clip(np.concatenate(parts), 0, 255).round()
    T = Y[rng.permutation(len(Y))[:4000]]
    ic, ip, ir = init_draws(len(T), c, m, mr)
    books = orc.train(T, c, m, mr, 4, ic, ip, ir)
    index = orc.build_index(Y, np.arange(len(Y)), books)
    X = np.concatenate([rng.normal(180, 12, size=(6, d)), rng.normal(60, 12, size=(3, d))]).astype(np.float32)
    ix = gpu_index_from_oracle(index)
    xq = queries_dev(X)
    ref_ids, ref_dist = ix.search(xq, 1, 100, 20)
    assert ix.search_stats()["dense_fallbacks"] >= 6
    compare_results(ref_ids.cpu().numpy(), ref_dist.cpu().numpy(), X, index, 1, 100, 20)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        s_ids, s_dist = ix.search(xq, 1, 100, 20)
    log("caller's stream", ix.search_stats())
    assert ix.search_stats()["dense_fallbacks"] >= 6
    assert torch.equal(ref_ids, s_ids) and torch.equal(ref_dist, s_dist)
    for batch in (2, 4):
        ix.set_tuning(batch=batch)
        with torch.cuda.stream(side):
            b_ids, b_dist = ix.search(xq, 1, 100, 20)
        info = ix.workspace_info()
        log("batch", batch, ix.search_stats(), info)
        assert info["batch_reruns"] >= 1 and ix.search_stats()["dense_fallbacks"] >= 6
        assert torch.equal(ref_ids, b_ids) and torch.equal(ref_dist, b_dist)
    ix.close()


def test_candidate_pool_grows_when_the_estimate_is_low():
    """The host sizes the candidate pool from the expected visited-list length.  Queries that all fall into one
    list far longer than that want more: the plan kernel notices, the batch does no list work, the pool grows
    and the batch runs again.  Later calls find the pool large enough."""
    rng = np.random.default_rng(29)
    d, c, m, mr = 32, 201, 4, 4
    coarse = (rng.normal(size=(c, d)) * 60 + 128).astype(np.float32)
    books = orc.Codebooks(coarse, (rng.normal(size=(m, 256, d // m)) * 8).astype(np.float32),
                          (rng.normal(size=(mr, 256, d // mr)) * 2).astype(np.float32))
    # list 0 holds 20000 vectors, every other list 1000: the expected visited-list length (sum of len^2 / N, about
    # 2700) is below the 8 k' = 4000 entries up to which a query keeps everything, the real one far above
    Y = np.concatenate([coarse[0][None] + rng.normal(size=(20000, d)) * 9] +
                       [coarse[l][None] + rng.normal(size=(1000, d)) * 3 for l in range(1, c)])
    index = orc.build_index(Y, np.arange(len(Y)), books)
    assert index.list_offsets[1] - index.list_offsets[0] >= 19000
    X = (coarse[0][None] + rng.normal(size=(40, d)) * 9).astype(np.float32)
    ix = gpu_index_from_oracle(index)
    xq = queries_dev(X)
    ids, dist = ix.search(xq, 1, 500, 20)
    info = ix.workspace_info()
    log("first call", info, ix.search_stats())
    assert info["batch_reruns"] == 1
    compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, 1, 500, 20)
    ids2, dist2 = ix.search(xq, 1, 500, 20)
    info2 = ix.workspace_info()
    assert info2["batch_reruns"] == 0 and info2["pool_bytes"] == info["pool_bytes"]
    assert np.array_equal(ids.cpu().numpy(), ids2.cpu().numpy()) and np.array_equal(dist.cpu().numpy(), dist2.cpu().numpy())
    ix.close()
    # the same in a call of several internal batches, all enqueued before the first status is read: every batch finds
    # the pool too small and is run again, one after the other
    ix = gpu_index_from_oracle(index)
    ix.set_tuning(batch=10)
    ids3, dist3 = ix.search(xq, 1, 500, 20)
    info3 = ix.workspace_info()
    log("four batches", info3, ix.search_stats())
    assert info3["batch_reruns"] >= 1
    assert np.array_equal(ids.cpu().numpy(), ids3.cpu().numpy()) and np.array_equal(dist.cpu().numpy(), dist3.cpu().numpy())
    ix.close()


def test_memory_limit_refuses_before_allocating():
    """Capacity checks on the host: with a cap below what finalize / search need the call fails with
    IVFR_ERR_OOM and leaves the index as it was; with the cap lifted the same call succeeds."""
    import paper_1102_3828_amd as pkg
    wl = tiny_workload(d=64, m=8, m_refine=16, c=24, N=5000, n_train=3000)
    index, X, Y, b = wl["index"], wl["X"], wl["Y"], wl["books"]
    ix = pkg.Index(64, 24, 8, 16)
    ix.set_codebooks(b.coarse, b.pq, b.rq)
    ix.add(Y, 0)
    ix.set_memory_limit(50_000)                       # the 5000 x 28 bytes of the lists alone are more
    with pytest.raises(pkg.IvfrError) as e:
        ix.finalize()
    assert e.value.code == pkg.binding.ERR_OOM
    ix.set_memory_limit(0)
    ix.finalize()
    xq = queries_dev(X)
    held = ix.workspace_info()["index_bytes"]
    ix.set_memory_limit(held + 100_000)               # the tables of 12 x 6 pairs alone take 590 KB
    with pytest.raises(pkg.IvfrError) as e:
        ix.search(xq, 6, 300, 20)
    assert e.value.code == pkg.binding.ERR_OOM and "memory limit" in str(e.value)
    assert ix.workspace_info()["workspace_bytes"] == 0
    ix.set_memory_limit(0)
    ids, dist = ix.search(xq, 6, 300, 20)
    offsets, i2, codes, rcodes = ix.export()
    gi = orc.Index(b, offsets, i2, codes, rcodes)
    compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, gi, 6, 300, 20)
    # import refuses negative ids
    ix2 = pkg.Index(64, 24, 8, 16)
    ix2.set_codebooks(b.coarse, b.pq, b.rq)
    bad = i2.copy()
    bad[7] = -3
    with pytest.raises(pkg.IvfrError) as e:
        ix2.import_(offsets, bad, codes, rcodes)
    assert e.value.code == pkg.binding.ERR_INVALID_ARG
    ix2.import_(offsets, i2, codes, rcodes)           # the refused call left nothing behind
    ids3, dist3 = ix2.search(xq, 6, 300, 20)
    assert np.array_equal(ids.cpu().numpy(), ids3.cpu().numpy())
    ix.close()
    ix2.close()


def test_empty_lists_and_short_results():
    """More lists than vectors: most lists are empty; k exceeds what the visited lists hold."""
    rng = np.random.default_rng(11)
    d, c, m, mr, N = 32, 64, 4, 4, 40
    books = orc.Codebooks((rng.normal(size=(c, d)) * 50).astype(np.float32),
                          (rng.normal(size=(m, 256, d // m)) * 5).astype(np.float32),
                          (rng.normal(size=(mr, 256, d // mr))).astype(np.float32))
    Y = rng.normal(size=(N, d)) * 50
    index = orc.build_index(Y, np.arange(N), books)
    X = (rng.normal(size=(9, d)) * 50).astype(np.float32)
    ix = gpu_index_from_oracle(index)
    for w, kp, k in ((5, 30, 30), (64, 100, 50), (1, 1, 1)):
        ids, dist = ix.search(queries_dev(X), w, kp, k)
        compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, w, kp, k)
    ix.close()
    # an index with no vectors at all
    import paper_1102_3828_amd as pkg
    ix = pkg.Index(d, c, m, mr)
    ix.set_codebooks(books.coarse, books.pq, books.rq)
    ix.finalize()
    ids, dist = ix.search(queries_dev(X), 3, 10, 5)
    assert (ids.cpu().numpy() == -1).all() and np.isinf(dist.cpu().numpy()).all()
    ix.close()


def test_visiting_thousands_of_lists_splits_the_batch():
    """w = c = 8192: the look-up tables of one query take 32 MB, so the 300 queries cannot share one internal
    batch (the library keeps a batch's tables under 8 GiB and splits the call into two batches of 150); results
    must not depend on the split."""
    rng = np.random.default_rng(23)
    d, c, m, mr, N = 32, 8192, 4, 4, 6000
    books = orc.Codebooks((rng.normal(size=(c, d)) * 40 + 128).astype(np.float32),
                          (rng.normal(size=(m, 256, d // m)) * 6).astype(np.float32),
                          (rng.normal(size=(mr, 256, d // mr))).astype(np.float32))
    Y = np.clip(rng.normal(128, 40, size=(N, d)), 0, 255).round()
    index = orc.build_index(Y, np.arange(N), books)
    X = np.clip(rng.normal(128, 40, size=(300, d)), 0, 255).astype(np.float32)
    ix = gpu_index_from_oracle(index)
    ids, dist = ix.search(queries_dev(X), c, 300, 10)
    assert ix.search_stats()["pairs"] == 300 * c
    sel = [0, 1, 148, 149, 150, 151, 298, 299]   # both sides of the split (the oracle builds 8192 tables per query)
    compare_results(ids.cpu().numpy()[sel], dist.cpu().numpy()[sel], X[sel], index, c, 300, 10)
    ix.close()


def _random_case(seed):
    """Seeded pick of a valid shape: d a multiple of 8; m, m' bytes with sub-vectors of 1..32 dimensions."""
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([8, 16, 32, 64, 128]))
    ms = [m for m in (4, 8, 16, 32, 64) if d % m == 0 and d // m in (1, 2, 4, 8, 16, 32)]
    mrs = [0] + ms
    m, mr = int(rng.choice(ms)), int(rng.choice(mrs))
    c = int(rng.choice([1, 2, 3, 7, 16, 33]))
    N = int(rng.integers(1, 4000))
    w = int(rng.integers(1, c + 1))
    kp = int(rng.choice([1, 5, 40, 300, 5000]))
    k = int(rng.integers(1, min(kp, 200) + 1))
    nq = int(rng.integers(1, 20))
    return dict(d=d, m=m, mr=mr, c=c, N=N, w=w, kp=kp, k=k, nq=nq)


@pytest.mark.parametrize("table_mode", [0, 1])
@pytest.mark.parametrize("seed", range(40))
def test_random_shapes(seed, table_mode):
    """Seeded random shapes: odd dimensions and code sizes, more lists than vectors, k' above and below what is
    visited, every list-sharing mode and both the filtered and the keep-everything paths."""
    cs = _random_case(seed)
    log("random case", seed, cs)
    rng = np.random.default_rng(2000 + seed)
    d, c, m, mr = cs["d"], cs["c"], cs["m"], cs["mr"]
    books = orc.Codebooks((rng.normal(size=(c, d)) * 30 + 128).astype(np.float32),
                          (rng.normal(size=(m, 256, d // m)) * 8).astype(np.float32),
                          (rng.normal(size=(mr, 256, d // mr)) * 2).astype(np.float32) if mr else None)
    Y = np.clip(rng.normal(128, 35, size=(cs["N"], d)), 0, 255).round()
    index = orc.build_index(Y, np.arange(cs["N"]), books)
    X = np.clip(rng.normal(128, 35, size=(cs["nq"], d)), 0, 255).astype(np.float32)
    ix = gpu_index_from_oracle(index)
    ix.set_table_mode(table_mode)
    xq = queries_dev(X)
    for mode, full_mult in ((2, 8), (1, 1), (0, 1)):
        ix.set_list_sharing(mode)
        ix.set_tuning(full_mult=full_mult)
        ids, dist = ix.search(xq, cs["w"], cs["kp"], cs["k"])
        exact, excused = compare_results(ids.cpu().numpy(), dist.cpu().numpy(), X, index, cs["w"], cs["kp"], cs["k"])
        assert excused <= max(2, exact // 50)
    ix.close()


def _crowded_case(seed):
    """Seeded pick of a shape where many queries of the batch visit the same few lists."""
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([32, 64, 128]))
    ms = [m for m in (4, 8, 16, 32) if d % m == 0 and d // m in (2, 4, 8, 16, 32)]
    m = int(rng.choice(ms))
    mr = int(rng.choice([0, 8]))
    if seed % 2 == 0:   # long lists and a tiny k': the bound passes so few estimates that the filtered units are used
        c = int(rng.choice([1, 2]))
        N = int(rng.integers(200000, 400000))
        kp = int(rng.choice([1, 4, 16]))
    else:
        c = int(rng.choice([1, 2, 3, 5]))
        N = int(rng.integers(2000, 120000))
        kp = int(rng.choice([1, 8, 40, 300]))
    w = int(rng.integers(1, c + 1))
    k = int(rng.integers(1, min(kp, 50) + 1))
    nq = int(rng.integers(70, 400))
    scale = float(rng.choice([1e-3, 1.0, 50.0]))
    return dict(d=d, m=m, mr=mr, c=c, N=N, w=w, kp=kp, k=k, nq=nq, scale=scale)


@pytest.mark.parametrize("table_mode", [0, 1])
@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_with_crowded_lists(seed, table_mode):
    """Seeded random shapes with 70-400 queries on one to five lists and codebooks / queries scaled by 0.001, 1
    or 50: units of 64, eight, four and two all occur.  Every sharing mode must return the bits of the per-pair
    scan; a few queries are checked against the oracle."""
    cs = _crowded_case(seed)
    log("crowded case", seed, cs)
    rng = np.random.default_rng(6000 + seed)
    d, c, m, mr, sc = cs["d"], cs["c"], cs["m"], cs["mr"], cs["scale"]
    books = orc.Codebooks(((rng.normal(size=(c, d)) * 10 + 128) * sc).astype(np.float32),
                          (rng.normal(size=(m, 256, d // m)) * 12 * sc).astype(np.float32),
                          (rng.normal(size=(mr, 256, d // mr)) * 2 * sc).astype(np.float32) if mr else None)
    Y = np.clip(rng.normal(128, 35, size=(cs["N"], d)), 0, 255).round() * sc
    index = orc.build_index(Y, np.arange(cs["N"]), books)
    X = (np.clip(rng.normal(128, 35, size=(cs["nq"], d)), 0, 255) * sc).astype(np.float32)
    ix = gpu_index_from_oracle(index)
    ix.set_table_mode(table_mode)
    xq = queries_dev(X)
    outs = {}
    for mode in (0, 3, 2, 1):
        ix.set_list_sharing(mode)
        ids, dist = ix.search(xq, cs["w"], cs["kp"], cs["k"])
        st = ix.search_stats()
        log("  mode", mode, {a: b for a, b in st.items() if b})
        outs[mode] = (ids.cpu().numpy(), dist.cpu().numpy())
        assert np.array_equal(outs[mode][0], outs[0][0]) and np.array_equal(outs[mode][1], outs[0][1])
    sel = list(range(0, cs["nq"], max(1, cs["nq"] // 5)))
    exact, excused = compare_results(outs[0][0][sel], outs[0][1][sel], X[sel], index, cs["w"], cs["kp"], cs["k"])
    assert excused <= max(2, exact // 50)
    ix.close()


def test_search_on_a_callers_stream():
    """The library enqueues on the stream it is given (here a non-default torch stream) and returns when that
    stream has drained: same bits as on the default stream."""
    torch = _torch()
    wl = tiny_workload(d=64, G=16, N=4000, n_train=2500, n_query=16, c=12, m=8, m_refine=8, iters=3)
    index, X = wl["index"], wl["X"]
    ix = gpu_index_from_oracle(index)
    xq = queries_dev(X)
    torch.cuda.synchronize()
    ids0, dist0 = ix.search(xq, 5, 150, 12)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ids1, dist1 = ix.search(xq, 5, 150, 12)
    assert torch.equal(ids0, ids1) and torch.equal(dist0, dist1)
    ids2, dist2 = ix.search(xq, 5, 150, 12, stream=side.cuda_stream)
    assert torch.equal(ids0, ids2) and torch.equal(dist0, dist2)
    ix.close()


def test_error_paths():
    import paper_1102_3828_amd as pkg
    torch = _torch()
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    b = index.books
    ix = pkg.Index(32, 8, 4, 4)
    xq = queries_dev(X)
    with pytest.raises(pkg.IvfrError) as e:
        ix.add(wl["Y"][:10], 0)
    assert e.value.code == pkg.binding.ERR_STATE
    ix.set_codebooks(b.coarse, b.pq, b.rq)
    with pytest.raises(pkg.IvfrError) as e:
        ix.search(xq, 2, 10, 5)
    assert e.value.code == pkg.binding.ERR_STATE
    ix.add(wl["Y"][:100], 0)
    with pytest.raises(pkg.IvfrError) as e:
        ix.add(wl["Y"][:100], 50)       # overlapping ids
    assert e.value.code == pkg.binding.ERR_INVALID_ARG
    with pytest.raises(pkg.IvfrError) as e:
        ix.set_codebooks(b.coarse, b.pq, b.rq)
    assert e.value.code == pkg.binding.ERR_STATE
    ix.finalize()
    with pytest.raises(pkg.IvfrError) as e:
        ix.add(wl["Y"][:10], 1000)
    assert e.value.code == pkg.binding.ERR_STATE
    for w, kp, k in ((0, 10, 5), (9, 10, 5), (2, 0, 0), (2, 5, 6)):
        with pytest.raises(pkg.IvfrError) as e:
            ix.search(xq, w, kp, k)
        assert e.value.code == pkg.binding.ERR_INVALID_ARG
    ids, _ = ix.search(xq, 2, 10, 5)    # still usable after errors
    assert ids.shape == (len(X), 5)
    # a query with a NaN or an infinite component is refused, and named
    for row, col, val in ((3, 7, float("nan")), (len(X) - 1, 0, float("inf")), (0, 31, float("-inf"))):
        bad = xq.clone()
        bad[row, col] = val
        with pytest.raises(pkg.IvfrError) as e:
            ix.search(bad, 2, 10, 5)
        assert e.value.code == pkg.binding.ERR_INVALID_ARG and f"query {row} " in str(e.value)
    ids2, _ = ix.search(xq, 2, 10, 5)
    assert torch.equal(ids, ids2)
    ix.close()
