"""Pins for the CPU oracle: each test ties one of its functions to something the paper or
the mathematics fixes, by a route that does not pass through the function itself."""
import os

import numpy as np
import pytest

import synthdata as sd
from oracle import ivfadcr_oracle as orc
from helpers import dense_reconstructions, init_draws, tiny_workload


# ---------------------------------------------------------------- building blocks

def test_sqdist_matches_hand_loops():
    rng = np.random.default_rng(0)
    A, B = rng.normal(size=(5, 7)), rng.normal(size=(6, 7))
    D = orc.sqdist(A, B)
    for i in range(5):
        for j in range(6):
            s = 0.0
            for t in range(7):
                s += (A[i, t] - B[j, t]) ** 2
            assert abs(D[i, j] - s) < 1e-12
    # integer-valued bytes: exact
    a = np.array([[0, 255, 3]], dtype=np.uint8)
    b = np.array([[255, 0, 1]], dtype=np.uint8)
    assert orc.sqdist(a, b)[0, 0] == 255 ** 2 * 2 + 4


def test_smallest_total_order_and_ties():
    d = np.array([3.0, 1.0, 1.0, 2.0, 1.0])
    tb = np.array([9, 7, 2, 0, 5])
    assert orc.smallest(d, tb, 4).tolist() == [2, 4, 1, 3]
    assert orc.argmin_rows(np.array([[2.0, 1.0, 1.0]])).tolist() == [1]


def test_subvector_split_is_contiguous():
    V = np.arange(24, dtype=np.float64).reshape(2, 12)
    S = orc.subvectors(V, 3)
    assert S[1, 2].tolist() == [20, 21, 22, 23] and S[0, 0].tolist() == [0, 1, 2, 3]


def test_pq_encode_is_bruteforce_argmin_and_decode_inverts():
    rng = np.random.default_rng(1)
    book = rng.normal(size=(3, 256, 4)).astype(np.float32)
    V = rng.normal(size=(40, 12))
    codes = orc.pq_encode(V, book)
    for i in range(40):
        for j in range(3):
            best, bd = -1, np.inf
            for k in range(256):
                dd = float(((V[i, 4 * j:4 * j + 4] - book[j, k].astype(np.float64)) ** 2).sum())
                if dd < bd:
                    best, bd = k, dd
            assert codes[i, j] == best
    dec = orc.pq_decode(codes, book)
    for i in range(40):
        for j in range(3):
            assert np.array_equal(dec[i, 4 * j:4 * j + 4], book[j, codes[i, j]].astype(np.float64))
    # a vector that is a reproduction value encodes to itself
    lattice = np.concatenate([book[0, 17], book[1, 200], book[2, 0]])[None].astype(np.float64)
    assert orc.pq_encode(lattice, book).tolist() == [[17, 200, 0]]


def test_kmeans_closed_forms():
    # two well-separated 1-d clusters: centroids are the cluster means after one iteration
    X = np.array([[0.0], [1.0], [2.0], [10.0], [12.0]])
    C, hist = orc.kmeans(X, X[[0, 3]], 3)
    assert np.allclose(C[:, 0], [1.0, 11.0])
    assert hist[0] == pytest.approx((0 + 1 + 4 + 0 + 4) / 5)
    assert hist[-1] == pytest.approx((1 + 0 + 1 + 1 + 1) / 5)
    # K = n: every point its own centroid, zero error
    C, hist = orc.kmeans(X, X, 2)
    assert hist == [0.0, 0.0] and np.allclose(C, X)
    # an empty cluster keeps its centroid
    C, _ = orc.kmeans(np.array([[0.0], [1.0]]), np.array([[0.5], [100.0]]), 2)
    assert C[1, 0] == 100.0 and C[0, 0] == 0.5


def test_kmeans_matches_library_lloyd_and_objective_decreases():
    from sklearn.cluster import KMeans
    mix = sd.make_mixture(8, 16)
    X = sd.gen_vectors(mix, sd.STREAM_TRAIN, 0, 1500).astype(np.float64)
    init = X[sd.draw_without_replacement(7, 1, 1500, 8)]
    C, hist = orc.kmeans(X, init, 6)
    assert all(hist[i + 1] <= hist[i] + 1e-9 for i in range(len(hist) - 1))
    km = KMeans(n_clusters=8, init=init, n_init=1, max_iter=6, tol=0.0, algorithm="lloyd").fit(X)
    assert np.allclose(C, km.cluster_centers_, rtol=0, atol=1e-3)


# ---------------------------------------------------------------- invariants of the method

def test_adc_table_sum_equals_distance_to_decoded_vector():
    """Eq. (5) is a decomposition of Eq. (1): the sum of m table entries equals the squared
    distance from x to the explicit first-stage approximation."""
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    dense = dense_reconstructions(index, refine=False)
    for x in X[:4]:
        for l in range(len(index.list_offsets) - 1):
            est = orc.adc_scan(x, index, l)
            a, b = index.list_offsets[l], index.list_offsets[l + 1]
            ref = ((dense[a:b] - x.astype(np.float64)) ** 2).sum(axis=1)
            assert np.allclose(est, ref, rtol=1e-12, atol=1e-9)
    e = int(index.N // 2)
    assert orc.adc_distance(X[0], index, e) == pytest.approx(((dense[e] - X[0].astype(np.float64)) ** 2).sum(), rel=1e-12)


def test_refined_distance_is_distance_to_refined_reconstruction():
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    dense = dense_reconstructions(index, refine=True)
    for e in (0, 17, index.N - 1):
        ref = ((dense[e] - X[1].astype(np.float64)) ** 2).sum()
        assert orc.refined_distance(X[1], index, e) == pytest.approx(ref, rel=1e-12)


def test_zero_refinement_bytes_is_plain_ivfadc():
    """Table 1 rows with m' = 0: without a refinement code the refined estimator is the ADC
    estimator and the output is the head of the short-list."""
    wl = tiny_workload(m_refine=0)
    index, X = wl["index"], wl["X"]
    assert index.rcodes.shape[1] == 0 and index.books.rq is None
    for x in X:
        ids, dist, tr = orc.search_one(x, index, 3, 50, 10)
        assert np.allclose(tr.short_refined, tr.short_est, rtol=1e-12)
        assert ids.tolist() == index.ids[tr.short_entries[:10]].tolist()
        assert np.allclose(dist, tr.short_est[:10], rtol=1e-12)


def test_all_lists_and_full_shortlist_is_exact_order_over_reconstructions():
    """Visiting every list with k' = n makes step 1 keep everything, so the output is the exact
    k-NN of x among the refined reconstructions (search steps 1-3 of section 3.2)."""
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    dense = dense_reconstructions(index, refine=True)
    c = len(index.books.coarse)
    for x in X[:6]:
        ids, dist, tr = orc.search_one(x, index, c, index.N, 20)
        assert tr.scanned == index.N
        D = ((dense - x.astype(np.float64)) ** 2).sum(axis=1)
        order = np.lexsort((index.ids, D))[:20]
        assert ids.tolist() == index.ids[order].tolist()
        assert np.allclose(dist, D[order], rtol=1e-12)


def test_lattice_database_gives_exact_distances():
    """Vectors that are themselves reproduction values (coarse + q_c + q_r lattice, scales
    separated so the encoders recover the generating codes) have zero quantization error:
    Eq. (10) equals the true squared distance and the search returns the exact neighbours."""
    rng = np.random.default_rng(5)
    d, c, m, mr, N = 16, 6, 4, 8, 800
    coarse = (rng.normal(size=(c, d)) * 100).astype(np.float32)
    pq = (rng.normal(size=(m, 256, d // m)) * 2.0).astype(np.float32)
    rq = (rng.normal(size=(mr, 256, d // mr)) * 1e-3).astype(np.float32)
    books = orc.Codebooks(coarse, pq, rq)
    l0 = rng.integers(0, c, N)
    c0 = rng.integers(0, 256, (N, m)).astype(np.uint8)
    r0 = rng.integers(0, 256, (N, mr)).astype(np.uint8)
    Y = coarse[l0].astype(np.float64) + orc.pq_decode(c0, pq) + orc.pq_decode(r0, rq)
    lists, codes, rcodes = orc.encode(Y, books)
    assert np.array_equal(lists, l0) and np.array_equal(codes, c0)
    index = orc.assemble_index(lists, np.arange(N), codes, rcodes, books)
    X = rng.normal(size=(5, d)) * 100
    true_i, true_d = orc.brute_force(X, Y, 5)
    ids, dist, _ = orc.search(X, index, c, N, 5)
    assert np.array_equal(ids, true_i)
    assert np.allclose(dist, true_d, rtol=1e-9)
    assert orc.recall_at(ids, true_i[:, 0], 1) == 1.0


def test_bruteforce_and_recall_definition():
    rng = np.random.default_rng(2)
    Y = rng.integers(0, 256, (200, 8)).astype(np.uint8)
    X = rng.integers(0, 256, (3, 8)).astype(np.uint8)
    ids, dist = orc.brute_force(X, Y, 4)
    for q in range(3):
        d_all = [sum((int(X[q, t]) - int(Y[i, t])) ** 2 for t in range(8)) for i in range(200)]
        order = sorted(range(200), key=lambda i: (d_all[i], i))[:4]
        assert ids[q].tolist() == order and dist[q].tolist() == [d_all[i] for i in order]
    res = np.array([[5, 1, 2], [0, 9, 3], [4, 4, 4]])
    nn = np.array([1, 3, 7])
    assert orc.recall_at(res, nn, 1) == 0.0
    assert orc.recall_at(res, nn, 2) == pytest.approx(1 / 3)
    assert orc.recall_at(res, nn, 3) == pytest.approx(2 / 3)


def test_inverted_lists_hold_every_id_once_in_ascending_order():
    wl = tiny_workload()
    index = wl["index"]
    assert sorted(index.ids.tolist()) == list(range(index.N))
    lists = orc.nearest(wl["Y"].astype(np.float64), index.books.coarse)
    for l in range(len(index.list_offsets) - 1):
        seg = index.ids[index.list_offsets[l]:index.list_offsets[l + 1]]
        assert np.all(np.diff(seg) > 0)
        assert np.array_equal(np.sort(np.nonzero(lists == l)[0]), seg)
    # memory per vector: m + m' bytes of codes (section 3.1) + 4 for the inverted file (section 3.3)
    assert index.bytes_per_vector() == 4 + 4 + 4


def test_short_results_are_padded():
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    n0 = int(index.list_offsets[1] - index.list_offsets[0])
    # visiting one list cannot return more than that list holds
    ids, dist, tr = orc.search_one(X[0], index, 1, 10 ** 6, 10 ** 4)
    assert (ids >= 0).sum() == tr.scanned and np.isinf(dist[tr.scanned:]).all()
    assert n0 >= 0


# ---------------------------------------------------------------- closed forms / shape of Table 1

def test_scanned_fraction_is_about_v_over_c():
    """Section 3.3: estimators are computed for a fraction of the order of v/c of the database."""
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    c = len(index.books.coarse)
    for w in (1, 2, 4):
        frac = np.mean([orc.search_one(x, index, w, 10, 5)[2].scanned for x in X]) / index.N
        assert 0.4 * w / c < frac < 3.0 * w / c
    assert orc.search_one(X[0], index, c, 10, 5)[2].scanned == index.N


def _table1():
    rows = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "table1_recall.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        meth, mr, r1, r10, r100, t = line.split()
        rows[(meth, int(mr))] = (float(r1), float(r10), float(r100), float(t))
    return rows


def test_refinement_reduces_error_and_recall_orders_as_table1():
    """Table 1: recall@r rises with m' and IVFADC+R >= IVFADC; the reconstruction error falls
    as refinement bytes are added (section 3.1).  Checked on the synthetic data; the table's
    absolute values need BIGANN."""
    t1 = _table1()
    for r in range(3):
        seq = [t1[("IVFADC", 0)][r]] + [t1[("IVFADC+R", mr)][r] for mr in (8, 16, 32)]
        assert seq == sorted(seq)
    errs, recalls = [], []
    for mr in (0, 4, 16):
        wl = tiny_workload(N=4000, n_query=40, m_refine=mr)
        index, X, Y = wl["index"], wl["X"], wl["Y"]
        dense = dense_reconstructions(index, refine=True)
        errs.append(((dense - Y[index.ids].astype(np.float64)) ** 2).sum(axis=1).mean())
        true_i, _ = orc.brute_force(X, Y, 1)
        ids, _, _ = orc.search(X, index, 4, 200, 10)
        recalls.append([orc.recall_at(ids, true_i[:, 0], r) for r in (1, 10)])
    assert errs[0] > errs[1] > errs[2]
    assert recalls[2][0] >= recalls[0][0] and recalls[2][1] >= recalls[0][1] - 1e-9
    assert recalls[2][0] > recalls[0][0]


# ---------------------------------------------------------------- planted mistakes must trip a pin

@pytest.mark.parametrize("mistake", ["drop_coarse", "wrong_sign", "interleaved_split", "refine_ignored"])
def test_planted_mistakes_are_caught(monkeypatch, mistake):
    wl = tiny_workload()
    index, X = wl["index"], wl["X"]
    dense_ref = dense_reconstructions(index, refine=True)
    dense_adc = dense_reconstructions(index, refine=False)

    def invariants():
        x = X[0]
        est = orc.adc_scan(x, index, 2)
        a, b = index.list_offsets[2], index.list_offsets[3]
        assert np.allclose(est, ((dense_adc[a:b] - x.astype(np.float64)) ** 2).sum(axis=1), rtol=1e-12)
        ids, dist, _ = orc.search_one(x, index, len(index.books.coarse), index.N, 10)
        D = ((dense_ref - x.astype(np.float64)) ** 2).sum(axis=1)
        order = np.lexsort((index.ids, D))[:10]
        assert ids.tolist() == index.ids[order].tolist() and np.allclose(dist, D[order], rtol=1e-12)

    invariants()
    if mistake == "drop_coarse":
        real = orc.reconstruct
        monkeypatch.setattr(orc, "reconstruct", lambda idx, e, l, refine=True:
                            real(idx, e, l, refine) - idx.books.coarse[l].astype(np.float64))
    elif mistake == "wrong_sign":
        real_t = orc.lookup_tables
        monkeypatch.setattr(orc, "lookup_tables", lambda x, cen, pq: real_t(x, -np.asarray(cen), pq))
    elif mistake == "interleaved_split":
        def bad_tables(x, cen, pq):
            m, _, sub = pq.shape
            r = np.asarray(x, dtype=np.float64) - np.asarray(cen, dtype=np.float64)
            T = np.empty((m, 256))
            for j in range(m):
                T[j] = ((r[j::m][None, :] - pq[j].astype(np.float64)) ** 2).sum(axis=1)
            return T
        monkeypatch.setattr(orc, "lookup_tables", bad_tables)
    elif mistake == "refine_ignored":
        real = orc.reconstruct
        monkeypatch.setattr(orc, "reconstruct", lambda idx, e, l, refine=True: real(idx, e, l, False))
    with pytest.raises(AssertionError):
        invariants()
