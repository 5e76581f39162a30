"""Pins for the two parts of the CPU oracle that the invariant tests do not reach:

* the truncated query stage (fewer lists visited than exist, a short-list shorter than what is
  scanned): section 3.3's "v lists visited", step 1's "list L of k' hypotheses" and step 3 of
  section 3.2, re-derived here with explicit Python loops and sorted() over tuples, without a
  call into search_one or the routines it is built from;
* the offline stage (section 3.2 step 1, Eq. (7)-(8)): that q_c is learned on the residuals to
  the coarse centroid and q_r on what q_c leaves, pinned by a training set planted on a
  three-level lattice whose levels the three quantizers must recover exactly.

Every planted mistake at the end must trip one of these pins.
"""
import itertools

import numpy as np
import pytest

from oracle import ivfadcr_oracle as orc
from helpers import dense_reconstructions, tiny_workload


# ---------------------------------------------------------------- the query stage by hand

def hand_search(x, index, w, kprime, k, dense_adc, dense_ref):
    """Query steps 1-3 with plain loops.  dense_adc / dense_ref: every entry's first-stage and
    refined reconstruction (helpers.dense_reconstructions, loop-built).  Returns a dict."""
    b = index.books
    x = [float(v) for v in x]
    c, d = b.coarse.shape
    # the w lists whose centroid is nearest, ties to the lower list index
    dc = []
    for l in range(c):
        s = 0.0
        for t in range(d):
            s += (x[t] - float(b.coarse[l, t])) ** 2
        dc.append(s)
    probe = sorted(range(c), key=lambda l: (dc[l], l))[:w]
    # Eq. (1): the estimate of an entry is the squared distance to coarse + decoded q_c code
    scanned = []
    for l in probe:
        for e in range(int(index.list_offsets[l]), int(index.list_offsets[l + 1])):
            s = 0.0
            for t in range(d):
                s += (x[t] - dense_adc[e, t]) ** 2
            scanned.append((s, int(index.ids[e]), e))
    short = sorted(scanned)[:kprime]                       # by (estimate, id)
    # Eq. (10) on the short-list only
    refined = []
    for est, i, e in short:
        s = 0.0
        for t in range(d):
            s += (x[t] - dense_ref[e, t]) ** 2
        refined.append((s, i, e))
    top = sorted(refined)[:k]                              # by (refined distance, id)
    return dict(probe=probe, probe_d=[dc[l] for l in probe], scanned=len(scanned),
                short=short, refined=refined, ids=[i for _, i, _ in top], dist=[s for s, _, _ in top])


def check_against_hand(x, index, w, kprime, k, dense_adc, dense_ref):
    ref = hand_search(x, index, w, kprime, k, dense_adc, dense_ref)
    ids, dist, tr = orc.search_one(x, index, w, kprime, k)
    assert tr.probe.tolist() == ref["probe"]
    assert np.allclose(tr.probe_d, ref["probe_d"], rtol=1e-12, atol=1e-9)
    assert tr.scanned == ref["scanned"]
    assert tr.short_entries.tolist() == [e for _, _, e in ref["short"]]
    assert np.allclose(tr.short_est, [s for s, _, _ in ref["short"]], rtol=1e-11, atol=1e-9)
    assert np.allclose(tr.short_refined, [s for s, _, _ in ref["refined"]], rtol=1e-11, atol=1e-9)
    n = len(ref["ids"])
    assert ids[:n].tolist() == ref["ids"] and (ids[n:] == -1).all()
    assert np.allclose(dist[:n], ref["dist"], rtol=1e-11, atol=1e-9) and np.isinf(dist[n:]).all()
    return ref


def test_truncated_search_equals_hand_loops():
    """w < c and k' < entries scanned, on a trained tiny workload, for every query."""
    wl = tiny_workload(d=16, G=8, N=700, n_train=900, n_query=8, c=6, m=4, m_refine=4, iters=3)
    index, X = wl["index"], wl["X"]
    dense_adc = dense_reconstructions(index, refine=False)
    dense_ref = dense_reconstructions(index, refine=True)
    seen_truncation = 0
    for (w, kp, k), x in itertools.product(((2, 40, 7), (3, 5, 5), (1, 9, 3), (5, 10 ** 6, 12)), X):
        ref = check_against_hand(x, index, w, kp, k, dense_adc, dense_ref)
        seen_truncation += int(ref["scanned"] > kp and w < 6)
    assert seen_truncation >= 20      # the branch under test was really taken


def _tie_index():
    """A hand-made index with exact ties at all three decision boundaries.
    Lists 1 and 4 have identical centroids (equal coarse distance for every query: the lower
    list index must be visited first).  Entries with identical codes in those two lists have
    identical estimates and refined distances; the one in the list visited first carries the
    HIGHER id, so ordering ties by position in the scan differs from ordering them by id."""
    rng = np.random.default_rng(42)
    d, c, m, mr = 8, 6, 2, 2
    coarse = rng.normal(size=(c, d)) * 50
    coarse[4] = coarse[1]
    books = orc.Codebooks(coarse.astype(np.float32), (rng.normal(size=(m, 256, d // m)) * 6).astype(np.float32),
                          (rng.normal(size=(mr, 256, d // mr))).astype(np.float32))
    lists, ids, codes, rcodes = [], [], [], []
    nxt = 1000
    for l in range(c):
        for _ in range(30):
            lists.append(l); ids.append(nxt); nxt += 1
            codes.append(rng.integers(0, 256, m)); rcodes.append(rng.integers(0, 256, mr))
    # twins: same codes in list 1 (ids 900.., higher) and list 4 (ids 100.., lower)
    for t in range(12):
        cd, rc = rng.integers(0, 256, m), rng.integers(0, 256, mr)
        lists += [1, 4]; ids += [900 + t, 100 + t]; codes += [cd, cd]; rcodes += [rc, rc]
    index = orc.assemble_index(np.array(lists), np.array(ids), np.array(codes, dtype=np.uint8),
                               np.array(rcodes, dtype=np.uint8), books)
    return index


def test_ties_at_the_wth_list_the_kprime_th_estimate_and_the_kth_distance():
    index = _tie_index()
    dense_adc = dense_reconstructions(index, refine=False)
    dense_ref = dense_reconstructions(index, refine=True)
    coarse = index.books.coarse.astype(np.float64)
    rng = np.random.default_rng(7)
    cut_w = cut_kp = cut_k = 0
    for trial in range(12):
        x = coarse[1] + rng.normal(size=8) * 4          # lists 1 and 4 are the two nearest
        # (a) the w-th boundary falls between the twin lists: list 1 is visited, list 4 is not
        ref = check_against_hand(x, index, 1, 20, 5, dense_adc, dense_ref)
        assert ref["probe"] == [1]
        cut_w += 1
        # (b) both visited; cut the short-list between two twins: the lower id (list 4) stays
        full = hand_search(x, index, 2, 10 ** 6, 10 ** 6, dense_adc, dense_ref)
        order = full["short"]
        for pos in range(len(order) - 1):
            if order[pos][0] == order[pos + 1][0]:       # equal estimates: a twin pair
                assert order[pos][1] < order[pos + 1][1] and order[pos][1] < 900 <= order[pos + 1][1]
                ref = check_against_hand(x, index, 2, pos + 1, pos + 1, dense_adc, dense_ref)
                assert order[pos][1] in ref["ids"] and order[pos + 1][1] not in ref["ids"]
                cut_kp += 1
                break
        # (c) the k-th boundary between two twins of equal refined distance
        final = sorted(full["refined"])
        for pos in range(len(final) - 1):
            if final[pos][0] == final[pos + 1][0]:
                ref = check_against_hand(x, index, 2, 10 ** 6, pos + 1, dense_adc, dense_ref)
                assert ref["ids"][-1] == final[pos][1] and final[pos][1] < 900
                cut_k += 1
                break
    assert cut_w == 12 and cut_kp == 12 and cut_k == 12


# ---------------------------------------------------------------- the offline stage on a planted lattice

def _grid(dim, scale):
    """256 points {-1.5, -0.5, 0.5, 1.5}^4 (first four coordinates; the rest zero) times scale;
    point 255 - k is the mirror image of point k."""
    pts = np.zeros((256, dim))
    for k in range(256):
        for a in range(4):
            pts[k, a] = (((k >> (2 * a)) & 3) - 1.5) * scale
    assert np.array_equal(pts[::-1], -pts)
    return pts


def _lattice_training_set(seed=3):
    """Training vectors  C[l] + P[code] + R[rcode]  on three separated scales (100 / 1 / 0.01
    grid spacings).  Every vector comes with its three mirror images (code and / or rcode
    replaced by 255 - code), so inside every coarse cell the P and R parts average to zero and
    inside every q_c cell the R part does: Lloyd's fixed point from an initialisation with one
    row per cell is the lattice itself."""
    rng = np.random.default_rng(seed)
    d, c, m, mr = 8, 5, 2, 2
    C = rng.integers(-3, 4, size=(c, d)) * 100.0
    while len({tuple(r) for r in C.tolist()}) < c:
        C = rng.integers(-3, 4, size=(c, d)) * 100.0
    P = np.stack([_grid(d // m, 1.0) for _ in range(m)])
    R = np.stack([_grid(d // mr, 0.01) for _ in range(mr)])
    rows, lab = [], []
    for l in range(c):
        half_p = np.stack([rng.permutation(128) for _ in range(m)], axis=1)      # representatives of {k, 255-k}
        half_r = np.stack([rng.permutation(128) for _ in range(mr)], axis=1)
        flip_p = rng.integers(0, 2, size=(128, m))
        flip_r = rng.integers(0, 2, size=(128, mr))
        for u in range(128):
            code = np.where(flip_p[u] == 1, 255 - half_p[u], half_p[u])
            rcode = np.where(flip_r[u] == 1, 255 - half_r[u], half_r[u])
            for cp, cr in ((code, rcode), (code, 255 - rcode), (255 - code, rcode), (255 - code, 255 - rcode)):
                y = C[l].copy()
                for j in range(m):
                    y[j * (d // m):(j + 1) * (d // m)] += P[j, cp[j]]
                for j in range(mr):
                    y[j * (d // mr):(j + 1) * (d // mr)] += R[j, cr[j]]
                rows.append(y); lab.append((l, tuple(cp), tuple(cr)))
    T = np.array(rows)
    # initial rows: one per coarse cell; per sub-quantizer one row per code value
    init_c = np.array([next(i for i, t in enumerate(lab) if t[0] == l) for l in range(c)])
    init_p = np.array([[next(i for i, t in enumerate(lab) if t[1][j] == k) for k in range(256)] for j in range(m)])
    init_r = np.array([[next(i for i, t in enumerate(lab) if t[2][j] == k) for k in range(256)] for j in range(mr)])
    return T, lab, (C, P, R), (init_c, init_p, init_r), (c, m, mr)


def lattice_pin(train_fn):
    """The trained quantizers must be the planted lattice levels (Eq. (7): q_c sees y - coarse,
    q_r sees y - coarse - q_c)."""
    T, lab, (C, P, R), (ic, ip, ir), (c, m, mr) = _lattice_training_set()
    books = train_fn(T, c, m, mr, 3, ic, ip, ir)
    assert np.allclose(books.coarse, C, atol=1e-4)
    assert np.allclose(books.pq, P, atol=1e-4)          # centroid k was initialised inside cell k
    assert np.allclose(books.rq, R, atol=1e-5)
    # and the encoders recover the planted codes through all three levels
    lists, codes, rcodes = orc.encode(T, books)
    assert lists.tolist() == [t[0] for t in lab]
    assert codes.tolist() == [list(t[1]) for t in lab]
    assert rcodes.tolist() == [list(t[2]) for t in lab]


def test_training_recovers_a_planted_three_level_lattice():
    lattice_pin(orc.train)


def _train_with(pq_input, rq_input):
    """A trainer assembled from the oracle's primitives with a chosen (possibly wrong) input to
    each product quantizer: 'r1' residual to the coarse centroid, 'raw' the vectors themselves,
    'r2' what q_c leaves."""
    def fn(T, c, m, mr, iters, ic, ip, ir):
        T = np.asarray(T, dtype=np.float64)
        coarse, _ = orc.kmeans(T, T[ic], iters)
        r1 = T - coarse[orc.nearest(T, coarse)].astype(np.float64)
        src = {"raw": T, "r1": r1}[pq_input]
        S = orc.subvectors(src, m)
        pq = np.stack([orc.kmeans(S[:, j, :], S[ip[j], j, :], iters)[0] for j in range(m)])
        r2 = src - orc.pq_decode(orc.pq_encode(src, pq), pq)
        src2 = {"r1": r1, "r2": r2}[rq_input]
        S2 = orc.subvectors(src2, mr)
        rq = np.stack([orc.kmeans(S2[:, j, :], S2[ir[j], j, :], iters)[0] for j in range(mr)])
        return orc.Codebooks(coarse, pq, rq)
    return fn


def test_lattice_pin_catches_wrong_training_inputs():
    lattice_pin(_train_with("r1", "r2"))                 # the right chaining passes
    with pytest.raises(AssertionError):
        lattice_pin(_train_with("raw", "r2"))            # q_c learned on the vectors, not on residuals
    with pytest.raises(AssertionError):
        lattice_pin(_train_with("r1", "r1"))             # q_r learned on r1 instead of r2


# ---------------------------------------------------------------- planted mistakes in the query stage

@pytest.mark.parametrize("mistake", ["farthest_lists", "descending_probe_order", "kprime_off_by_one",
                                     "k_off_by_one", "tie_by_scan_position", "shortlist_by_refined"])
def test_planted_search_mistakes_are_caught(monkeypatch, mistake):
    """search_one calls smallest() three times: visited lists, short-list, final result.  Each
    planted mistake alters one of those selections; the hand-loop pins must notice."""
    wl = tiny_workload(d=16, G=8, N=700, n_train=900, n_query=8, c=6, m=4, m_refine=4, iters=3)
    index, X = wl["index"], wl["X"]
    dense = (dense_reconstructions(index, refine=False), dense_reconstructions(index, refine=True))
    tie_index = _tie_index()
    tie_dense = (dense_reconstructions(tie_index, refine=False), dense_reconstructions(tie_index, refine=True))

    def pins():
        for x in X[:4]:
            check_against_hand(x, index, 2, 40, 7, *dense)
        x = tie_index.books.coarse[1].astype(np.float64) + 0.5
        full = hand_search(x, tie_index, 2, 10 ** 6, 10 ** 6, *tie_dense)["short"]
        pos = next(p for p in range(len(full) - 1) if full[p][0] == full[p + 1][0])
        check_against_hand(x, tie_index, 2, pos + 1, pos + 1, *tie_dense)
        check_against_hand(x, tie_index, 1, 20, 5, *tie_dense)

    pins()
    real = orc.smallest
    calls = {"n": 0}

    def bad(dist, tiebreak, count):
        calls["n"] += 1
        which = (calls["n"] - 1) % 3          # 0 = lists, 1 = short-list, 2 = final
        if mistake == "farthest_lists" and which == 0:
            return real(-np.asarray(dist), tiebreak, count)
        if mistake == "descending_probe_order" and which == 0:
            return real(dist, tiebreak, count)[::-1]
        if mistake == "kprime_off_by_one" and which == 1:
            return real(dist, tiebreak, max(count - 1, 0))
        if mistake == "k_off_by_one" and which == 2:
            return real(dist, tiebreak, max(count - 1, 0))
        if mistake == "tie_by_scan_position" and which == 1:
            return real(dist, np.arange(len(dist)), count)
        if mistake == "shortlist_by_refined" and which == 1:
            return real(dist, tiebreak, count)[::-1]        # right members, wrong order in the trace
        return real(dist, tiebreak, count)

    monkeypatch.setattr(orc, "smallest", bad)
    with pytest.raises(AssertionError):
        pins()
