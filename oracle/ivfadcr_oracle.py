"""CPU oracle for IVFADC+R (index construction and search), numpy float64.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the GPU library
must compute, written from the paper "Searching in one billion vectors: re-rank with source
coding".  It shares no code with the HIP path and is imported only by tests, the smoke
check and the benchmark's cpu_baseline leg.  All arithmetic is float64 on the fp32
codebooks (the mathematical definition; the paper fixes no precision).

Notation follows the paper: d dimension, c coarse centroids, v lists visited (called w in
the library interface), m bytes of the first-stage product-quantizer code q_c, m' bytes of
the refinement code q_r, k' short-list length, k results.

Readings taken where the paper is silent (section 3.3 defers the inverted-file details to
the product-quantization paper it cites):
  * the first-stage product quantizer encodes the residual of a vector to its coarse
    centroid, so the explicit approximation of y is  coarse[l(y)] + decode_P(code)  and the
    look-up tables of Eq. (5) are built from  x - coarse[l]  for every visited list l;
  * the refinement quantizer of Eq. (8) encodes  y - coarse[l(y)] - decode_P(code);
  * sub-vectors are contiguous slices in natural dimension order (section 2, Eq. (4));
  * 8 bits per sub-quantizer (section 2 last paragraph, section 3.1 last paragraph);
  * every argmin / top-k breaks ties towards the lowest index (centroid index, list index
    or vector id); entries of an inverted list are kept in ascending id order;
  * distances are squared L2 throughout (Eq. (1)-(10));
  * k-means: Lloyd iterations from given initial points; an empty cluster keeps its
    previous centroid.

Pins (tests/test_oracle_*.py): ADC table sum == distance to the decoded vector (Eq. (1) =
Eq. (5)); m' = 0 reduces to plain IVFADC (Table 1 rows with m' = 0); v = c and k' = n gives
the exact ordering over reconstructions (search steps 1-3 of section 3.2); data on the
quantizer lattice gives exact distances; encoders are brute-force argmins (Eq. (8)); the
distance routine is checked against hand loops; k-means against a library Lloyd and its
monotone objective; the truncated query stage (v < c lists visited, k' below what is scanned)
against explicit loops and sorted() over (distance, index) tuples, with constructed exact ties
at the v-th list, the k'-th estimate and the k-th refined distance; train() against a
training set planted on a three-level lattice that the coarse quantizer, q_c and q_r must
recover level by level (Eq. (7)).  Absolute recall values of Table 1 need the BIGANN data: parity
unpinned for those (only the table's ordering in m' is checked).
"""
from __future__ import annotations

import dataclasses

import numpy as np
from scipy.spatial.distance import cdist

KS = 256  # reproduction values per sub-quantizer: 8 bits (section 2, last paragraph)


def sqdist(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """All squared Euclidean distances ||a - b||^2, float64 [len(A), len(B)] (Eq. (3) body)."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    return cdist(A, B, "sqeuclidean")


def argmin_rows(D: np.ndarray) -> np.ndarray:
    """Row-wise argmin, ties to the lowest index (numpy's argmin returns the first minimum)."""
    return np.argmin(D, axis=1)


def smallest(dist: np.ndarray, tiebreak: np.ndarray, count: int) -> np.ndarray:
    """Indices of the `count` smallest entries under the total order (dist, tiebreak), ascending."""
    order = np.lexsort((tiebreak, dist))
    return order[:count]


def nearest(X: np.ndarray, C: np.ndarray, rows: int = 4096) -> np.ndarray:
    """argmin_l ||x - C[l]||^2 for each row of X (rows are independent; processed in slabs
    only to bound memory)."""
    out = np.empty(len(X), dtype=np.int64)
    for a in range(0, len(X), rows):
        out[a:a + rows] = argmin_rows(sqdist(X[a:a + rows], C))
    return out


def kmeans(X: np.ndarray, init: np.ndarray, iters: int):
    """Lloyd's algorithm (named in section 2 for every sub-quantizer and used for the coarse
    quantizer).  X float [n, dim]; init float [K, dim] starting centroids.  Returns
    (centroids fp32 [K, dim], objective per iteration = mean squared distance to the
    assigned centroid, measured before that iteration's update)."""
    X = np.asarray(X, dtype=np.float64)
    C = np.array(init, dtype=np.float64)
    K = len(C)
    history = []
    for _ in range(iters):
        assign = np.empty(len(X), dtype=np.int64)
        err = 0.0
        for a in range(0, len(X), 4096):
            D = sqdist(X[a:a + 4096], C)
            assign[a:a + 4096] = argmin_rows(D)
            err += D[np.arange(len(D)), assign[a:a + 4096]].sum()
        history.append(err / len(X))
        counts = np.bincount(assign, minlength=K)
        sums = np.zeros_like(C)
        np.add.at(sums, assign, X)
        filled = counts > 0
        C[filled] = sums[filled] / counts[filled, None]
    return C.astype(np.float32), history


def subvectors(V: np.ndarray, parts: int) -> np.ndarray:
    """Split [n, d] into `parts` contiguous sub-vectors: [n, parts, d/parts] (Eq. (4))."""
    n, d = V.shape
    assert d % parts == 0
    return V.reshape(n, parts, d // parts)


def pq_encode(V: np.ndarray, book: np.ndarray) -> np.ndarray:
    """Product-quantizer codes: code[i, j] = argmin_k ||V[i]^j - book[j, k]||^2
    (Eq. (4); Eq. (8) when V holds residuals).  book fp32 [parts, 256, d/parts]."""
    parts = book.shape[0]
    S = subvectors(np.asarray(V, dtype=np.float64), parts)
    codes = np.empty((len(V), parts), dtype=np.uint8)
    for j in range(parts):
        codes[:, j] = nearest(S[:, j, :], book[j])
    return codes


def pq_decode(codes: np.ndarray, book: np.ndarray) -> np.ndarray:
    """Reproduction value of each code: concatenation of the selected sub-centroids."""
    parts, _, sub = book.shape
    out = np.empty((len(codes), parts * sub), dtype=np.float64)
    for j in range(parts):
        out[:, j * sub:(j + 1) * sub] = book[j][codes[:, j]].astype(np.float64)
    return out


@dataclasses.dataclass
class Codebooks:
    coarse: np.ndarray            # fp32 [c, d]
    pq: np.ndarray                # fp32 [m, 256, d/m]
    rq: np.ndarray | None         # fp32 [m', 256, d/m'] or None when m' = 0

    @property
    def m_refine(self) -> int:
        return 0 if self.rq is None else self.rq.shape[0]


def train(train_set: np.ndarray, c: int, m: int, m_refine: int, iters: int,
          init_coarse: np.ndarray, init_pq: np.ndarray, init_rq: np.ndarray | None,
          history: dict | None = None) -> Codebooks:
    """Offline step 1 (section 3.2): learn the coarse quantizer, q_c and q_r on one training
    set.  init_* are row indices into train_set (drawn outside: the method's random choices
    are inputs).  init_pq [m, 256], init_rq [m', 256]."""
    T = np.asarray(train_set, dtype=np.float64)
    coarse, h = kmeans(T, T[init_coarse], iters)
    if history is not None:
        history["coarse"] = h
    lists = nearest(T, coarse)
    r1 = T - coarse[lists].astype(np.float64)
    S = subvectors(r1, m)
    pq = np.empty((m, KS, T.shape[1] // m), dtype=np.float32)
    for j in range(m):
        pq[j], h = kmeans(S[:, j, :], S[init_pq[j], j, :], iters)
        if history is not None:
            history[f"pq{j}"] = h
    rq = None
    if m_refine:
        r2 = r1 - pq_decode(pq_encode(r1, pq), pq)      # Eq. (7) for the training vectors
        S2 = subvectors(r2, m_refine)
        rq = np.empty((m_refine, KS, T.shape[1] // m_refine), dtype=np.float32)
        for j in range(m_refine):
            rq[j], h = kmeans(S2[:, j, :], S2[init_rq[j], j, :], iters)
            if history is not None:
                history[f"rq{j}"] = h
    return Codebooks(coarse, pq, rq)


def encode(Y: np.ndarray, books: Codebooks):
    """Offline steps 2-3 (section 3.2) for database vectors Y: coarse list, q_c code of the
    coarse residual, q_r code of what q_c leaves (Eq. (7), (8))."""
    Yf = np.asarray(Y, dtype=np.float64)
    lists = nearest(Yf, books.coarse)
    r1 = Yf - books.coarse[lists].astype(np.float64)
    codes = pq_encode(r1, books.pq)
    if books.rq is None:
        rcodes = np.zeros((len(Y), 0), dtype=np.uint8)
    else:
        r2 = r1 - pq_decode(codes, books.pq)
        rcodes = pq_encode(r2, books.rq)
    return lists, codes, rcodes


@dataclasses.dataclass
class Index:
    """Inverted file (section 3.3): list l holds entries list_offsets[l] .. list_offsets[l+1]-1
    of the flat arrays, in ascending id order."""
    books: Codebooks
    list_offsets: np.ndarray      # int64 [c+1]
    ids: np.ndarray               # int32 [N]
    codes: np.ndarray             # uint8 [N, m]
    rcodes: np.ndarray            # uint8 [N, m']

    @property
    def N(self) -> int:
        return len(self.ids)

    def list_of_entry(self) -> np.ndarray:
        return np.repeat(np.arange(len(self.list_offsets) - 1), np.diff(self.list_offsets))

    def bytes_per_vector(self) -> int:
        """m + m' code bytes (section 3.1) + 4 for the inverted-file id (section 3.3)."""
        return self.codes.shape[1] + self.rcodes.shape[1] + 4


def build_index(Y: np.ndarray, ids: np.ndarray, books: Codebooks) -> Index:
    lists, codes, rcodes = encode(Y, books)
    return assemble_index(lists, ids, codes, rcodes, books)


def assemble_index(lists, ids, codes, rcodes, books: Codebooks) -> Index:
    c = len(books.coarse)
    order = np.lexsort((ids, lists))
    offsets = np.zeros(c + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(np.bincount(lists, minlength=c))
    return Index(books, offsets, np.asarray(ids)[order].astype(np.int32),
                 np.ascontiguousarray(codes[order]), np.ascontiguousarray(rcodes[order]))


def reconstruct(index: Index, entries: np.ndarray, lists: np.ndarray, refine: bool = True) -> np.ndarray:
    """Explicit approximation of the given index entries: coarse centroid + decoded q_c code,
    plus the decoded refinement code when refine (Eq. (9))."""
    b = index.books
    y = b.coarse[lists].astype(np.float64) + pq_decode(index.codes[entries], b.pq)
    if refine and b.rq is not None:
        y = y + pq_decode(index.rcodes[entries], b.rq)
    return y


def lookup_tables(x: np.ndarray, centroid: np.ndarray, pq: np.ndarray) -> np.ndarray:
    """Tables of Eq. (5) for one query and one visited list: T[j, k] = ||(x - centroid)^j - pq[j, k]||^2."""
    m, _, sub = pq.shape
    r = np.asarray(x, dtype=np.float64) - np.asarray(centroid, dtype=np.float64)
    T = np.empty((m, KS), dtype=np.float64)
    for j in range(m):
        diff = r[j * sub:(j + 1) * sub][None, :] - pq[j].astype(np.float64)
        T[j] = (diff * diff).sum(axis=1)
    return T


def adc_scan(x: np.ndarray, index: Index, l: int) -> np.ndarray:
    """ADC estimator (Eq. (5)) of every entry of list l: the sum of m table look-ups."""
    a, b = index.list_offsets[l], index.list_offsets[l + 1]
    T = lookup_tables(x, index.books.coarse[l], index.books.pq)
    codes = index.codes[a:b]
    est = np.zeros(b - a, dtype=np.float64)
    for j in range(codes.shape[1]):
        est += T[j, codes[:, j]]
    return est


@dataclasses.dataclass
class QueryTrace:
    probe: np.ndarray          # visited lists, nearest first
    probe_d: np.ndarray        # their coarse distances
    short_entries: np.ndarray  # index entries of the short-list L, ordered by (estimate, id)
    short_est: np.ndarray      # their ADC estimates
    short_refined: np.ndarray  # their refined distances (Eq. (10))
    scanned: int               # number of entries whose estimator was computed


def search_one(x: np.ndarray, index: Index, w: int, kprime: int, k: int):
    """Query stage of section 3.2 on the inverted file of section 3.3, one query.
    Returns (ids int32 [k], squared distances float64 [k], trace); short results are padded
    with id -1 and distance +inf."""
    b = index.books
    x = np.asarray(x, dtype=np.float64)
    c = len(b.coarse)
    # visit the w lists whose coarse centroid is nearest to x
    Dc = sqdist(x[None, :], b.coarse)[0]
    probe = smallest(Dc, np.arange(c), w)
    # step 1: ADC estimates of every entry of the visited lists, k' smallest kept
    ent, est = [], []
    for l in probe:
        ent.append(np.arange(index.list_offsets[l], index.list_offsets[l + 1]))
        est.append(adc_scan(x, index, l))
    ent = np.concatenate(ent) if ent else np.zeros(0, dtype=np.int64)
    est = np.concatenate(est) if est else np.zeros(0)
    keep = smallest(est, index.ids[ent], min(kprime, len(ent)))
    L, L_est = ent[keep], est[keep]
    # step 2: explicit reconstruction (Eq. (9)) and refined distance (Eq. (10))
    L_lists = np.searchsorted(index.list_offsets, L, side="right") - 1
    yhat = reconstruct(index, L, L_lists, refine=True)
    diff = yhat - x[None, :]
    refined = (diff * diff).sum(axis=1)
    # step 3: the k smallest refined distances
    top = smallest(refined, index.ids[L], min(k, len(L)))
    ids = np.full(k, -1, dtype=np.int32)
    dist = np.full(k, np.inf)
    ids[:len(top)] = index.ids[L[top]]
    dist[:len(top)] = refined[top]
    return ids, dist, QueryTrace(probe, Dc[probe], L, L_est, refined, len(ent))


def search(X: np.ndarray, index: Index, w: int, kprime: int, k: int):
    ids = np.empty((len(X), k), dtype=np.int32)
    dist = np.empty((len(X), k))
    traces = []
    for i, x in enumerate(X):
        ids[i], dist[i], t = search_one(x, index, w, kprime, k)
        traces.append(t)
    return ids, dist, traces


def entry_of_id(index: Index) -> np.ndarray:
    """Inverse of index.ids for ids 0..N-1 (assumes ids are a permutation of 0..N-1)."""
    inv = np.empty(index.N, dtype=np.int64)
    inv[index.ids] = np.arange(index.N)
    return inv


def adc_distance(x: np.ndarray, index: Index, entry: int) -> float:
    """Eq. (1) for one index entry, by the look-up tables of Eq. (5)."""
    l = int(np.searchsorted(index.list_offsets, entry, side="right") - 1)
    T = lookup_tables(x, index.books.coarse[l], index.books.pq)
    return float(sum(T[j, index.codes[entry, j]] for j in range(index.codes.shape[1])))


def refined_distance(x: np.ndarray, index: Index, entry: int) -> float:
    """Eq. (10) for one index entry."""
    l = np.searchsorted(index.list_offsets, [entry], side="right") - 1
    y = reconstruct(index, np.array([entry]), l, refine=True)[0]
    diff = y - np.asarray(x, dtype=np.float64)
    return float((diff * diff).sum())


def brute_force(X: np.ndarray, Y: np.ndarray, k: int, ids: np.ndarray | None = None):
    """Exact k nearest neighbours of Eq. (3): ids [nq, k] and squared distances, order (dist, id)."""
    ids = np.arange(len(Y)) if ids is None else np.asarray(ids)
    out_i = np.empty((len(X), k), dtype=np.int64)
    out_d = np.empty((len(X), k))
    for a in range(0, len(X), 64):
        D = sqdist(X[a:a + 64], Y)
        for r in range(len(D)):
            o = smallest(D[r], ids, k)
            out_i[a + r], out_d[a + r] = ids[o], D[r][o]
    return out_i, out_d


def recall_at(result_ids: np.ndarray, true_nn: np.ndarray, r: int) -> float:
    """recall@r of section 4.2: fraction of queries whose true nearest neighbour is ranked in
    the first r returned positions."""
    hit = (result_ids[:, :r] == np.asarray(true_nn)[:, None]).any(axis=1)
    return float(hit.mean())
