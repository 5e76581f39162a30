"""Seeded synthetic 128-d uint8 vectors (numpy implementation).

Stands in for the BIGANN SIFT descriptors of the paper's section 4.1 (one billion
128-dimensional byte vectors, 10k queries, a separate learning set), which are not
available offline.  Every vector is drawn from a Gaussian mixture: G components with
centres uniform in [0,100)^d, per-dimension sigma 20, rounded and clipped to [0,255].

The generator is counter based: any vector of any stream can be produced alone from
(seed, stream, index), so a base set of 10^9 vectors is made chunk by chunk on either
side and never stored.  This module holds no arithmetic of the search method; it is the
one module the CPU oracle and the GPU library's tests both draw inputs from.  A HIP
implementation of the same integer recipe lives beside it (gen.hip) and must produce
the same bytes.

Recipe for vector i of a stream with 64-bit key K:
  h(t)   = mix64(K + (t + 1) * GOLDEN)      (the splitmix64 output function)
  comp   = number of entries of the cumulative uint32 weight table that are
           <= (h(64 i) >> 32), clipped to G-1
  for r in 1..d/4:  h(64 i + r) supplies four 16-bit fields u (low field first) for
                    dimensions 4(r-1) .. 4(r-1)+3
  value  = clip(rint(fp32(centre[comp][e]) + gauss_table[u]), 0, 255)  (one IEEE fp32 add,
           round-half-to-even)
The Gaussian table has 65536 fp32 entries  sigma * Phi^-1((u + 1/2) / 65536)  computed once
in float64; no transcendental is evaluated per sample.
"""
from __future__ import annotations

import dataclasses

import numpy as np
from scipy.special import ndtri

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

BASE_SEED = 11023828

STREAM_CENTRES = 1
STREAM_TRAIN = 2
STREAM_QUERY = 3
STREAM_INIT = 4          # k-means initial-centroid draws
STREAM_BASE0 = 16        # base chunk j uses stream 16 + j

BASE_CHUNK = 10_000_000  # vectors per base chunk (config 5 is built from 100 of them)


def mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 finalizer on uint64 arrays (wrapping arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def stream_key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        s = np.uint64(seed) * GOLDEN + np.uint64(stream)
    return mix64(mix64(s) + np.uint64(stream))


def hash_at(key: np.uint64, t: np.ndarray) -> np.ndarray:
    t = np.asarray(t, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return mix64(key + (t + np.uint64(1)) * GOLDEN)


def gauss_table(sigma: float = 20.0) -> np.ndarray:
    u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return (sigma * ndtri(u)).astype(np.float32)


@dataclasses.dataclass(frozen=True)
class Mixture:
    """Shared tables of one configuration's mixture (host arrays, passed to either generator)."""
    d: int
    centres: np.ndarray      # fp32 [G, d]
    cum_thresh: np.ndarray   # uint32 [G]: component g is chosen when cum[g-1] <= u < cum[g]
    gauss: np.ndarray        # fp32 [65536]
    seed: int

    @property
    def G(self) -> int:
        return self.centres.shape[0]


def make_mixture(G: int, d: int = 128, zipf: float | None = None, seed: int = BASE_SEED,
                 sigma: float = 20.0) -> Mixture:
    """Centres uniform in [0,100)^d; weights uniform, or proportional to rank^-zipf."""
    key = stream_key(seed, STREAM_CENTRES)
    h = hash_at(key, np.arange(G * d, dtype=np.uint64))
    centres = ((h >> np.uint64(40)).astype(np.float64) * (100.0 / float(1 << 24))).astype(np.float32)
    centres = centres.reshape(G, d)
    if zipf is None:
        wts = np.full(G, 1.0 / G)
    else:
        wts = np.arange(1, G + 1, dtype=np.float64) ** (-float(zipf))
        wts /= wts.sum()
    cum = np.cumsum(wts)
    cum_thresh = np.minimum(np.floor(cum * 4294967296.0), 4294967295.0).astype(np.uint32)
    cum_thresh[-1] = np.uint32(4294967295)
    return Mixture(d=d, centres=centres, cum_thresh=cum_thresh, gauss=gauss_table(sigma), seed=seed)


def gen_vectors(mix: Mixture, stream: int, start: int, n: int, return_comp: bool = False):
    """uint8 [n, d]: vectors start .. start+n-1 of the given stream."""
    d = mix.d
    assert d % 4 == 0 and d // 4 < 64
    key = stream_key(mix.seed, stream)
    out = np.empty((n, d), dtype=np.uint8)
    comp_all = np.empty(n, dtype=np.int32) if return_comp else None
    step = 1 << 16
    sh = (np.arange(4, dtype=np.uint64) * np.uint64(16))[None, None, :]
    for a in range(0, n, step):
        b = min(n, a + step)
        i = np.arange(start + a, start + b, dtype=np.uint64)
        u32 = (hash_at(key, i * np.uint64(64)) >> np.uint64(32)).astype(np.uint32)
        comp = np.searchsorted(mix.cum_thresh, u32, side="right")
        comp = np.minimum(comp, mix.G - 1)
        t = i[:, None] * np.uint64(64) + np.arange(1, d // 4 + 1, dtype=np.uint64)[None, :]
        h = hash_at(key, t)                                   # [b-a, d/4]
        u16 = ((h[:, :, None] >> sh) & np.uint64(0xFFFF)).astype(np.int64).reshape(b - a, d)
        v = mix.centres[comp] + mix.gauss[u16]                # one fp32 add
        v = np.clip(np.rint(v), 0.0, 255.0)
        out[a:b] = v.astype(np.uint8)
        if return_comp:
            comp_all[a:b] = comp
    return (out, comp_all) if return_comp else out


def base_chunk(mix: Mixture, chunk_idx: int, n: int = BASE_CHUNK, start: int = 0) -> np.ndarray:
    """Vectors start..start+n-1 of base chunk chunk_idx (global id = chunk_idx*BASE_CHUNK + index)."""
    return gen_vectors(mix, STREAM_BASE0 + chunk_idx, start, n)


def gen_base(mix: Mixture, N: int) -> np.ndarray:
    """The first N base vectors, concatenating chunks of BASE_CHUNK (host memory: N*d bytes)."""
    out = np.empty((N, mix.d), dtype=np.uint8)
    for j, a in enumerate(range(0, N, BASE_CHUNK)):
        b = min(N, a + BASE_CHUNK)
        out[a:b] = base_chunk(mix, j, b - a)
    return out


def draw_without_replacement(seed: int, stream: int, n: int, k: int) -> np.ndarray:
    """k distinct indices in [0, n): ranks of the k smallest hashes of 0..n-1 (ties by index)."""
    assert 0 < k <= n
    h = hash_at(stream_key(seed, stream), np.arange(n, dtype=np.uint64))
    order = np.lexsort((np.arange(n), h))
    return np.sort(order[:k]).astype(np.int64)


@dataclasses.dataclass(frozen=True)
class Config:
    """One workload: sizes and search parameters (c = coarse centroids, w = lists visited,
    m / m_refine = bytes of the first-stage and refinement codes)."""
    name: str
    N: int
    n_train: int
    n_query: int
    G: int
    zipf: float | None
    c: int
    m: int
    m_refine: int
    w: int
    kprime: int
    k: int
    d: int = 128
    batch: int = 1000   # queries handed to one search call

    def mixture(self) -> Mixture:
        return make_mixture(self.G, self.d, self.zipf)


CONFIGS = {
    "cfg0": Config("cfg0", 100_000, 10_000, 100, 256, None, 256, 8, 8, 8, 100, 10),
    "cfg1": Config("cfg1", 1_000_000, 100_000, 1000, 1024, None, 1024, 8, 16, 8, 1000, 100),
    "cfg2": Config("cfg2", 10_000_000, 1_000_000, 1000, 4096, None, 8192, 8, 32, 16, 1000, 100),
    "cfg3": Config("cfg3", 100_000_000, 1_000_000, 10_000, 16384, 1.1, 8192, 8, 16, 64, 10_000, 100),
    "cfg4": Config("cfg4", 1_000_000_000, 2_000_000, 10_000, 16384, 1.1, 8192, 8, 8, 64, 1000, 100),
}
