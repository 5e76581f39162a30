// Internal declarations shared by the translation units of libivfadcr (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdarg.h>
#include <stdio.h>
#include <vector>

#include "ivfadcr.h"

#define IVFR_KS 256            // reproduction values per sub-quantizer (8 bits)
#define IVFR_LIST_ALIGN 32u    // every inverted list starts at a multiple of 32 entries
#define IVFR_BLOCK 512u        // entries per scan block: one 16-byte load per thread of a 256-thread group
#define IVFR_SAMPLE_CHUNK 2048u   // entries of a sample prefix scored by one wavefront
#define IVFR_TAIL_PAD 1024u    // zero entries after the last list so vector loads never run off the end

void ivfr_set_error(const char* fmt, ...);

#define IVFR_HIP(expr)                                                                         \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) {                                                                \
            ivfr_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return (e_ == hipErrorOutOfMemory) ? IVFR_ERR_OOM : IVFR_ERR_HIP;                  \
        }                                                                                      \
    } while (0)

#define IVFR_TRY(expr)                  \
    do {                                \
        int r_ = (expr);                \
        if (r_ != IVFR_OK) return r_;   \
    } while (0)

#define IVFR_REQUIRE(cond, ...)              \
    do {                                     \
        if (!(cond)) {                       \
            ivfr_set_error(__VA_ARGS__);     \
            return IVFR_ERR_INVALID_ARG;     \
        }                                    \
    } while (0)

// Grow-only device buffer.
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    int reserve(size_t need) {
        if (need <= bytes) return IVFR_OK;
        if (p) { IVFR_HIP(hipFree(p)); p = nullptr; bytes = 0; }
        size_t want = need + need / 8 + 256;
        hipError_t e = hipMalloc(&p, want);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            p = nullptr;
            e = hipMalloc(&p, need);
            want = need;
        }
        if (e != hipSuccess) {
            (void)hipGetLastError();
            p = nullptr;
            ivfr_set_error("device allocation of %zu bytes failed", need);
            return IVFR_ERR_OOM;
        }
        bytes = want;
        return IVFR_OK;
    }
    void release() { if (p) (void)hipFree(p); p = nullptr; bytes = 0; }
    template <class T> T* as() const { return reinterpret_cast<T*>(p); }
};

// Status words of one internal batch of a search call.  They live in device memory, are cleared by the batch's
// first kernel, filled by the plan / scan / select kernels, and copied to a pinned host slot by one asynchronous
// copy at the end of the batch: the host reads them once, after the stream has drained.
struct DevStatus {
    unsigned long long totals[2];   // [0] sum over queries of the visited lists' lengths, [1] candidate-pool records the plan wants
    unsigned long long work[8];     // [0] list entries streamed; [1..5] estimates by units of eight, four, two, single pairs, units of 64
    int32_t over_total;             // queries whose filter failed its check (too many or too few survivors)
    uint32_t bad_query;             // row + 1 of a query with a component that is not finite (0: none)
    uint32_t pool_short;            // 1: the candidate pool is smaller than totals[1]; the batch did no list work
    uint32_t n_sample_chunks;       // chunks of the sample pass
    uint32_t counts[8];             // units of eight, four, two, single pairs, units of 64
};
#define IVFR_STATUS_SLOTS 16        // batches of one call in flight between two host waits
#define IVFR_REDO_CHUNK 4096        // failed-check flags read back per copy by the redo path
#define IVFR_STATIC_SCRATCH_BYTES (128u << 20)   // workspace of ivfr_search_static: one such array per device

// One staged (encoded, not yet list-sorted) batch of database vectors.
struct StagedChunk {
    int64_t n = 0;
    int32_t* list = nullptr;   // coarse list of each vector
    uint32_t* rank = nullptr;  // position inside that list (insertion order)
    int32_t* ids = nullptr;
    uint8_t* codes = nullptr;  // [n, m]
    uint8_t* rcodes = nullptr; // [n, m']
};

struct ivfr_index {
    ivfr_params p;
    int dsub = 0, dsub_r = 0;

    // codebooks (device) and their squared norms
    float* coarse = nullptr;       // [c, d]
    float* coarse_norm = nullptr;  // [c]
    float* pq = nullptr;           // [m, 256, dsub]
    float* pq_norm = nullptr;      // [m, 256]
    float* pq_maxnorm = nullptr;   // [m] largest centroid norm of each sub-quantizer
    float* rq = nullptr;           // [m', 256, dsub_r]
    float* list_term = nullptr;    // [c, m, 256] per-list part of the look-up tables (split tables), built on demand
    int split_tables = 0;          // 1: look-up tables are summed in the scan's prologue from list and query terms
    bool has_books = false;

    // staging
    std::vector<StagedChunk> staged;
    unsigned long long* list_fill = nullptr;  // [c] entries per list so far (device)
    int64_t n_added = 0;
    int64_t next_id = INT64_MIN;

    // finished inverted file (device, padded layout: list l occupies
    // [list_start[l], list_start[l] + list_len[l]) and list_start[l] % IVFR_LIST_ALIGN == 0)
    bool finalized = false;
    int64_t N = 0;
    uint64_t n_slots = 0;            // padded entry count incl. tail pad
    uint32_t* list_start = nullptr;  // [c+1]
    uint32_t* list_len = nullptr;    // [c]
    uint8_t* codes = nullptr;        // [n_slots, m]: the dense stream the list scan reads
    // One record per entry slot for everything that is fetched per candidate (re-rank, tie-breaks by id):
    //   int32 id | uint32 list | m code bytes | m' refinement code bytes | padding to rec_stride
    // rec_stride is a power of two up to 128 (a multiple of 64 beyond), so a record never straddles a 128-byte
    // line: a short-list candidate costs one line instead of three from separate id / code / refinement arrays.
    uint8_t* rec = nullptr;          // [n_slots, rec_stride]
    int rec_stride = 0;
    std::vector<int64_t> h_offsets;  // logical CSR offsets [c+1] (host)
    std::vector<uint32_t> h_start;   // padded starts [c+1] (host)

    // tuning
    int full_mult = 8, cap_mult = 16, batch = 16384, scan_groups = 0;
    int share_lists = -1;            // -1 = 2 or 0 by the size of the batch's scan; 0 = every pair on its own; 1 = fp32 units of four / two;
                                     // 2 = also fp16 units of eight; 3 = also matrix-core units of 64
    int min_cap = 8192;

    // scratch
    DevBuf search_ws, cand_ws, encode_ws, dense_ws;
    char* static_ws = nullptr;       // this device's copy of the static workspace array (address from the runtime)
    DevStatus* h_slots = nullptr;    // pinned host copies of the batches' status words [IVFR_STATUS_SLOTS]
    uint32_t* h_redo = nullptr;      // pinned scratch of the (rare) per-query redo path [16 + IVFR_REDO_CHUNK]
    hipStream_t side[4] = {nullptr, nullptr, nullptr, nullptr};   // the smaller scan launches overlap the large one
    hipEvent_t ev_fork[IVFR_STATUS_SLOTS] = {nullptr};            // one set of fork / join events per batch in flight
    hipEvent_t ev_join[IVFR_STATUS_SLOTS][4] = {{nullptr}};
    hipEvent_t ev_group[IVFR_STATUS_SLOTS][2] = {{nullptr}};      // the pair grouping of a batch runs beside its table kernel

    // stats of the last search
    int64_t st_reruns = 0;           // batches of the last search that ran twice (pool grown, or brought back for a redo)
    int64_t st_codes = 0, st_pairs = 0, st_dense = 0, st_streamed = 0, st_shared_codes = 0, st_shared2_codes = 0, st_shared8_codes = 0, st_retries = 0, st_shared64_codes = 0;
    int profiling = 0;   // 0 off, 1 list-scan launches only, 2 every stage
    std::vector<hipEvent_t> prof_events;   // timing events, created once and reused by every search call
    double prof_ms[IVFR_N_STAGES] = {0};
    int prof_scan_launches = 0;
    int n_cu = 256;
    // share of a batch's estimates that each scan launch computed in the previous call (units of eight, four, two,
    // single pairs, units of 64), relative to pairs x mean visited-list length: sizes the next call's launches
    double work_ratio[5] = {1.0, 1.0, 1.0, 1.0, 1.0};
    double wmean_len = 0.0;          // expected length of a visited list: sum of len^2 / N (lists are hit in proportion to their size)
    int64_t mem_limit = 0;           // > 0: device bytes the index may use in total (capacity checks refuse beyond it)
    size_t index_bytes = 0;          // device bytes held by the finished inverted file
};

// Device bytes of the finished inverted file with n_slots padded entry slots.
// Bytes between two records of the per-entry record array (see ivfr_index::rec).
inline int ivfr_record_stride(const ivfr_params& p) {
    const int need = 8 + p.m + p.m_refine;
    int r = 32;
    while (r < need && r < 128) r <<= 1;
    if (r < need) r = (need + 63) / 64 * 64;
    return r;
}
inline size_t ivfr_index_bytes(const ivfr_params& p, uint64_t n_slots) {
    return (size_t)n_slots * ((size_t)p.m + (size_t)ivfr_record_stride(p)) + ((size_t)p.c * 2 + 1) * sizeof(uint32_t);
}
// IVFR_ERR_OOM (before anything is allocated) when `more` further device bytes do not fit: beyond the index's
// memory limit, when one is set, or beyond what the device reports as free.
int ivfr_check_room(const ivfr_index* ix, size_t more);
// Address of the current device's copy of the static workspace array (search.hip).
int ivfr_static_scratch_address(int device, char** out);
// Allocates and fills the per-list term table of the split look-up tables if the index does not hold it yet.
int ivfr_ensure_list_terms(ivfr_index* ix, hipStream_t st);

// ---- kernels' host launchers (each enqueues on `st` and returns a status) -------------------

// squared norms of the rows of X [n, dim]
// bad (optional, zero on entry) is raised to row + 1 for a row whose squared norm is NaN, infinite or overflows
int ivfr_launch_row_norms(const float* X, int64_t n, int dim, float* out, hipStream_t st, uint32_t* bad = nullptr);
int ivfr_launch_group_max_norm(const float* norm2, int groups, int per, float* out, hipStream_t st);
// uint8 [n, d] -> fp32
int ivfr_launch_u8_to_f32(const uint8_t* x, int64_t count, float* out, hipStream_t st);

// fp32 MFMA distance GEMM: rows X [n, d] against centroids C [c, d].
//  keys[row * c + col] = (bits(max(0, ||x||^2 + ||c||^2 - 2 x.c)) << 32) | col
int ivfr_launch_dist_keys(const float* X, const float* xnorm, int64_t n, const float* C, const float* cnorm,
                          int c, int d, uint64_t* keys, hipStream_t st);
//  assign[row] = argmin_col (||c||^2 - 2 x.c), ties to the lowest col
int ivfr_launch_assign(const float* X, int64_t n, const float* C, const float* cnorm, int c, int d,
                       int32_t* assign, hipStream_t st);

// Where each query's candidate records live: query q owns cap(q) records from base(q).  Either
// per-query arrays (off, capq) or a uniform (stride, ucap) layout.
struct CandLayout {
    const unsigned long long* off = nullptr;
    const uint32_t* capq = nullptr;
    uint64_t stride = 0;
    uint32_t ucap = 0;
    __host__ __device__ uint64_t base(int q) const { return off ? off[q] : (uint64_t)q * stride; }
    __host__ __device__ uint32_t cap(int q) const { return capq ? capq[q] : ucap; }
};

// Segmented exact top-K by 64-bit key (ascending).  One workgroup per segment (select.hip).
struct SelectArgs {
    int nseg = 0;
    int K = 0;
    // source A: keys[seg * seg_stride + i], i < count
    const uint64_t* keys = nullptr;
    int64_t seg_stride = 0;
    int64_t fixed_count = 0;   // elements per segment (source A)
    // source B: records (estimate bits, entry position) with key = (estimate bits << 32) | ids[position];
    // segment q holds min(counts[q], lay.cap(q)) records from lay.base(q)
    const uint2* recs = nullptr;
    const int32_t* ids = nullptr;      // id of the entry at position pos is ids[pos * id_stride]
    uint32_t id_stride = 1;            // in 32-bit words (the ids sit at the start of the per-entry records)
    const uint32_t* counts = nullptr;
    CandLayout lay;
};
// Bound on the k'-th smallest estimate of each query from its uniform sample (a.counts records of the
// query's sq visited entries): tau = the r-th smallest sampled estimate, r = mu + 5 sqrt(mu) + 6 with
// mu = k' * sampled / sq the expected number of the true k' best inside the sample (+inf when the
// sample holds fewer than r).  fixed_rank > 0 takes that rank instead.  skip[seg] != 0 leaves tau alone.
// tau_id (optional) receives the id of the record taken, i.e. the low half of its key.  values_only: segment
// q holds counts[q] bare estimates (4 bytes each) from the start of its record buffer instead of records.
// mostly_skipped: the caller expects nearly every segment to be skipped (a few workgroups then walk over them).
int ivfr_launch_select_tau(const SelectArgs& a, const unsigned long long* sq, int kprime, int fixed_rank,
                           const uint8_t* skip, float* tau, uint32_t* tau_id, hipStream_t st,
                           bool values_only = false, bool mostly_skipped = false);
int ivfr_select_init();   // one-time function attributes

// Per-query part of the search plan, shared by the plan kernel and by the host's estimate of the candidate
// pool.  A query that visits `total` entries keeps every estimate when total <= full_limit (or when its sample
// would be a third of them or more); otherwise a sample bounds the k'-th smallest estimate.  Scoring a sampled
// entry and handling a surviving one cost about the same order, and the survivors fall as k' (1 + 5/sqrt(mu) + 6/mu)
// with mu = k' n_s / (entries sampled from), so the cheapest sample size n_s grows as the cube root of k' * total
// (the factor 16 is measured).  Where that leaves mu small (a short-list that is tiny against the visit: mu = 3 at
// 10^7 visited entries and k' = 1000) the sample is drawn from the nearest visited lists only: the lists in probe
// order up to the first that brings their entries to `total_u` = k' n_s / 16 (mu = 16), but not fewer than
// total / IVFR_SAMPLE_NEAR_DIV or 8 k'.  Any subset of the visited entries with k' members at or below a bound makes
// the bound valid for the whole visit; the nearest lists hold most of the short-list, their tables are a fraction
// of the tables the sample has to load, and the larger mu means a tighter rank.  One entry in `stride` of the
// sampled lists is taken (the same leading fraction of each); the stride is at most stride_k (= k' / mu_min) and
// at least what keeps the sample below max_sample.
#define IVFR_SAMPLE_NEAR_DIV 4
#ifndef IVFR_SAMPLE_FACTOR
#define IVFR_SAMPLE_FACTOR 16.0   // n_s = factor * (k' total)^(1/3)
#endif
struct QueryPlan {
    bool fully;
    uint32_t stride;
};
// entries of the nearest lists that the sample is drawn from, given the whole visit (the plan kernel walks the
// lists up to this threshold; the host's estimate takes the threshold itself)
__host__ __device__ inline unsigned long long ivfr_sample_threshold(unsigned long long total, int kprime) {
    const double kp = (double)(kprime > 0 ? kprime : 1);
    const double want = kp * (IVFR_SAMPLE_FACTOR / 16.0) * cbrt(kp * (double)total);   // k' n_s / 16: mu = 16
    unsigned long long t = want >= (double)total ? total : (unsigned long long)want;
    if (t < total / IVFR_SAMPLE_NEAR_DIV) t = total / IVFR_SAMPLE_NEAR_DIV;
    if (t < 8ull * (unsigned long long)kp) t = 8ull * (unsigned long long)kp;
    return t < total ? t : total;
}
__host__ __device__ inline QueryPlan ivfr_plan_query(unsigned long long total, unsigned long long total_u,
                                                     uint32_t full_limit, uint32_t stride_k, uint32_t max_sample,
                                                     int kprime) {
    QueryPlan r;
    r.fully = total <= full_limit;
    const double ns = IVFR_SAMPLE_FACTOR * cbrt((double)kprime * (double)total);
    unsigned long long strides[2];   // one entry in strides[0] of the whole visit, in strides[1] of the nearest lists
    const unsigned long long sizes[2] = {total, total_u};
    for (int i = 0; i < 2; ++i) {
        const double st_d = (double)sizes[i] / (ns > 1.0 ? ns : 1.0);
        unsigned long long st = st_d > 4.0e9 ? 4000000000ull : (unsigned long long)st_d;
        if (st > (stride_k < 1 ? 1ull : stride_k)) st = stride_k < 1 ? 1ull : stride_k;
        const unsigned long long widen = (sizes[i] + max_sample - 1) / max_sample;
        if (widen > st) st = widen;
        if (st < 1) st = 1;
        strides[i] = st;
    }
    if (strides[0] <= 3) r.fully = true;   // a sample of a third or more of the entries saves nothing
    r.stride = (uint32_t)(strides[1] > 0xFFFFFFFFull ? 0xFFFFFFFFull : strides[1]);
    return r;
}
// Records of the query's candidate buffer: everything (no filter), or the largest of the sample, min_cap and the
// survivors expected from the bound plus six deviations.  The bound is the rank-th smallest of the sample, one
// sampled entry standing for `stride` entries of the sampled lists; how many entries of the other lists lie below
// it is not known beforehand, so the buffer allows for the case that they are as dense there as in the sampled
// lists (total / total_u times as many).  exact_only: so large a share of the estimates will pass the bound that
// the half-precision units do not pay off.
__host__ __device__ inline unsigned long long ivfr_plan_capacity(unsigned long long total, unsigned long long total_u,
                                                                 unsigned long long sampled, QueryPlan qp,
                                                                 uint32_t min_cap, int kprime, float half_frac,
                                                                 bool* exact_only) {
    unsigned long long capv = total;
    *exact_only = true;
    if (!qp.fully) {
        const double mu = (double)kprime / (double)qp.stride;
        const double rank = mu + 5.0 * sqrt(mu) + 6.0;
        const double spread = (double)total / (double)(total_u > 0 ? total_u : 1ull);
        const double expect_u = rank * (double)qp.stride;   // entries of the sampled lists below the bound
        capv = sampled > min_cap ? sampled : (unsigned long long)min_cap;
        // the number of visited entries below the rank-th sampled one scatters by ~1/sqrt(rank): six deviations
        const double roomy = expect_u * spread * (1.0 + 6.0 / sqrt(rank));
        if ((double)capv < roomy) capv = (unsigned long long)roomy;
        // what is likely rather than what is possible: the other lists add a quarter
        *exact_only = expect_u * (spread < 1.25 ? spread : 1.25) > (double)half_frac * (double)total;
    }
    if (capv > 0xFFFFFFF0ull) capv = 0xFFFFFFF0ull;
    return capv;
}

// Where the scan kernels get the look-up table of a (query, list) pair from (Eq. (5)).
//  materialised: lut[pair][j][k], written per batch by the table kernel;
//  split:        ||(x - c_l)^j - p_jk||^2 = ||(x - c_l)^j||^2 + (||p_jk||^2 + 2 c_l^j . p_jk) - 2 x^j . p_jk:
//                the bracket is a per-list table kept with the index (list_term[l][j][k]), the last term a
//                per-query table (lut[query][j][k]), the first a per-pair scalar (pbase[pair][j]); the entry is
//                max(0, (list_term + query term) + pbase), evaluated by the same expression wherever it is needed
//                (table prologues and exact re-evaluations alike), so every kernel sees the same bits.
struct PairTable {
    const float* a;      // the pair's materialised table, or its list's term table   [m][256]
    const float* b;      // nullptr, or the query's term table                         [m][256]
    const float* base;   // split: ||(x - c_l)^j||^2, j < m
    __device__ __forceinline__ float get(int e) const {   // e = j * 256 + k
        return b ? fmaxf(0.f, (a[e] + b[e]) + base[e >> 8]) : a[e];
    }
    __device__ __forceinline__ float4 get4(int e) const {   // e a multiple of 4
        const float4 va = *reinterpret_cast<const float4*>(a + e);
        if (!b) return va;
        const float4 vb = *reinterpret_cast<const float4*>(b + e);
        const float s = base[e >> 8];
        return make_float4(fmaxf(0.f, (va.x + vb.x) + s), fmaxf(0.f, (va.y + vb.y) + s), fmaxf(0.f, (va.z + vb.z) + s),
                           fmaxf(0.f, (va.w + vb.w) + s));
    }
};
// Entry e of the tables of G pairs that visit the same list (a unit of the shared scans): with split tables the
// list's term is loaded once for all of them.  Same expression, hence the same bits, as PairTable::get.
template <int G>
__device__ __forceinline__ void unit_table_entries(const PairTable (&pt)[G], int e, float (&v)[G]) {
    if (pt[0].b) {
        const float ae = pt[0].a[e];
#pragma unroll
        for (int x = 0; x < G; ++x) v[x] = fmaxf(0.f, (ae + pt[x].b[e]) + pt[x].base[e >> 8]);
    } else {
#pragma unroll
        for (int x = 0; x < G; ++x) v[x] = pt[x].a[e];
    }
}

struct TableSrc {
    const float* lut = nullptr;        // [pairs][m][256], or in split mode [queries][m][256]
    const float* list_term = nullptr;  // split mode: [c][m][256]
    const float* pbase = nullptr;      // split mode: [pairs][m]
    const int32_t* probe = nullptr;    // split mode: list of every pair
    int w = 1, table_words = 0;        // pairs per query; m * 256
    int m = 0;
    __device__ __forceinline__ PairTable pair(int64_t pid) const {
        PairTable t;
        if (list_term) {
            t.a = list_term + (int64_t)probe[pid] * table_words;
            t.b = lut + (pid / w) * table_words;
            t.base = pbase + pid * m;
        } else {
            t.a = lut + pid * table_words;
            t.b = nullptr;
            t.base = nullptr;
        }
        return t;
    }
    // the same tables seen from a query's pair range [first, first + n): for launches over a slice of the batch
    TableSrc slice(int64_t first_pair) const {
        TableSrc s = *this;
        if (list_term) {
            s.lut = lut + (first_pair / w) * table_words;
            s.pbase = pbase + first_pair * m;
            s.probe = probe + first_pair;
        } else {
            s.lut = lut + first_pair * table_words;
        }
        return s;
    }
};

// Search plan, look-up tables, sample and list scan (scan.hip)
struct PlanBuffers {
    uint32_t* pair_start;  // [P] first padded entry of the pair's list
    uint32_t* len;         // [P] entries of the pair's list
    uint32_t* len_s;       // [P] leading entries of the pair's list that belong to the sample
    uint32_t* blkpre;      // [P+1] exclusive prefix of scan blocks over the pairs
    uint32_t* blkpre_s;    // [P+1] exclusive prefix of the sample's chunks (IVFR_SAMPLE_CHUNK entries) over the pairs
    uint32_t* items_s;     // [blkpre_s[P]] pair of every sample chunk
    uint32_t* soff;        // [P] first record of the pair's sample inside the query's candidate buffer; for a query that
                           //     keeps everything (no sample) the place of the pair's first entry in that buffer
    uint32_t* qblk;        // [nq] scan blocks of the query, then (after the plan's scan) its first block
    uint32_t* qblk_s;      // [nq] same for the sample
    uint32_t* nsample;     // [nq] sampled entries of the query
    uint32_t* capq;        // [nq] records in the query's candidate buffer
    uint32_t* cnt;         // [nq] record counters of the scan (zero on entry; preset for queries that keep everything)
    int place;             // 1 = the scans place the records of such queries by position (DirectPlace); 0 = they count them
    unsigned long long* coff;    // [nq] first record of the query's candidate buffer in the pool
    unsigned long long* sq;      // [nq] entries in the query's visited lists
    unsigned long long* su;      // [nq] entries in the nearest visited lists, which the query's sample is drawn from
    uint8_t* fully;              // [nq] 1 = few enough entries to keep them all (no sample, tau = +inf)
    uint8_t* exact_only;         // [nq] 1 = too large a share of the estimates will pass the bound for fp16 units
    unsigned long long* totals;  // [2]: [0] = sum of sq, [1] = records in the candidate pool
    DevStatus* status;           // the batch's status words (totals points into it)
    unsigned long long pool_cap; // records the candidate pool holds; a plan that wants more voids the batch
};
// pb.totals must be zero on entry.
int ivfr_launch_plan(const ivfr_index* ix, const int32_t* probe, int nq, int w, uint32_t full_limit,
                     uint32_t stride_k, uint32_t min_cap, uint32_t max_sample, int kprime, float half_frac,
                     const PlanBuffers& pb, hipStream_t st);
int ivfr_launch_lut(const ivfr_index* ix, const float* queries, const int32_t* probe, int nq, int w,
                    float* lut, float* lut_scale, hipStream_t st);
// Split tables.  list terms [c][m][256] = ||p_jk||^2 + 2 c_l^j . p_jk (once per index); per batch the query terms
// [nq][m][256] = -2 x^j . p_jk and, per pair, pbase [P][m] = ||(x - c_l)^j||^2 with the fp16 scale of the pair's table.
int ivfr_launch_list_terms(const ivfr_index* ix, float* list_term, hipStream_t st);
int ivfr_launch_query_terms(const ivfr_index* ix, const float* queries, const int32_t* probe, int nq, int w,
                            float* qterm, float* pbase, float* lut_scale, hipStream_t st);
// Geometry of a list-scan launch.  The number of units (pairs, or units of several pairs) is either known on
// the host or read by the kernel from a device word; the kernel spreads the launch's blocks over
// min(groups, max(g_min, blocks / bpg)) workgroups (a multiple of eight: one contiguous share of the block
// stream per XCD) and the remaining workgroups exit at once, so the host can launch from an estimate.
struct ScanShape {
    int n_host = 0;                  // units when n_dev is null
    const uint32_t* n_dev = nullptr; // device word with the number of units
    int groups = 8;                  // workgroups launched
    uint32_t bpg = 0;                // blocks of IVFR_BLOCK entries wanted per workgroup; 0 = use every launched workgroup
    uint32_t g_min = 8;
};
// unit_pairs == nullptr: unit u of the launch is pair u; otherwise pair unit_pairs[u].  An entry is kept
// when its estimate is <= tau[q]; with tau_id, when its key (estimate, id) is <= (tau[q], tau_id[q]).
// blkpre may be a slice of a longer prefix array: the launch's blocks are blkpre[0] .. blkpre[units].
// Queries that keep every estimate need no counter: entry e of pair p is record off[p] + e of the query's buffer
// (the plan presets the query's counter to its number of visited entries).  fully == nullptr: nobody is placed so.
struct DirectPlace {
    const uint8_t* fully = nullptr;   // [nq]
    const uint32_t* off = nullptr;    // [P]
};
int ivfr_launch_scan(const ivfr_index* ix, const TableSrc& ts, const uint32_t* pair_start, const uint32_t* pair_len,
                     const uint32_t* blkpre, const uint32_t* unit_pairs, ScanShape shape, int w, const float* tau,
                     uint2* cand, uint32_t* cand_cnt, CandLayout lay, hipStream_t st,
                     const uint32_t* tau_id = nullptr, DirectPlace direct = DirectPlace());

// Sample pass: the estimate of entry e < len_s[p] of pair p is written as a bare float at index soff[p] + e of
// the query's buffer (no counters involved; only the values are needed to bound the k'-th smallest).  One wavefront per chunk of IVFR_SAMPLE_CHUNK entries; items[i] is the
// pair of chunk i, chunk_pre the pairs' chunk prefix.
// n_items: device word with the number of chunks; max_items: a host-side upper bound (sizes the grid, whose
// wavefronts walk over the chunks).
int ivfr_launch_sample_scan(const ivfr_index* ix, const TableSrc& ts, const uint32_t* pair_start, const uint32_t* len_s,
                            const uint32_t* chunk_pre, const uint32_t* items, const uint32_t* n_items, size_t max_items,
                            const uint32_t* soff, int w, uint2* cand, CandLayout lay, hipStream_t st);

// Shared scan: pairs of one batch grouped by list into units of eight, four, two and single pairs
struct GroupBuffers {
    uint32_t* list_np;      // [2c] pairs visiting each list, by class (0 = filtered query, 1 = keeps everything)
    uint32_t* gpre;         // [5][c] exclusive prefixes of units of eight / four / two / single pairs / units of 64
    uint32_t* cur;          // [2c] fill cursors
    uint32_t* counts;       // [5] units of eight, four, two, single pairs, units of 64
    uint32_t* unit8_pairs;  // pair ids, eight per unit (0xFFFFFFFF = empty slot); unit4_pairs follows contiguously
    uint32_t* unit4_pairs;  // pair ids, four per unit
    size_t unit_bytes;      // bytes of unit8_pairs + unit4_pairs (cleared to empty before every fill)
    uint32_t* unit2_pairs;  // [2c] pair ids, two per unit
    uint32_t* lo_pairs;     // [c] single pair ids
    uint32_t* blk8;         // block prefix over units of eight
    uint32_t* blk4;         // ... of four
    uint32_t* blk2;         // ... of two
    uint32_t* blklo;        // ... over single pairs
    uint32_t* unit64_pairs; // pair ids, 64 per unit (always full)
    uint32_t* blk64;        // block prefix over units of 64
    unsigned long long* work;  // [6] list entries streamed; estimates computed by units of eight, four, two, singles, 64
};
// On entry gb.list_np and gb.work must be zero and the unit8 / unit4 arrays filled with IVFR_NO_PAIR.
int ivfr_launch_group_plan(const int32_t* probe, int P, int w, int c, const uint8_t* exact_only, bool use8, bool use64,
                           const uint32_t* pair_len, const GroupBuffers& gb, hipStream_t st);
// With lut_scale and exact_only (per query: 1 = keep to fp32), units of four whose queries all allow it run on
// half-precision tables with an exact re-evaluation, like the units of eight.
bool ivfr_shared_scan_supported(const ivfr_index* ix);
bool ivfr_shared8h_supported(const ivfr_index* ix);
int ivfr_launch_scan_shared(const ivfr_index* ix, int G, const TableSrc& ts, const uint32_t* pair_start,
                            const uint32_t* pair_len, const uint32_t* blkpre, const uint32_t* unit_pairs,
                            ScanShape shape, int w, const float* tau, uint2* cand, uint32_t* cand_cnt, CandLayout lay,
                            hipStream_t st, const float* lut_scale = nullptr, const uint8_t* exact_only = nullptr,
                            DirectPlace direct = DirectPlace());
int ivfr_launch_scan_shared8h(const ivfr_index* ix, const TableSrc& ts, const float* lut_scale,
                              const uint32_t* pair_start, const uint32_t* pair_len, const uint32_t* blkpre,
                              const uint32_t* unit_pairs, ScanShape shape, int w, const float* tau, uint2* cand,
                              uint32_t* cand_cnt, CandLayout lay, hipStream_t st);
// Units of 64 queries on the matrix cores (fp16 decode x query contraction as the filter, exact fp32 sums for
// what passes).  queries: the batch's [nq][d] floats; probe: the list of every pair.
bool ivfr_mfma_scan_supported(const ivfr_index* ix);
int ivfr_launch_scan_mfma64(const ivfr_index* ix, const float* queries, const int32_t* probe, const TableSrc& ts,
                            const float* lut_scale, const uint32_t* pair_start, const uint32_t* pair_len,
                            const uint32_t* blkpre, const uint32_t* unit_pairs, ScanShape shape, int w, const float* tau,
                            uint2* cand, uint32_t* cand_cnt, CandLayout lay, hipStream_t st);
// One-time function attributes (dynamic LDS beyond 48 KB) of every kernel of a translation unit, for the current device.
int ivfr_scan_init();
int ivfr_rerank_init();

// Encoding (encode.hip)
int ivfr_launch_residual(float* X, int64_t n, int d, const float* C, const int32_t* assign, hipStream_t st);
int ivfr_launch_pq_encode(float* R, int64_t n, int d, const float* book, int parts, uint8_t* codes,
                          bool subtract, hipStream_t st);
