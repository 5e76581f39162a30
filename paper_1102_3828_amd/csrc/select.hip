// Segmented exact top-K selection by 64-bit key, one workgroup per segment (gfx950).
//
// Serves the three selections of the query stage: the w nearest coarse centroids
// (section 3.3), the k' smallest ADC estimates that form the short-list (step 1 of section
// 3.2) and the k smallest refined distances (step 3).  A key is (distance bits << 32) | index:
// non-negative IEEE floats order like their bit patterns, and the index in the low half makes
// every key distinct, so "the K smallest keys" is the K smallest distances with ties broken
// towards the lowest index, exactly.
//
// Method: the K-th smallest key (the pivot) is found by narrowing a range of distance words.  One sweep takes the
// minimum and maximum word of the segment; each further sweep histograms the words inside the current range
// into up to 1024 equal power-of-two bins (LDS atomics), a workgroup scan finds the bin that holds the K-th
// smallest, and the range shrinks to that bin.  Starting at the minimum and maximum skips the leading bits that
// all estimates of a query share, so one histogram sweep usually leaves a handful of keys; at most four are ever
// needed for 32 bits.  The few keys left in the range are gathered into LDS with their index words and ranked by
// counting.  Only if more than 512 keys share one distance word does the same narrowing go on over their index
// words.  A last sweep by the caller emits every key <= pivot.  For short-list records the index word (the
// vector id) is fetched from the record array only for the gathered keys.  When few keys are wanted out of many
// (K <= 256 of more than 4096: the bound from the sample, the visited lists, the final top-k) the range comes from
// one sweep instead of two: the K-th smallest of the 512 per-thread minima is an upper bound with few keys below it.
#include "ivfr_internal.h"

#include <algorithm>

#define SEL_T 512
#define SEL_BINS (2 * SEL_T)
#define SEL_RC 512        // keys ranked by counting
#define SEL_RANK_SORT 256 // results sorted by counting rather than by a bitonic network
#define SORT_MAX 16384

struct SegView {
    const uint64_t* keys;   // source A (nullptr for records)
    const uint2* recs;      // source B
    const int32_t* ids;
    int64_t base;
    int64_t n;
    const uint32_t* vals = nullptr;   // source C: bare distance words; the element index is the low half of the key
    uint32_t id_stride = 1;           // ids[pos * id_stride] is the id of the entry at position pos
};

enum { SRC_VALS = 0, SRC_KEYS = 1, SRC_RECS = 2 };   // which of the three sources a segment uses (compile-time in the kernels)

template <int SRC>
__device__ __forceinline__ uint32_t seg_lo(const SegView& s, uint32_t pos) {
    return SRC != SRC_RECS ? pos : (uint32_t)s.ids[(size_t)pos * s.id_stride];
}

// One sweep of the workgroup over the segment: body(distance word, pos) for every element, thread tid taking
// elements tid, tid + SEL_T, ...  Four loads are issued before the first is used (a sweep is a chain of load
// latencies otherwise: a segment of 50000 sampled estimates is 98 elements per thread).
template <int SRC, class B>
__device__ __forceinline__ void sweep(const SegView& s, B body) {
    const int64_t n = s.n;
    int64_t i = threadIdx.x;
    if (SRC == SRC_VALS) {
        const uint32_t* v = s.vals + s.base;
        for (; i + 3 * SEL_T < n; i += 4 * SEL_T) {
            const uint32_t a = v[i], b = v[i + SEL_T], c = v[i + 2 * SEL_T], d = v[i + 3 * SEL_T];
            body(a, (uint32_t)i); body(b, (uint32_t)(i + SEL_T)); body(c, (uint32_t)(i + 2 * SEL_T)); body(d, (uint32_t)(i + 3 * SEL_T));
        }
        for (; i < n; i += SEL_T) body(v[i], (uint32_t)i);
    } else if (SRC == SRC_KEYS) {
        const uint64_t* v = s.keys + s.base;
        for (; i + 3 * SEL_T < n; i += 4 * SEL_T) {
            const uint64_t a = v[i], b = v[i + SEL_T], c = v[i + 2 * SEL_T], d = v[i + 3 * SEL_T];
            body((uint32_t)(a >> 32), (uint32_t)a); body((uint32_t)(b >> 32), (uint32_t)b);
            body((uint32_t)(c >> 32), (uint32_t)c); body((uint32_t)(d >> 32), (uint32_t)d);
        }
        for (; i < n; i += SEL_T) { const uint64_t a = v[i]; body((uint32_t)(a >> 32), (uint32_t)a); }
    } else {
        const uint2* v = s.recs + s.base;
        for (; i + 3 * SEL_T < n; i += 4 * SEL_T) {
            const uint2 a = v[i], b = v[i + SEL_T], c = v[i + 2 * SEL_T], d = v[i + 3 * SEL_T];
            body(a.x, a.y); body(b.x, b.y); body(c.x, c.y); body(d.x, d.y);
        }
        for (; i < n; i += SEL_T) { const uint2 a = v[i]; body(a.x, a.y); }
    }
}

struct SelShared {
    uint32_t hist[SEL_BINS];
    uint64_t cand[SEL_RC];
    uint32_t wa[SEL_T / 64], wb[SEL_T / 64];
    uint32_t bin, need, cnt, fill;
    uint64_t pivot;
};

// Narrows [lo, hi] around the need-th smallest of the words that word(f) feeds to f (one call sweeps this thread's
// share of them), until at most `stop` words are left in the range or the range is a single value.  count is the
// number of words on entry and in the final range on return; need becomes the rank inside the final range.  All
// threads call.
template <class F>
__device__ void narrow_range(SelShared& sh, F word, uint32_t& lo, uint32_t& hi, uint32_t& need,
                             uint64_t& count, uint32_t stop = SEL_RC) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    uint32_t mn = 0xFFFFFFFFu, mx = 0u;
    word([&](uint32_t v) { mn = v < mn ? v : mn; mx = v > mx ? v : mx; });
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t a = __shfl_xor(mn, off, 64), b = __shfl_xor(mx, off, 64);
        mn = a < mn ? a : mn;
        mx = b > mx ? b : mx;
    }
    if (lane == 0) { sh.wa[wv] = mn; sh.wb[wv] = mx; }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < SEL_T / 64; ++i) {
        mn = sh.wa[i] < mn ? sh.wa[i] : mn;
        mx = sh.wb[i] > mx ? sh.wb[i] : mx;
    }
    __syncthreads();   // wa is used again below
    lo = mn;
    hi = mx;
    // each pass leaves a span below 2^shift <= span / 512: four passes reach a single value from any 32-bit span
    for (int pass = 0; pass < 4 && count > stop && hi > lo; ++pass) {
        const uint32_t span = hi - lo;
        int shift = 0;
        while ((span >> shift) >= SEL_BINS) ++shift;
        for (int i = tid; i < SEL_BINS; i += SEL_T) sh.hist[i] = 0;
        __syncthreads();
        word([&](uint32_t v) {
            if (v >= lo && v <= hi) atomicAdd(&sh.hist[(v - lo) >> shift], 1u);
        });
        __syncthreads();
        // two bins per thread; inclusive scan over the workgroup
        const uint32_t a = sh.hist[2 * tid], b = sh.hist[2 * tid + 1];
        uint32_t inc = a + b;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(inc, off, 64);
            if (lane >= off) inc += o;
        }
        if (lane == 63) sh.wa[wv] = inc;
        __syncthreads();
        uint32_t exc = inc - (a + b);
        for (int i = 0; i < wv; ++i) exc += sh.wa[i];
        if (exc < need && need <= exc + a) {
            sh.bin = 2u * tid; sh.need = need - exc; sh.cnt = a;
        } else if (exc + a < need && need <= exc + a + b) {
            sh.bin = 2u * tid + 1u; sh.need = need - exc - a; sh.cnt = b;
        }
        __syncthreads();
        const uint32_t nlo = lo + (sh.bin << shift);
        const uint64_t nhi = (uint64_t)nlo + ((1ull << shift) - 1ull);
        hi = nhi < (uint64_t)hi ? (uint32_t)nhi : hi;
        lo = nlo;
        need = sh.need;
        count = sh.cnt;
        __syncthreads();
    }
}

// Returns the K-th smallest key of the segment (1 <= K <= n).  All threads must call; ends with a barrier.
template <int SRC>
__device__ uint64_t kth_key(const SegView& s, uint32_t K) {
    __shared__ SelShared sh;
    const int tid = threadIdx.x;
    // keys with distance word in [lo, hi] (and, with by_index, index word in [lo2, hi2]) go to LDS; returns how many
    // there were (only the first SEL_RC are kept)
    auto gather = [&](uint32_t lo, uint32_t hi, bool by_index, uint32_t lo2, uint32_t hi2) -> uint32_t {
        if (tid == 0) sh.fill = 0;
        __syncthreads();
        sweep<SRC>(s, [&](uint32_t h, uint32_t pos) {
            if (h < lo || h > hi) return;
            const uint32_t l = seg_lo<SRC>(s, pos);
            if (by_index && (l < lo2 || l > hi2)) return;
            const uint32_t slot = atomicAdd(&sh.fill, 1u);
            if (slot < SEL_RC) sh.cand[slot] = ((uint64_t)h << 32) | l;
        });
        __syncthreads();
        const uint32_t got = sh.fill;
        __syncthreads();
        return got;
    };
    // the need-th smallest of the got <= SEL_RC gathered keys, by counting: the key with fewer than `need` keys below
    // it and at least `need` at or below it (equal keys agree)
    auto ranked = [&](uint32_t got, uint32_t need) -> uint64_t {
        if ((uint32_t)tid < got) {
            const uint64_t key = sh.cand[tid];
            uint32_t lt = 0, le = 0;
            for (uint32_t j = 0; j < got; ++j) {
                const uint64_t kj = sh.cand[j];
                lt += kj < key ? 1u : 0u;
                le += kj <= key ? 1u : 0u;
            }
            if (lt < need && need <= le) sh.pivot = key;
        }
        __syncthreads();
        const uint64_t pivot = sh.pivot;
        __syncthreads();
        return pivot;
    };
    if (K <= SEL_T / 2 && s.n > 8 * SEL_T) {
        // Few of many: every thread takes the minimum distance word of its strided share; the K-th smallest of those
        // SEL_T minima bounds the K-th smallest key from above, and at least K keys (a few more as a rule) lie at or
        // below it.  One sweep for the minima, one to gather those keys; the bound itself is found by narrowing over
        // the minima in LDS.
        uint32_t* mins = reinterpret_cast<uint32_t*>(sh.cand);
        uint32_t mn = 0xFFFFFFFFu;
        sweep<SRC>(s, [&](uint32_t h, uint32_t) { mn = h < mn ? h : mn; });
        mins[tid] = mn;
        __syncthreads();
        auto min_words = [&](auto f) { f(mins[tid]); };   // one minimum per thread
        uint32_t mlo = 0u, bound = 0xFFFFFFFFu, mneed = K;
        uint64_t mcount = SEL_T;
        narrow_range(sh, min_words, mlo, bound, mneed, mcount, 1u);   // ends with a barrier: mins may be overwritten
        const uint32_t got = gather(0u, bound, false, 0u, 0u);
        if (got <= SEL_RC) return ranked(got, K);
        // a crowd of equal distance words at the bound: the general way
    }
    uint32_t need = K;
    uint64_t count = (uint64_t)s.n;
    uint32_t lo = 0u, hi = 0xFFFFFFFFu, lo2 = 0u, hi2 = 0xFFFFFFFFu;
    bool by_index = false;
    if (count > SEL_RC) {
        auto dist_words = [&](auto f) { sweep<SRC>(s, [&](uint32_t h, uint32_t) { f(h); }); };
        narrow_range(sh, dist_words, lo, hi, need, count);
        if (count > SEL_RC) {   // lo == hi: that many keys share the distance word, their index words decide
            by_index = true;
            const uint32_t fixed = lo;
            auto index_words = [&](auto f) {
                sweep<SRC>(s, [&](uint32_t h, uint32_t pos) { if (h == fixed) f(seg_lo<SRC>(s, pos)); });
            };
            narrow_range(sh, index_words, lo2, hi2, need, count);
            if (count > SEL_RC) return ((uint64_t)fixed << 32) | lo2;   // equal keys throughout
        }
    }
    uint32_t got = gather(lo, hi, by_index, lo2, hi2);
    got = got < SEL_RC ? got : SEL_RC;
    return ranked(got, need);
}

__device__ __forceinline__ int64_t seg_count(const uint32_t* counts, uint32_t cap, int seg, bool* over) {
    *over = false;
    uint32_t c = counts[seg];
    if (c > cap) { *over = true; return cap; }
    return c;
}

// ---- bound from a uniform sample --------------------------------------------------------------
// The sample holds n of the query's sq visited entries, so about mu = k' n / sq of the true k'
// best are in it (Poisson-like).  Taking the r-th smallest sampled estimate with r = mu + 5
// sqrt(mu) + 6 makes it all but certain (beyond five standard deviations) that at least k'
// visited entries lie at or below it; the filtered scan verifies that by counting.
// WALK: few workgroups walk over the segments (for batches in which hardly any query has a sample: launching a
// workgroup per query only to find its skip flag set costs more than the whole selection); otherwise one
// workgroup per segment.
template <bool WALK>
__global__ __launch_bounds__(SEL_T) void select_tau_kernel(const uint2* recs, const int32_t* ids, uint32_t id_stride,
                                                           CandLayout lay, const uint32_t* counts,
                                                           const unsigned long long* sq, int kprime,
                                                           int fixed_rank, const uint8_t* skip, float* tau,
                                                           uint32_t* tau_id, int values_only, int nseg) {
    // seg is uniform over the workgroup, so every barrier is reached by all its threads
    for (int seg = blockIdx.x; seg < nseg; seg += WALK ? (int)gridDim.x : nseg) {
        if (skip && skip[seg]) continue;
        bool over;
        int64_t n = seg_count(counts, values_only ? 0xFFFFFFFFu : lay.cap(seg), seg, &over);
        const double mu = (double)kprime * (double)n / (double)(sq[seg] ? sq[seg] : 1ull);
        // fixed_rank > 0: the records are a subset of the visited entries and their fixed_rank-th smallest is wanted
        const int64_t r = fixed_rank > 0 ? (int64_t)fixed_rank : (int64_t)ceil(mu + 5.0 * sqrt(mu) + 6.0);
        if (n < r || n == 0) {
            if (threadIdx.x == 0) {
                tau[seg] = INFINITY;
                if (tau_id) tau_id[seg] = 0xFFFFFFFFu;
            }
            continue;
        }
        SegView s{nullptr, recs, ids, (int64_t)lay.base(seg), n};
        s.id_stride = id_stride;
        if (values_only) {   // the segment holds n bare estimates (4 bytes each) at the start of its record buffer
            s.recs = nullptr;
            s.vals = reinterpret_cast<const uint32_t*>(recs);
            s.base = 2 * (int64_t)lay.base(seg);
        }
        // ends with a barrier: its LDS state is free for the next segment
        const uint64_t pivot = values_only ? kth_key<SRC_VALS>(s, (uint32_t)r) : kth_key<SRC_RECS>(s, (uint32_t)r);
        if (threadIdx.x == 0) {
            tau[seg] = __uint_as_float((uint32_t)(pivot >> 32));
            if (tau_id) tau_id[seg] = (uint32_t)pivot;
        }
    }
}

int ivfr_launch_select_tau(const SelectArgs& a, const unsigned long long* sq, int kprime, int fixed_rank,
                           const uint8_t* skip, float* tau, uint32_t* tau_id, hipStream_t st, bool values_only,
                           bool mostly_skipped) {
    if (a.nseg <= 0) return IVFR_OK;
    if (mostly_skipped)
        hipLaunchKernelGGL(select_tau_kernel<true>, dim3(std::min(a.nseg, 256)), dim3(SEL_T), 0, st, a.recs, a.ids,
                           a.id_stride, a.lay, a.counts, sq, kprime, fixed_rank, skip, tau, tau_id, values_only ? 1 : 0, a.nseg);
    else
        hipLaunchKernelGGL(select_tau_kernel<false>, dim3(a.nseg), dim3(SEL_T), 0, st, a.recs, a.ids, a.id_stride,
                           a.lay, a.counts, sq, kprime, fixed_rank, skip, tau, tau_id, values_only ? 1 : 0, a.nseg);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// ---- unordered compaction of the K smallest records -----------------------------------------
__global__ __launch_bounds__(SEL_T) void select_records_kernel(const uint2* recs, const int32_t* ids,
                                                               uint32_t id_stride,
                                                               CandLayout lay, const uint32_t* counts, int K,
                                                               int out_base,
                                                               const unsigned long long* sq, uint32_t* out_pos,
                                                               float* out_est, int32_t* out_n, int32_t* overflow,
                                                               int32_t* overflow_total) {
    __shared__ uint32_t s_slot;
    const int seg = blockIdx.x;
    const int q = out_base + seg;
    bool over;
    int64_t n = seg_count(counts, lay.cap(seg), seg, &over);
    // the filter was too tight if it kept fewer than k' although more entries were visited
    if (sq && n < K && (unsigned long long)n < sq[seg]) over = true;
    if (threadIdx.x == 0) {
        s_slot = 0;
        if (overflow) overflow[q] = over ? 1 : 0;
        if (over && overflow_total) atomicAdd(overflow_total, 1);
    }
    __syncthreads();
    if (over) {
        if (threadIdx.x == 0) out_n[q] = 0;
        return;
    }
    SegView s{nullptr, recs, ids, (int64_t)lay.base(seg), n};
    s.id_stride = id_stride;
    uint32_t* op = out_pos + (int64_t)q * K;
    float* oe = out_est + (int64_t)q * K;
    if (n <= K) {
        for (int64_t i = threadIdx.x; i < n; i += SEL_T) {
            uint2 r = recs[s.base + i];
            op[i] = r.y;
            oe[i] = __uint_as_float(r.x);
        }
        if (threadIdx.x == 0) out_n[q] = (int32_t)n;
        return;
    }
    const uint64_t pivot = kth_key<SRC_RECS>(s, (uint32_t)K);
    const uint32_t p_hi = (uint32_t)(pivot >> 32), p_lo = (uint32_t)pivot;
    sweep<SRC_RECS>(s, [&](uint32_t est, uint32_t pos) {
        const bool take = est < p_hi || (est == p_hi && (uint32_t)ids[(size_t)pos * id_stride] <= p_lo);
        if (take) {
            const uint32_t slot = atomicAdd(&s_slot, 1u);
            if (slot < (uint32_t)K) { op[slot] = pos; oe[slot] = __uint_as_float(est); }
        }
    });
    if (threadIdx.x == 0) out_n[q] = K;
}

int ivfr_launch_select_records(const SelectArgs& a, int out_base, const unsigned long long* sq, uint32_t* out_pos,
                               float* out_est, int32_t* out_n, int32_t* overflow, int32_t* overflow_total,
                               hipStream_t st) {
    if (a.nseg <= 0) return IVFR_OK;
    hipLaunchKernelGGL(select_records_kernel, dim3(a.nseg), dim3(SEL_T), 0, st, a.recs, a.ids, a.id_stride, a.lay, a.counts, a.K,
                       out_base, sq, out_pos, out_est, out_n, overflow, overflow_total);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// ---- sorted K smallest keys -----------------------------------------------------------------
// counts (optional) gives each segment's element count (int32, e.g. the short-list length).
__global__ __launch_bounds__(SEL_T) void select_sorted_kernel(const uint64_t* keys, int64_t seg_stride,
                                                              int64_t fixed_count, const int32_t* counts, int K,
                                                              int n2, int out_base, int32_t* out_lo, float* out_hi) {
    extern __shared__ uint64_t sk[];   // n2 keys
    __shared__ uint32_t s_slot;
    const int seg = blockIdx.x;
    const int q = out_base + seg;
    int64_t n = counts ? (int64_t)counts[q] : fixed_count;
    if (threadIdx.x == 0) s_slot = 0;
    for (int i = threadIdx.x; i < n2; i += SEL_T) sk[i] = ~0ull;
    __syncthreads();
    SegView s{keys, nullptr, nullptr, (int64_t)seg * seg_stride, n};
    int m_out;
    if (n <= K) {
        for (int64_t i = threadIdx.x; i < n; i += SEL_T) sk[i] = keys[s.base + i];
        m_out = (int)n;
    } else {
        const uint64_t pivot = kth_key<SRC_KEYS>(s, (uint32_t)K);
        sweep<SRC_KEYS>(s, [&](uint32_t h, uint32_t l) {
            const uint64_t k = ((uint64_t)h << 32) | l;
            if (k <= pivot) {
                const uint32_t slot = atomicAdd(&s_slot, 1u);
                if (slot < (uint32_t)n2) sk[slot] = k;
            }
        });
        m_out = K;
    }
    __syncthreads();
    if (n2 <= SEL_RANK_SORT) {
        // few results: every key counts the keys before it and goes straight to its place
        const int m_have = n <= K ? m_out : (int)(s_slot < (uint32_t)n2 ? s_slot : (uint32_t)n2);
        for (int i = threadIdx.x; i < m_have; i += SEL_T) {
            const uint64_t key = sk[i];
            int r = 0;
            for (int j = 0; j < m_have; ++j) {
                const uint64_t kj = sk[j];
                r += (kj < key || (kj == key && j < i)) ? 1 : 0;
            }
            if (r < m_out) {
                const int64_t o = (int64_t)q * K + r;
                out_lo[o] = (int32_t)(uint32_t)key;
                out_hi[o] = __uint_as_float((uint32_t)(key >> 32));
            }
        }
        for (int i = m_out + threadIdx.x; i < K; i += SEL_T) {
            const int64_t o = (int64_t)q * K + i;
            out_lo[o] = -1;
            out_hi[o] = INFINITY;
        }
        return;
    }
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < n2; i += SEL_T) {
                int ixj = i ^ j;
                if (ixj > i) {
                    uint64_t a = sk[i], b = sk[ixj];
                    bool asc = (i & k) == 0;
                    if ((a > b) == asc) { sk[i] = b; sk[ixj] = a; }
                }
            }
            __syncthreads();
        }
    }
    for (int i = threadIdx.x; i < K; i += SEL_T) {
        int64_t o = (int64_t)q * K + i;
        if (i < m_out) {
            uint64_t k = sk[i];
            out_lo[o] = (int32_t)(uint32_t)k;
            out_hi[o] = __uint_as_float((uint32_t)(k >> 32));
        } else {
            out_lo[o] = -1;
            out_hi[o] = INFINITY;
        }
    }
}

static int g_sort_max = 4096;   // keys that fit the default dynamic-LDS limit until the attribute is raised

int ivfr_select_init() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_sorted_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SORT_MAX * 8);
    if (e == hipSuccess) g_sort_max = SORT_MAX;
    else (void)hipGetLastError();
    return IVFR_OK;
}

int ivfr_launch_select_sorted(const SelectArgs& a, const int32_t* counts_i32, int out_base, int32_t* out_lo,
                              float* out_hi, hipStream_t st) {
    if (a.nseg <= 0) return IVFR_OK;
    if (a.K > g_sort_max) {
        ivfr_set_error("sorted selection supports at most %d results per query (got %d)", g_sort_max, a.K);
        return IVFR_ERR_INVALID_ARG;
    }
    int n2 = 2;
    while (n2 < a.K) n2 <<= 1;
    hipLaunchKernelGGL(select_sorted_kernel, dim3(a.nseg), dim3(SEL_T), (size_t)n2 * 8, st, a.keys, a.seg_stride,
                       a.fixed_count, counts_i32, a.K, n2, out_base, out_lo, out_hi);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}
