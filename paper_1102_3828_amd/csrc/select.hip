// Segmented exact top-K selection by 64-bit key, one workgroup per segment (gfx950).
//
// Serves the three selections of the query stage: the w nearest coarse centroids
// (section 3.3), the k' smallest ADC estimates that form the short-list (step 1 of section
// 3.2) and the k smallest refined distances (step 3).  A key is (distance bits << 32) | index:
// non-negative IEEE floats order like their bit patterns, and the index in the low half makes
// every key distinct, so "the K smallest keys" is the K smallest distances with ties broken
// towards the lowest index, exactly.
//
// Method: most-significant-digit radix select, 8 passes of 8 bits.  Each pass histograms the
// digit of the keys that still match the prefix found so far (LDS atomics), a workgroup scan
// finds the digit bucket that holds the K-th smallest, and the prefix grows by one byte.
// After 8 passes the prefix is the K-th smallest key itself (the pivot); a last sweep emits
// every key <= pivot.  (As soon as few keys still match the prefix they are sorted in LDS
// instead, which ends the passes early.)  For short-list records the low half (the vector id) is fetched from
// the id array only in passes 4-7 and only for records whose estimate equals the pivot's.
#include "ivfr_internal.h"

#include <algorithm>

#define SEL_T 512
#define SEL_LCAP 2048
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

__device__ __forceinline__ uint32_t seg_hi(const SegView& s, int64_t i, uint32_t* pos) {
    if (s.vals) {
        *pos = (uint32_t)i;
        return s.vals[s.base + i];
    }
    if (s.keys) {
        uint64_t k = s.keys[s.base + i];
        *pos = (uint32_t)k;
        return (uint32_t)(k >> 32);
    }
    uint2 r = s.recs[s.base + i];
    *pos = r.y;
    return r.x;
}

__device__ __forceinline__ uint32_t seg_lo(const SegView& s, uint32_t pos) {
    return (s.keys || s.vals) ? pos : (uint32_t)s.ids[(size_t)pos * s.id_stride];
}

// Returns the K-th smallest key of the segment (1 <= K <= n).  All threads must call.
// Radix passes run only while more than SEL_LCAP keys still match the prefix; the remaining
// candidates are then gathered into LDS, sorted there, and the pivot is read off directly.
__device__ uint64_t radix_pivot(const SegView& s, uint32_t K) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wsum[SEL_T / 64];
    __shared__ uint32_t s_bin, s_need, s_match, s_fill;
    __shared__ uint64_t lbuf[SEL_LCAP];
    const int tid = threadIdx.x;
    uint64_t prefix = 0;
    uint32_t need = K;
    uint64_t nmatch = (uint64_t)s.n;
    if (K <= SEL_T / 2 && s.n > SEL_LCAP) {
        // Small K: every thread takes the minimum distance word of its strided share; the K-th
        // smallest of those SEL_T minima bounds the K-th smallest key from above, and at least K
        // keys lie at or below it.  Those few keys are gathered and sorted in LDS: two sweeps.
        uint32_t mn = 0xFFFFFFFFu;
        for (int64_t i = tid; i < s.n; i += SEL_T) {
            uint32_t pos;
            uint32_t hi = seg_hi(s, i, &pos);
            mn = hi < mn ? hi : mn;
        }
        lbuf[tid] = mn;
        __syncthreads();
        for (uint32_t k = 2; k <= SEL_T; k <<= 1)
            for (uint32_t j = k >> 1; j > 0; j >>= 1) {
                uint32_t i = tid, ixj = i ^ j;
                if (ixj > i) {
                    uint64_t a = lbuf[i], b = lbuf[ixj];
                    bool asc = (i & k) == 0;
                    if ((a > b) == asc) { lbuf[i] = b; lbuf[ixj] = a; }
                }
                __syncthreads();
            }
        const uint32_t bound = (uint32_t)lbuf[K - 1];
        __syncthreads();
        if (tid == 0) s_fill = 0;
        __syncthreads();
        for (int64_t i = tid; i < s.n; i += SEL_T) {
            uint32_t pos;
            uint32_t hi = seg_hi(s, i, &pos);
            if (hi <= bound) {
                uint32_t slot = atomicAdd(&s_fill, 1u);
                if (slot < SEL_LCAP) lbuf[slot] = ((uint64_t)hi << 32) | seg_lo(s, pos);
            }
        }
        __syncthreads();
        const uint32_t got = s_fill;
        __syncthreads();
        if (got <= SEL_LCAP) {
            uint32_t n2 = 2;
            while (n2 < got) n2 <<= 1;
            for (uint32_t i = got + tid; i < n2; i += SEL_T) lbuf[i] = ~0ull;
            __syncthreads();
            for (uint32_t k = 2; k <= n2; k <<= 1)
                for (uint32_t j = k >> 1; j > 0; j >>= 1) {
                    for (uint32_t i = tid; i < n2; i += SEL_T) {
                        uint32_t ixj = i ^ j;
                        if (ixj > i) {
                            uint64_t a = lbuf[i], b = lbuf[ixj];
                            bool asc = (i & k) == 0;
                            if ((a > b) == asc) { lbuf[i] = b; lbuf[ixj] = a; }
                        }
                    }
                    __syncthreads();
                }
            const uint64_t pivot = lbuf[K - 1];
            __syncthreads();
            return pivot;
        }
        // too many equal distance words: fall through to the radix passes
    }
    int pass = 0;
    for (; pass < 8 && nmatch > SEL_LCAP; ++pass) {
        const int shift = 56 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const uint32_t pre_hi = (pass >= 4) ? (uint32_t)(prefix >> (8 * (pass - 4))) : 0u;
        for (int64_t i = tid; i < s.n; i += SEL_T) {
            uint32_t pos;
            uint32_t hi = seg_hi(s, i, &pos);
            if (pass < 4) {
                uint64_t key = (uint64_t)hi << 32;
                if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1u);
            } else if (hi == pre_hi) {
                uint64_t key = ((uint64_t)hi << 32) | seg_lo(s, pos);
                if ((key >> (shift + 8)) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1u);
            }
        }
        __syncthreads();
        // inclusive scan of the 256 buckets by the first 256 threads
        uint32_t h = 0, inc = 0;
        if (tid < 256) {
            h = hist[tid];
            inc = h;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                uint32_t o = __shfl_up(inc, off, 64);
                if ((tid & 63) >= off) inc += o;
            }
            if ((tid & 63) == 63) wsum[tid >> 6] = inc;
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t add = 0;
            for (int wv = 0; wv < (tid >> 6); ++wv) add += wsum[wv];
            inc += add;
            uint32_t exc = inc - h;
            if (exc < need && need <= inc) { s_bin = (uint32_t)tid; s_need = need - exc; s_match = h; }
        }
        __syncthreads();
        prefix = (prefix << 8) | s_bin;
        need = s_need;
        nmatch = s_match;
        __syncthreads();
    }
    if (pass == 8) return prefix;
    // gather the keys whose top `pass` bytes equal the prefix
    if (tid == 0) s_fill = 0;
    __syncthreads();
    for (int64_t i = tid; i < s.n; i += SEL_T) {
        uint32_t pos;
        uint32_t hi = seg_hi(s, i, &pos);
        bool match;
        if (pass == 0) match = true;
        else if (pass <= 4) match = (hi >> (32 - 8 * pass)) == (uint32_t)prefix;
        else match = hi == (uint32_t)(prefix >> (8 * (pass - 4)));
        if (match) {
            uint64_t key = ((uint64_t)hi << 32) | seg_lo(s, pos);
            if (pass > 4 && (key >> (64 - 8 * pass)) != prefix) continue;
            uint32_t slot = atomicAdd(&s_fill, 1u);
            if (slot < SEL_LCAP) lbuf[slot] = key;
        }
    }
    __syncthreads();
    const uint32_t mcount = s_fill < SEL_LCAP ? s_fill : SEL_LCAP;
    uint32_t n2 = 2;
    while (n2 < mcount) n2 <<= 1;
    for (uint32_t i = mcount + tid; i < n2; i += SEL_T) lbuf[i] = ~0ull;
    __syncthreads();
    for (uint32_t k = 2; k <= n2; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = tid; i < n2; i += SEL_T) {
                uint32_t ixj = i ^ j;
                if (ixj > i) {
                    uint64_t a = lbuf[i], b = lbuf[ixj];
                    bool asc = (i & k) == 0;
                    if ((a > b) == asc) { lbuf[i] = b; lbuf[ixj] = a; }
                }
            }
            __syncthreads();
        }
    }
    const uint64_t pivot = lbuf[need - 1];
    __syncthreads();
    return pivot;
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
        uint64_t pivot = radix_pivot(s, (uint32_t)r);   // ends with a barrier: its LDS state is free for the next segment
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
    const uint64_t pivot = radix_pivot(s, (uint32_t)K);
    const uint32_t p_hi = (uint32_t)(pivot >> 32), p_lo = (uint32_t)pivot;
    for (int64_t i = threadIdx.x; i < n; i += SEL_T) {
        uint2 r = recs[s.base + i];
        bool take = r.x < p_hi || (r.x == p_hi && (uint32_t)ids[(size_t)r.y * id_stride] <= p_lo);
        if (take) {
            uint32_t slot = atomicAdd(&s_slot, 1u);
            if (slot < (uint32_t)K) { op[slot] = r.y; oe[slot] = __uint_as_float(r.x); }
        }
    }
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
        const uint64_t pivot = radix_pivot(s, (uint32_t)K);
        for (int64_t i = threadIdx.x; i < n; i += SEL_T) {
            uint64_t k = keys[s.base + i];
            if (k <= pivot) {
                uint32_t slot = atomicAdd(&s_slot, 1u);
                if (slot < (uint32_t)n2) sk[slot] = k;
            }
        }
        m_out = K;
    }
    __syncthreads();
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
