// Query step 1 of section 3.2 on the inverted file of section 3.3 (gfx950): plan of the
// visited (query, list) pairs, per-pair look-up tables of Eq. (5), and the ADC list scan.
#include "ivfr_internal.h"

#include <algorithm>

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ------------------------------------------------------------------------------------------
// Plan.  Pair p = q * w + r is the r-th nearest list of query q.  Per query the plan fixes how
// the k'-th smallest estimate is bounded before the scan:
//  - a query whose visited lists hold at most `full_limit` entries keeps every estimate
//    (tau = +inf) and is selected from directly;
//  - otherwise a sample is scored first: the first ceil(len / stride) entries of every visited
//    list; about mu = k' / stride of the true k' best fall in the sample (mu >= 4; a query
//    that visits very many entries gets a wider stride so its sample stays below max_sample).  Entries
//    of a list are in id order, which carries no information about the distance to a query,
//    so a prefix is as good as a random draw, and taking the same fraction of every visited
//    list keeps the sample stratified over near and far lists.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    return v;
}

// One wavefront per query: the lanes take the query's w pairs in turn.  Block counts are prefix-summed
// inside the query here (blkpre, blkpre_s hold query-relative values, qblk / qblk_s the query totals;
// blkpre counts scan blocks of IVFR_BLOCK entries, blkpre_s sample chunks of IVFR_SAMPLE_CHUNK entries);
// plan_scan_kernel turns them into batch-wide prefixes.
__global__ __launch_bounds__(256) void plan_pairs_kernel(const int32_t* __restrict__ probe, int nq, int w,
                                                         const uint32_t* __restrict__ list_start,
                                                         const uint32_t* __restrict__ list_len, uint32_t full_limit,
                                                         uint32_t stride_k, uint32_t min_cap, uint32_t max_sample,
                                                         int kprime, float half_frac, PlanBuffers pb) {
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.x * 4 + (threadIdx.x >> 6);   // uniform over the wavefront
    if (q >= nq) return;
    unsigned long long total = 0;
    for (int r = lane; r < w; r += 64) total += list_len[probe[(int64_t)q * w + r]];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) total += __shfl_xor(total, off, 64);
    // the sample comes from the nearest lists: those whose predecessors in probe order hold fewer than `thresh` entries
    const unsigned long long thresh = ivfr_sample_threshold(total, kprime);
    unsigned long long total_u = 0, before = 0;
    for (int r0 = 0; r0 < w; r0 += 64) {
        const int r = r0 + lane;
        const unsigned long long len = r < w ? (unsigned long long)list_len[probe[(int64_t)q * w + r]] : 0ull;
        unsigned long long inc = len;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned long long o = __shfl_up(inc, off, 64);
            if (lane >= off) inc += o;
        }
        if (before + inc - len < thresh) total_u += len;
        before += __shfl(inc, 63, 64);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) total_u += __shfl_xor(total_u, off, 64);
    const QueryPlan qp = ivfr_plan_query(total, total_u, full_limit, stride_k, max_sample, kprime);
    const bool fully = qp.fully;
    const uint32_t stride = qp.stride;
    unsigned long long sampled = 0;
    uint32_t carry = 0, carry_s = 0, carry_e = 0;
    before = 0;
    for (int r0 = 0; r0 < w; r0 += 64) {
        const int r = r0 + lane;
        uint32_t len = 0, ls = 0;
        {
            // the same walk as above: is this pair one of the sampled lists?
            const unsigned long long l64 = r < w ? (unsigned long long)list_len[probe[(int64_t)q * w + r]] : 0ull;
            unsigned long long inc = l64;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned long long o = __shfl_up(inc, off, 64);
                if (lane >= off) inc += o;
            }
            const bool in_u = before + inc - l64 < thresh;
            before += __shfl(inc, 63, 64);
            if (r < w) ls = (fully || !in_u) ? 0u : ((uint32_t)l64 + stride - 1) / stride;
        }
        if (r < w) {
            const int64_t p = (int64_t)q * w + r;
            const int l = probe[p];
            len = list_len[l];
            pb.pair_start[p] = list_start[l];
            pb.len[p] = len;
            pb.len_s[p] = ls;
        }
        const uint32_t nb = (len + IVFR_BLOCK - 1) / IVFR_BLOCK, nbs = (ls + IVFR_SAMPLE_CHUNK - 1) / IVFR_SAMPLE_CHUNK;
        const uint32_t inc = wave_incl_scan(nb, lane), inc_s = wave_incl_scan(nbs, lane);
        // entries before the pair in the query's buffer: of the sample (below 2^32: max_sample + w), or, for a
        // query that keeps everything, of the lists themselves (at most full_limit)
        const uint32_t le = fully ? len : ls;
        const uint32_t inc_e = wave_incl_scan(le, lane);
        if (r < w) {
            const int64_t p = (int64_t)q * w + r;
            pb.blkpre[p] = carry + inc - nb;
            pb.blkpre_s[p] = carry_s + inc_s - nbs;
            pb.soff[p] = carry_e + inc_e - le;
        }
        carry += __shfl(inc, 63, 64);
        carry_s += __shfl(inc_s, 63, 64);
        carry_e += __shfl(inc_e, 63, 64);
        sampled += ls;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sampled += __shfl_xor(sampled, off, 64);
    if (lane != 0) return;
    pb.qblk[q] = carry;
    pb.qblk_s[q] = carry_s;
    pb.sq[q] = total;
    pb.su[q] = total_u;
    pb.nsample[q] = (uint32_t)(sampled > 0xFFFFFFF0ull ? 0xFFFFFFF0ull : sampled);
    pb.fully[q] = fully ? 1 : 0;
    if (fully && pb.place) pb.cnt[q] = (uint32_t)total;   // its records are placed by position, not counted
    bool exact_only = true;
    const unsigned long long capv = ivfr_plan_capacity(total, total_u, sampled, qp, min_cap, kprime, half_frac, &exact_only);
    pb.exact_only[q] = exact_only ? 1 : 0;
    pb.capq[q] = (uint32_t)capv;
    atomicAdd(pb.totals, total);
}

// One workgroup: exclusive prefix sums over the nq queries (candidate-buffer offsets; scan and sample blocks).
__global__ __launch_bounds__(1024) void plan_scan_kernel(int nq, int w, PlanBuffers pb) {
    __shared__ uint32_t wtot[2][16];
    __shared__ uint32_t carry[2];
    __shared__ unsigned long long wtot64[16];
    __shared__ unsigned long long carry64;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) { carry[0] = carry[1] = 0; carry64 = 0; }
    __syncthreads();
    for (int base = 0; base < nq; base += 1024) {
        const int q = base + tid;
        const unsigned long long v64 = q < nq ? (((unsigned long long)pb.capq[q] + 31ull) & ~31ull) : 0ull;
        unsigned long long inc64 = v64;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            unsigned long long o = __shfl_up(inc64, off, 64);
            if (lane >= off) inc64 += o;
        }
        const uint32_t v[2] = {q < nq ? pb.qblk[q] : 0u, q < nq ? pb.qblk_s[q] : 0u};
        uint32_t inc[2] = {wave_incl_scan(v[0], lane), wave_incl_scan(v[1], lane)};
        if (lane == 63) { wtot64[wv] = inc64; wtot[0][wv] = inc[0]; wtot[1][wv] = inc[1]; }
        __syncthreads();
        unsigned long long add64 = carry64;
        uint32_t add[2] = {carry[0], carry[1]};
        for (int x = 0; x < wv; ++x) { add64 += wtot64[x]; add[0] += wtot[0][x]; add[1] += wtot[1][x]; }
        inc64 += add64; inc[0] += add[0]; inc[1] += add[1];
        if (q < nq) {
            pb.coff[q] = inc64 - v64;
            pb.qblk[q] = inc[0] - v[0];     // now the query's first block in the batch-wide stream
            pb.qblk_s[q] = inc[1] - v[1];
        }
        __syncthreads();
        if (tid == 1023) { carry64 = inc64; carry[0] = inc[0]; carry[1] = inc[1]; }
        __syncthreads();
    }
    if (tid == 0) {
        // A candidate pool smaller than the plan wants voids the batch: no block of any pair is scanned (the host
        // reads the flag after the call's only wait, grows the pool and runs the batch again).
        const bool dead = carry64 > pb.pool_cap;
        pb.totals[1] = carry64;
        pb.status->pool_short = dead ? 1u : 0u;
        pb.blkpre[nq * w] = dead ? 0u : carry[0];
        pb.blkpre_s[nq * w] = dead ? 0u : carry[1];
        pb.status->n_sample_chunks = dead ? 0u : carry[1];
    }
}

// The per-query block offsets are added to the query-relative prefixes of the P pairs, and the pair of
// every sample chunk is written out.
__global__ __launch_bounds__(256) void plan_expand_kernel(int P, int w, PlanBuffers pb) {
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= P) return;
    const int q = p / w;
    if (pb.status->pool_short) {   // void batch: every pair is empty, no query has a sample
        pb.len[p] = 0; pb.len_s[p] = 0; pb.blkpre[p] = 0; pb.blkpre_s[p] = 0;
        if (p == q * w) { pb.nsample[q] = 0; pb.cnt[q] = 0; }
        return;
    }
    pb.blkpre[p] += pb.qblk[q];
    const uint32_t first = pb.blkpre_s[p] + pb.qblk_s[q];
    pb.blkpre_s[p] = first;
    const uint32_t nchunk = (pb.len_s[p] + IVFR_SAMPLE_CHUNK - 1) / IVFR_SAMPLE_CHUNK;
    for (uint32_t i = 0; i < nchunk; ++i) pb.items_s[first + i] = (uint32_t)p;
}

int ivfr_launch_plan(const ivfr_index* ix, const int32_t* probe, int nq, int w, uint32_t full_limit,
                     uint32_t stride_k, uint32_t min_cap, uint32_t max_sample, int kprime, float half_frac,
                     const PlanBuffers& pb, hipStream_t st) {
    hipLaunchKernelGGL(plan_pairs_kernel, dim3((nq + 3) / 4), dim3(256), 0, st, probe, nq, w, ix->list_start,
                       ix->list_len, full_limit, stride_k, min_cap, max_sample, kprime, half_frac, pb);
    IVFR_HIP(hipGetLastError());
    hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(1024), 0, st, nq, w, pb);
    hipLaunchKernelGGL(plan_expand_kernel, dim3((nq * w + 255) / 256), dim3(256), 0, st, nq * w, w, pb);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// ------------------------------------------------------------------------------------------
// Look-up tables of Eq. (5), one per (query, visited list):
//   T[p][j][k] = || (x_q - coarse[l])^j - pq[j][k] ||^2 = ||r^j||^2 + ||pq[j][k]||^2 - 2 r^j . pq[j][k]
// The dot products are a [pairs x dsub] . [dsub x 256] contraction per sub-quantizer and run
// on the matrix cores (v_mfma_f32_32x32x2_f32): a workgroup takes 32 pairs, keeps their
// residuals in LDS, and each wavefront walks its share of the (j, 32-centroid tile) grid.
// Negative round-off is clamped to zero (the quantity is a squared norm).
// ------------------------------------------------------------------------------------------
// Sixteen wavefronts per workgroup: a wavefront's (j, tile) units are chains of dependent loads (codebook rows from
// L2, then the matrix instructions, then the stores), so the latency is hidden by the number of wavefronts.
#define LUT_T 1024
__global__ __launch_bounds__(LUT_T) void lut_mfma_kernel(const float* __restrict__ queries,
                                                       const int32_t* __restrict__ probe, int P, int w, int d, int m,
                                                       int dsub, const float* __restrict__ coarse,
                                                       const float* __restrict__ pq, const float* __restrict__ pq_norm,
                                                       const float* __restrict__ pq_maxnorm,
                                                       float* __restrict__ lut, float* __restrict__ lut_scale) {
    extern __shared__ float smem[];
    const int stride = d + 4;
    float* R = smem;                   // [32][d + 4]
    float* rn = smem + 32 * stride;    // [32][m]
    const int p0 = blockIdx.x * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 32 * (d / 4); i += LUT_T) {
        int pr = i / (d / 4), e = (i % (d / 4)) * 4;
        int p = p0 + pr;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p < P) {
            int q = p / w;
            int l = probe[p];
            float4 x = *reinterpret_cast<const float4*>(queries + (int64_t)q * d + e);
            float4 cc = *reinterpret_cast<const float4*>(coarse + (int64_t)l * d + e);
            v = make_float4(x.x - cc.x, x.y - cc.y, x.z - cc.z, x.w - cc.w);
        }
        *reinterpret_cast<float4*>(R + pr * stride + e) = v;
    }
    __syncthreads();
    for (int i = tid; i < 32 * m; i += LUT_T) {
        int pr = i / m, j = i % m;
        float s = 0.f;
        for (int e = 0; e < dsub; ++e) { float v = R[pr * stride + j * dsub + e]; s = fmaf(v, v, s); }
        rn[i] = s;
    }
    __syncthreads();
    // fp16 scale of the pair's table: every entry is at most (||r^j|| + max_k ||pq[j][k]||)^2, so with
    // s = 60000 / sum_j of those bounds no sum of m scaled entries overflows half precision
    if (tid < 32 && p0 + tid < P) {
        float ub = 0.f;
        for (int j = 0; j < m; ++j) { float a = sqrtf(rn[tid * m + j]) + pq_maxnorm[j]; ub = fmaf(a, a, ub); }
        lut_scale[p0 + tid] = ub > 0.f ? 60000.f / ub : 1.f;
    }
    const int r = lane & 31, h = lane >> 5;
    const int ntile = m * 8;   // (j, 32-centroid tile) units
    for (int u = wave; u < ntile; u += LUT_T / 64) {
        const int j = u >> 3, nt = u & 7;
        floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        const float* brow = pq + ((int64_t)j * IVFR_KS + nt * 32 + r) * dsub;
        for (int kk = 0; kk < dsub; kk += 8) {
            float4 a = *reinterpret_cast<const float4*>(R + r * stride + j * dsub + kk + 4 * h);
            float4 b = *reinterpret_cast<const float4*>(brow + kk + 4 * h);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
        const float pn = pq_norm[j * IVFR_KS + nt * 32 + r];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int pr = 8 * (v >> 2) + 4 * h + (v & 3);
            int p = p0 + pr;
            if (p < P) {
                float val = fmaxf(0.f, fmaf(-2.f, acc[v], rn[pr * m + j] + pn));
                lut[((int64_t)p * m + j) * IVFR_KS + nt * 32 + r] = val;
            }
        }
    }
}

// Direct-form tables for sub-vector widths the MFMA path does not cover (dsub % 8 != 0).
__global__ __launch_bounds__(256) void lut_direct_kernel(const float* __restrict__ queries,
                                                         const int32_t* __restrict__ probe, int P, int w, int d, int m,
                                                         int dsub, const float* __restrict__ coarse,
                                                         const float* __restrict__ pq,
                                                         const float* __restrict__ pq_maxnorm,
                                                         float* __restrict__ lut, float* __restrict__ lut_scale) {
    extern __shared__ float smem[];   // residual [d]
    const int p = blockIdx.x;
    const int q = p / w, l = probe[p];
    for (int e = threadIdx.x; e < d; e += 256) smem[e] = queries[(int64_t)q * d + e] - coarse[(int64_t)l * d + e];
    __syncthreads();
    if (threadIdx.x == 0) {
        float ub = 0.f;
        for (int j = 0; j < m; ++j) {
            float s2 = 0.f;
            for (int e = 0; e < dsub; ++e) s2 = fmaf(smem[j * dsub + e], smem[j * dsub + e], s2);
            float a = sqrtf(s2) + pq_maxnorm[j];
            ub = fmaf(a, a, ub);
        }
        lut_scale[p] = ub > 0.f ? 60000.f / ub : 1.f;
    }
    for (int i = threadIdx.x; i < m * IVFR_KS; i += 256) {
        int j = i / IVFR_KS;
        const float* cb = pq + (int64_t)i * dsub;
        float s = 0.f;
        for (int e = 0; e < dsub; ++e) { float df = smem[j * dsub + e] - cb[e]; s = fmaf(df, df, s); }
        lut[(int64_t)p * m * IVFR_KS + i] = s;
    }
}

int ivfr_launch_lut(const ivfr_index* ix, const float* queries, const int32_t* probe, int nq, int w, float* lut,
                    float* lut_scale, hipStream_t st) {
    const int P = nq * w, d = ix->p.d, m = ix->p.m;
    if (P <= 0) return IVFR_OK;
    if (ix->dsub % 8 == 0) {
        size_t lds = (size_t)(32 * (d + 4) + 32 * m) * sizeof(float);
        hipLaunchKernelGGL(lut_mfma_kernel, dim3((P + 31) / 32), dim3(LUT_T), lds, st, queries, probe, P, w, d, m,
                           ix->dsub, ix->coarse, ix->pq, ix->pq_norm, ix->pq_maxnorm, lut, lut_scale);
    } else {
        hipLaunchKernelGGL(lut_direct_kernel, dim3(P), dim3(256), (size_t)d * sizeof(float), st, queries, probe, P, w,
                           d, m, ix->dsub, ix->coarse, ix->pq, ix->pq_maxnorm, lut, lut_scale);
    }
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// ------------------------------------------------------------------------------------------
// Split tables.  The table entry of Eq. (5) for query x, list l (centroid c_l), sub-quantizer j, value k is
//   ||(x - c_l)^j - p_jk||^2 = ||(x - c_l)^j||^2 + (||p_jk||^2 + 2 c_l^j . p_jk) - 2 x^j . p_jk .
// The bracket depends on the list only and is computed once per index (c tables), the last term on the query
// only (one table per query instead of one per (query, list) pair), and the first is m scalars per pair; the
// scan kernels add the three when a pair's table enters LDS, so no per-pair table is ever written to memory.
// Both term tables are rows V [n, d] against the PQ codebook:  out[row][j][k] = beta ||p_jk||^2 + alpha V[row]^j . p_jk
// (list terms: V = coarse centroids, alpha = 2, beta = 1; query terms: V = queries, alpha = -2, beta = 0), the
// dot products on the matrix cores exactly as in the per-pair table kernel above.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void term_mfma_kernel(const float* __restrict__ V, int n, int d, int m, int dsub,
                                                        const float* __restrict__ pq, const float* __restrict__ pq_norm,
                                                        float alpha, float beta, float* __restrict__ out) {
    extern __shared__ float smem[];
    const int stride = d + 4;
    float* R = smem;                   // [32][d + 4]
    const int p0 = blockIdx.x * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 32 * (d / 4); i += 256) {
        int pr = i / (d / 4), e = (i % (d / 4)) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p0 + pr < n) v = *reinterpret_cast<const float4*>(V + (int64_t)(p0 + pr) * d + e);
        *reinterpret_cast<float4*>(R + pr * stride + e) = v;
    }
    __syncthreads();
    const int r = lane & 31, h = lane >> 5;
    const int ntile = m * 8;   // (j, 32-centroid tile) units
    for (int u = wave; u < ntile; u += 4) {
        const int j = u >> 3, nt = u & 7;
        floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        const float* brow = pq + ((int64_t)j * IVFR_KS + nt * 32 + r) * dsub;
        for (int kk = 0; kk < dsub; kk += 8) {
            float4 a = *reinterpret_cast<const float4*>(R + r * stride + j * dsub + kk + 4 * h);
            float4 b = *reinterpret_cast<const float4*>(brow + kk + 4 * h);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
        const float pn = beta * pq_norm[j * IVFR_KS + nt * 32 + r];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int pr = 8 * (v >> 2) + 4 * h + (v & 3);
            if (p0 + pr < n) out[((int64_t)(p0 + pr) * m + j) * IVFR_KS + nt * 32 + r] = fmaf(alpha, acc[v], pn);
        }
    }
}

// the same for sub-vector widths the MFMA path does not cover (dsub % 8 != 0): one thread per output
__global__ __launch_bounds__(256) void term_direct_kernel(const float* __restrict__ V, int64_t n, int d, int m, int dsub,
                                                          const float* __restrict__ pq,
                                                          const float* __restrict__ pq_norm, float alpha, float beta,
                                                          float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;   // row * m * 256 + j * 256 + k
    if (i >= n * m * IVFR_KS) return;
    const int64_t row = i / (m * IVFR_KS);
    const int e = (int)(i % (m * IVFR_KS)), j = e >> 8;
    const float* v = V + row * d + j * dsub;
    const float* cb = pq + (int64_t)e * dsub;
    float s = 0.f;
    for (int t = 0; t < dsub; ++t) s = fmaf(v[t], cb[t], s);
    out[i] = fmaf(alpha, s, beta * pq_norm[e]);
}

static int launch_terms(const ivfr_index* ix, const float* V, int64_t n, float alpha, float beta, float* out,
                        hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    const int d = ix->p.d, m = ix->p.m;
    if (ix->dsub % 8 == 0) {
        const size_t lds = (size_t)(32 * (d + 4)) * sizeof(float);
        hipLaunchKernelGGL(term_mfma_kernel, dim3((unsigned)((n + 31) / 32)), dim3(256), lds, st, V, (int)n, d, m, ix->dsub,
                           ix->pq, ix->pq_norm, alpha, beta, out);
    } else {
        const int64_t total = n * m * IVFR_KS;
        hipLaunchKernelGGL(term_direct_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, V, n, d, m,
                           ix->dsub, ix->pq, ix->pq_norm, alpha, beta, out);
    }
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// Per pair: pbase[p][j] = ||(x_q - c_l)^j||^2 (the same fused multiply-add chain as in the per-pair table kernel) and
// the fp16 scale of the pair's table.  The m lanes of a pair sit side by side.
__global__ __launch_bounds__(256) void pair_base_kernel(const float* __restrict__ queries,
                                                        const int32_t* __restrict__ probe, int P, int w, int d, int m,
                                                        int dsub, const float* __restrict__ coarse,
                                                        const float* __restrict__ pq_maxnorm,
                                                        float* __restrict__ pbase, float* __restrict__ lut_scale) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t p = i / m;
    const int j = (int)(i % m);
    float a2 = 0.f;
    if (p < P) {
        const float* x = queries + (p / w) * d + j * dsub;
        const float* cc = coarse + (int64_t)probe[p] * d + j * dsub;
        float s = 0.f;
        for (int e = 0; e < dsub; ++e) { const float v = x[e] - cc[e]; s = fmaf(v, v, s); }
        pbase[p * m + j] = s;
        const float a = sqrtf(s) + pq_maxnorm[j];
        a2 = a * a;
    }
    // upper bound of the table's entries: sum over the pair's m lanes (m is a power of two, at most 64)
    for (int off = m >> 1; off >= 1; off >>= 1) a2 += __shfl_xor(a2, off, 64);
    if (p < P && j == 0) lut_scale[p] = a2 > 0.f ? 60000.f / a2 : 1.f;
}

int ivfr_launch_list_terms(const ivfr_index* ix, float* list_term, hipStream_t st) {
    return launch_terms(ix, ix->coarse, ix->p.c, 2.f, 1.f, list_term, st);
}

int ivfr_launch_query_terms(const ivfr_index* ix, const float* queries, const int32_t* probe, int nq, int w,
                            float* qterm, float* pbase, float* lut_scale, hipStream_t st) {
    IVFR_TRY(launch_terms(ix, queries, nq, -2.f, 0.f, qterm, st));
    const int64_t total = (int64_t)nq * w * ix->p.m;
    if (total > 0) {
        hipLaunchKernelGGL(pair_base_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, queries, probe,
                           nq * w, w, ix->p.d, ix->p.m, ix->dsub, ix->coarse, ix->pq_maxnorm, pbase, lut_scale);
        IVFR_HIP(hipGetLastError());
    }
    return IVFR_OK;
}

// ------------------------------------------------------------------------------------------
// ADC list scan (Eq. (5)): estimate = sum over the m code bytes of T[j][byte_j].
//
// The visited (pair, block) work of a pass is one virtual stream of blocks of IVFR_BLOCK entries;
// workgroup g of G takes the contiguous share [total*g/G, total*(g+1)/G) of it, so every
// workgroup streams the same number of code bytes whatever the list-length skew, and reloads
// the pair's table (m KB, LDS) only when its share crosses into the next pair.  A thread
// loads 16 code bytes per block with one coalesced dwordx4 load.  Estimates <= tau[q] are
// appended to query q's candidate buffer as (estimate bits, entry position) records, slots
// reserved by wavefront-aggregated atomics (collected in a small LDS queue first when a
// filter is active, see below); the counter keeps counting past the buffer's capacity so
// the host can tell an overflow.
// ------------------------------------------------------------------------------------------

// Workgroups are dealt to the eight XCDs (each with its own L2) round-robin by blockIdx.  Giving the
// workgroups of one XCD a contiguous eighth of the block stream keeps neighbours in the stream - which
// work on the same pair or unit and read the same tables - behind the same L2.
__device__ __forceinline__ uint32_t xcd_share_index(uint32_t block, uint32_t groups) {
    return (groups & 7u) ? block : (block & 7u) * (groups >> 3) + (block >> 3);
}

// The share [b, b_end) of the launch's block stream that this workgroup (or, with `parts` > 1, this one of the
// workgroup's `parts` wavefronts) takes.  The stream is blkpre[0] .. blkpre[n] (blkpre may be a slice of a longer
// prefix array, so positions are absolute).  With bpg > 0 only min(gridDim.x, max(g_min, blocks / bpg))
// workgroups, rounded up to a multiple of eight, take part; the others return false at once.
__device__ __forceinline__ bool scan_share(const uint32_t* __restrict__ blkpre, int n, uint32_t bpg, uint32_t g_min,
                                           uint32_t parts, uint32_t part, uint32_t& b, uint32_t& b_end) {
    const uint32_t base = blkpre[0], total = blkpre[n] - base;
    uint32_t G = gridDim.x;
    if (bpg) {
        uint32_t want = total / bpg;
        want = want < g_min ? g_min : want;
        want = (want + 7u) & ~7u;
        if (want < G) G = want;
    }
    if (blockIdx.x >= G) return false;
    const uint32_t g = xcd_share_index(blockIdx.x, G) * parts + part, NG = G * parts;
    b = base + (uint32_t)(((uint64_t)total * g) / NG);
    b_end = base + (uint32_t)(((uint64_t)total * (g + 1)) / NG);
    return b < b_end;
}

template <int M>
__device__ __forceinline__ float adc_sum(const float* lut, const uint32_t* wds) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int t = 0; t < M / 4; ++t) {
        uint32_t v = wds[t];
        const float* L = lut + t * 4 * IVFR_KS;
        s0 += L[v & 0xff];
        s1 += L[IVFR_KS + ((v >> 8) & 0xff)];
        s0 += L[2 * IVFR_KS + ((v >> 16) & 0xff)];
        s1 += L[3 * IVFR_KS + (v >> 24)];
    }
    return s0 + s1;
}

// The same sum, in the same order, read entry by entry from the pair's table in global memory (exact
// re-evaluation of candidates that a reduced-precision filter let through).
template <int M>
__device__ __forceinline__ float adc_sum_pair(const PairTable& pt, const uint32_t* wds) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int t = 0; t < M / 4; ++t) {
        uint32_t v = wds[t];
        const int o = t * 4 * IVFR_KS;
        s0 += pt.get(o + (int)(v & 0xff));
        s1 += pt.get(o + IVFR_KS + (int)((v >> 8) & 0xff));
        s0 += pt.get(o + 2 * IVFR_KS + (int)((v >> 16) & 0xff));
        s1 += pt.get(o + 3 * IVFR_KS + (int)(v >> 24));
    }
    return s0 + s1;
}

__device__ __forceinline__ void append_records(bool keep0, float e0, uint32_t pos0, bool keep1, float e1,
                                               uint32_t pos1, uint2* cand, uint32_t* cnt, uint32_t cap) {
    const uint64_t m0 = __ballot(keep0), m1 = __ballot(keep1);
    if ((m0 | m1) == 0) return;
    const int lane = threadIdx.x & 63;
    const uint32_t n0 = __popcll(m0), n1 = __popcll(m1);
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(cnt, n0 + n1);
    base = __shfl(base, 0, 64);
    const uint64_t below = (1ull << lane) - 1ull;
    if (keep0) {
        uint32_t s = base + __popcll(m0 & below);
        if (s < cap) cand[s] = make_uint2(__float_as_uint(e0), pos0);
    }
    if (keep1) {
        uint32_t s = base + n0 + __popcll(m1 & below);
        if (s < cap) cand[s] = make_uint2(__float_as_uint(e1), pos1);
    }
}


// ------------------------------------------------------------------------------------------
// Appending through a wavefront queue.  When a noticeable share of the estimates passes the bound,
// an atomic (with its round trip) in most passes of the scan loop stalls all 64 lanes.  The fp32
// scans therefore collect what they keep in a small LDS queue per wavefront, (estimate, position,
// query slot of the unit), and write it out when the queue is nearly full or the unit ends: one
// atomic per query slot and 64 queued records, issued together.
// ------------------------------------------------------------------------------------------
#define WQ_CAP 160   // records per wavefront queue; a push adds at most 128
struct WaveQueue {
    uint32_t* est;   // [WQ_CAP] LDS
    uint32_t* pos;   // [WQ_CAP]
    uint32_t* tag;   // [WQ_CAP] query slot inside the unit
    uint32_t n;      // uniform over the wavefront
};
#define WQ_WORDS (3 * WQ_CAP)   // LDS words per wavefront

__device__ __forceinline__ void wq_push(WaveQueue& wq, bool k0, float e0, uint32_t p0, bool k1, float e1, uint32_t p1,
                                        uint32_t tag) {
    const uint64_t m0 = __ballot(k0), m1 = __ballot(k1);
    if ((m0 | m1) == 0) return;
    const uint64_t below = (1ull << (threadIdx.x & 63)) - 1ull;
    const uint32_t n0 = __popcll(m0);
    if (k0) {
        const uint32_t s = wq.n + __popcll(m0 & below);
        wq.est[s] = __float_as_uint(e0); wq.pos[s] = p0; wq.tag[s] = tag;
    }
    if (k1) {
        const uint32_t s = wq.n + n0 + __popcll(m1 & below);
        wq.est[s] = __float_as_uint(e1); wq.pos[s] = p1; wq.tag[s] = tag;
    }
    wq.n += n0 + __popcll(m1);
}

// qc[x], cnt[x], cap[x]: buffer, counter and capacity of query slot x of the current unit
template <int G>
__device__ __forceinline__ void wq_flush(WaveQueue& wq, uint2* const (&qc)[G], uint32_t* const (&cnt)[G],
                                         const uint32_t (&cap)[G]) {
    const int lane = threadIdx.x & 63;
    const uint64_t below = (1ull << lane) - 1ull;
    for (uint32_t base = 0; base < wq.n; base += 64) {
        const uint32_t i = base + lane;
        const bool valid = i < wq.n;
        const uint32_t tag = valid ? wq.tag[i] : 0xFFFFFFFFu;
        uint32_t rank = 0, mine = 0;
        uint32_t* my_cnt = cnt[0];
#pragma unroll
        for (int x = 0; x < G; ++x) {
            const uint64_t bx = __ballot(tag == (uint32_t)x);
            if (tag == (uint32_t)x) rank = __popcll(bx & below);
            if (lane == x) { mine = __popcll(bx); my_cnt = cnt[x]; }
        }
        uint32_t got = 0;
        if (lane < G && mine) got = atomicAdd(my_cnt, mine);   // the G atomics are in flight together
#pragma unroll
        for (int x = 0; x < G; ++x) {
            const uint32_t gx = __shfl(got, x, 64);
            if (tag == (uint32_t)x) {
                const uint32_t slot = gx + rank;
                if (slot < cap[x]) qc[x][slot] = make_uint2(wq.est[i], wq.pos[i]);
            }
        }
    }
    wq.n = 0;
}

// PLACE: some queries of the launch may keep everything with their records placed by position (`direct`); without it
// the argument is never read.
template <int M, bool PLACE>
__global__ __launch_bounds__(256) void adc_scan_kernel(const uint8_t* __restrict__ codes,
                                                       TableSrc ts,
                                                       const uint32_t* __restrict__ pair_start,
                                                       const uint32_t* __restrict__ pair_len,
                                                       const uint32_t* __restrict__ blkpre,
                                                       const uint32_t* __restrict__ unit_pairs, int n_host,
                                                       const uint32_t* __restrict__ n_dev, uint32_t bpg,
                                                       uint32_t g_min, int w,
                                                       const float* __restrict__ tau, uint2* __restrict__ cand,
                                                       uint32_t* __restrict__ cand_cnt, CandLayout lay,
                                                       const uint32_t* __restrict__ tau_id,
                                                       const int32_t* __restrict__ ids, uint32_t id_stride,
                                                       DirectPlace direct) {
    extern __shared__ float s_lut[];   // M * 256 floats, then the wavefronts' append queues
    WaveQueue wq;
    wq.est = reinterpret_cast<uint32_t*>(s_lut) + M * IVFR_KS + (threadIdx.x >> 6) * WQ_WORDS;
    wq.pos = wq.est + WQ_CAP;
    wq.tag = wq.pos + WQ_CAP;
    wq.n = 0;
    const int P = n_dev ? (int)*n_dev : n_host;
    uint32_t b, b_end;
    if (P <= 0 || !scan_share(blkpre, P, bpg, g_min, 1u, 0u, b, b_end)) return;
    // last pair p with blkpre[p] <= b
    int lo = 0, hi = P;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (blkpre[mid] <= b) lo = mid; else hi = mid;
    }
    int p = lo;
    const int tid = threadIdx.x;
    while (b < b_end) {
        while (blkpre[p + 1] <= b) ++p;   // skip pairs without blocks in this pass
        const uint32_t pb0 = blkpre[p], pb1 = blkpre[p + 1];
        const uint32_t stop = pb1 < b_end ? pb1 : b_end;
        const int64_t pid = unit_pairs ? (int64_t)unit_pairs[p] : (int64_t)p;   // unit p of this launch is pair pid
        const int q = (int)(pid / w);
        const uint32_t start = pair_start[pid], len = pair_len[pid];
        const float t = tau[q];
        // with tau_id the bound is the 64-bit key (estimate, id): an estimate equal to tau passes only up to that id
        const uint32_t t_id = tau_id ? tau_id[q] : 0xFFFFFFFFu;
        const bool keep_all = t == INFINITY;
        const bool placed = PLACE && direct.fully[q];   // implies keep_all
        const uint32_t place0 = placed ? direct.off[pid] : 0u;
        uint2* const qc[1] = {cand + lay.base(q)};
        const uint32_t cap[1] = {lay.cap(q)};
        uint32_t* const cnt[1] = {cand_cnt + q};
        __syncthreads();   // previous pair's table no longer in use
        {
            const PairTable pt = ts.pair(pid);
            float4* dst = reinterpret_cast<float4*>(s_lut);
            for (int i = tid; i < M * IVFR_KS / 4; i += 256) dst[i] = pt.get4(4 * i);
        }
        __syncthreads();
        // two blocks per iteration: both loads are issued before the first table look-up
        for (uint32_t bb = b; bb < stop; bb += 2) {
            uint32_t wds[2][2][M / 4];
            uint32_t e0[2];
            bool in0[2], in1[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                e0[u] = (bb + u - pb0) * IVFR_BLOCK + 2u * tid;   // entry inside the list
                in0[u] = bb + u < stop && e0[u] < len;
                in1[u] = bb + u < stop && e0[u] + 1 < len;
                if (in0[u]) {
                    const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + e0[u]) * M);
                    if (M == 8) {
                        uint4 v = *reinterpret_cast<const uint4*>(src);
                        wds[u][0][0] = v.x; wds[u][0][1] = v.y; wds[u][1][0] = v.z; wds[u][1][1] = v.w;
                    } else {
#pragma unroll
                        for (int t2 = 0; t2 < M / 4; ++t2) { wds[u][0][t2] = src[t2]; wds[u][1][t2] = src[M / 4 + t2]; }
                    }
                } else {
#pragma unroll
                    for (int t2 = 0; t2 < M / 4; ++t2) { wds[u][0][t2] = 0; wds[u][1][t2] = 0; }
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const float est0 = adc_sum<M>(s_lut, wds[u][0]);
                const float est1 = adc_sum<M>(s_lut, wds[u][1]);
                bool k0 = in0[u] && est0 <= t, k1 = in1[u] && est1 <= t;
                if (tau_id) {
                    if (k0 && est0 == t) k0 = (uint32_t)ids[(size_t)(start + e0[u]) * id_stride] <= t_id;
                    if (k1 && est1 == t) k1 = (uint32_t)ids[(size_t)(start + e0[u] + 1) * id_stride] <= t_id;
                }
                if (PLACE && placed) {   // every entry has its own place: no counter
                    const uint32_t s0 = place0 + e0[u];
                    if (in0[u] && s0 < cap[0]) qc[0][s0] = make_uint2(__float_as_uint(est0), start + e0[u]);
                    if (in1[u] && s0 + 1 < cap[0]) qc[0][s0 + 1] = make_uint2(__float_as_uint(est1), start + e0[u] + 1);
                } else if (keep_all) {   // nothing is filtered: a full wavefront of records per pass, one atomic for all of them
                    append_records(k0, est0, start + e0[u], k1, est1, start + e0[u] + 1, qc[0], cnt[0], cap[0]);
                } else {
                    if (wq.n > WQ_CAP - 128) wq_flush<1>(wq, qc, cnt, cap);
                    wq_push(wq, k0, est0, start + e0[u], k1, est1, start + e0[u] + 1, 0u);
                }
            }
        }
        wq_flush<1>(wq, qc, cnt, cap);   // the queue belongs to this pair's query
        b = stop;
    }
}

template <int M>
static size_t scan_lds_bytes() { return (size_t)(M * IVFR_KS + 4 * WQ_WORDS) * sizeof(float); }

template <int M>
static int launch_scan_m(const ivfr_index* ix, const TableSrc& ts, const uint32_t* pair_start, const uint32_t* pair_len,
                         const uint32_t* blkpre, const uint32_t* unit_pairs, const ScanShape& sh, int w,
                         const float* tau, uint2* cand, uint32_t* cand_cnt, CandLayout lay, hipStream_t st,
                         const uint32_t* tau_id, DirectPlace direct) {
#define IVFR_SCAN_LAUNCH(PL)                                                                                      \
    hipLaunchKernelGGL((adc_scan_kernel<M, PL>), dim3(sh.groups), dim3(256), scan_lds_bytes<M>(), st, ix->codes, ts,  \
                       pair_start, pair_len, blkpre, unit_pairs, sh.n_host, sh.n_dev, sh.bpg, sh.g_min, w, tau, cand, \
                       cand_cnt, lay, tau_id, reinterpret_cast<const int32_t*>(ix->rec),                              \
                       (uint32_t)(ix->rec_stride / 4), direct)
    if (direct.fully) IVFR_SCAN_LAUNCH(true);
    else IVFR_SCAN_LAUNCH(false);
#undef IVFR_SCAN_LAUNCH
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

int ivfr_launch_scan(const ivfr_index* ix, const TableSrc& ts, const uint32_t* pair_start, const uint32_t* pair_len,
                     const uint32_t* blkpre, const uint32_t* unit_pairs, ScanShape sh, int w, const float* tau,
                     uint2* cand, uint32_t* cand_cnt, CandLayout lay, hipStream_t st, const uint32_t* tau_id,
                     DirectPlace direct) {
    if (!sh.n_dev && sh.n_host <= 0) return IVFR_OK;
#define IVFR_SCAN_CASE(MM)                                                                                     \
    case MM:                                                                                                   \
        return launch_scan_m<MM>(ix, ts, pair_start, pair_len, blkpre, unit_pairs, sh, w, tau, cand, cand_cnt, \
                                 lay, st, tau_id, direct)
    switch (ix->p.m) {
        IVFR_SCAN_CASE(4);
        IVFR_SCAN_CASE(8);
        IVFR_SCAN_CASE(16);
        IVFR_SCAN_CASE(32);
        IVFR_SCAN_CASE(64);
        default:
            ivfr_set_error("list scan supports m in {4, 8, 16, 32, 64}; got %d", ix->p.m);
            return IVFR_ERR_INVALID_ARG;
    }
#undef IVFR_SCAN_CASE
}

// ------------------------------------------------------------------------------------------
// Shared scan: queries of one batch that visit the same list are scanned together.
//
// Four (query, list) pairs with the same list form a unit: the list's codes are loaded once
// and every code byte indexes a table of float4 whose lanes are the four queries' entries
// (LDS layout [j][k][4]), so one 16-byte LDS read serves four queries.  On this chip a random
// 64-lane ds_read_b128 costs ~10 LDS cycles for 256 values against ~7 cycles for the 64
// values of a random ds_read_b32, and the list is read from HBM once instead of four times.
// Each query keeps its own bound tau, counter and candidate buffer, and its estimate is the
// same sum of the same eight fp32 terms in the same order as in the per-pair kernel.
// A list visited by 4n+3 queries gets one unit with an empty slot, 4n+2 a unit of two (8-byte
// LDS reads), 4n+1 leaves a single pair to the per-pair kernel.
// ------------------------------------------------------------------------------------------
#define IVFR_NO_PAIR 0xFFFFFFFFu   // empty slot of a unit

// Pairs of a query whose bound lets only a tiny share of its estimates pass (class 0) may go into the
// half-precision units of eight; pairs of the other queries (class 1) only into the fp32 units.
__global__ void group_count_kernel(const int32_t* __restrict__ probe, int P, int w, const uint8_t* __restrict__ exact_only,
                                   int use8, uint32_t* __restrict__ list_np) {
    int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const int cls = (use8 && !exact_only[p / w]) ? 0 : 1;
    atomicAdd(&list_np[2 * probe[p] + cls], 1u);
}

// A list visited by nA class-0 and nB class-1 pairs yields: with use64, units of 64 from every full 64 class-0
// pairs; units of eight from the other class-0 pairs
// (a remainder of 5..7 becomes one more unit with empty slots); the other class-0 pairs join the
// class-1 pairs in a pool of n that gives n/4 units of four (a remainder of 3 becomes one more
// unit with an empty slot), a remainder of 2 a unit of two, a remainder of 1 a single pair.
struct ListSplit { uint32_t n64, in64, n8, in8, restA, n4, in4, n2, n1; };
__device__ __forceinline__ ListSplit split_units(uint32_t nA, uint32_t nB, int use64) {
    ListSplit s;
    // full units of 64 class-0 pairs first (matrix-core scan); the rest as below
    s.n64 = use64 ? nA / 64u : 0u;
    s.in64 = s.n64 * 64u;
    nA -= s.in64;
    const uint32_t rA = nA & 7u;
    s.n8 = nA / 8 + (rA >= 5 ? 1u : 0u);
    s.in8 = rA >= 5 ? nA : nA - rA;
    s.restA = nA - s.in8;
    const uint32_t n = s.restA + nB, r = n & 3u;
    s.n4 = n / 4 + (r == 3 ? 1u : 0u);
    s.in4 = r == 3 ? n : n - r;
    s.n2 = r == 2 ? 1u : 0u;
    s.n1 = r == 1 ? 1u : 0u;
    return s;
}

// per list: exclusive prefixes of the five kinds of unit (eight, four, two, single, 64); one workgroup per kind
__global__ __launch_bounds__(1024) void group_scan_lists_kernel(int c, int use64, const uint32_t* __restrict__ list_np,
                                                                uint32_t* __restrict__ gpre /*[5][c]*/,
                                                                uint32_t* __restrict__ cur /*[2c]*/,
                                                                uint32_t* __restrict__ counts /*[5]*/) {
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int a = blockIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < c; base += 1024) {
        const int l = base + tid;
        uint32_t v = 0;
        if (l < c) {
            const ListSplit sp = split_units(list_np[2 * l], list_np[2 * l + 1], use64);
            v = a == 0 ? sp.n8 : (a == 1 ? sp.n4 : (a == 2 ? sp.n2 : (a == 3 ? sp.n1 : sp.n64)));
        }
        uint32_t inc = wave_incl_scan(v, lane);
        if (lane == 63) wtot[wv] = inc;
        __syncthreads();
        uint32_t add = carry;
        for (int x = 0; x < wv; ++x) add += wtot[x];
        inc += add;
        if (l < c) {
            gpre[(int64_t)a * c + l] = inc - v;
            if (a == 0) { cur[2 * l] = 0; cur[2 * l + 1] = 0; }
        }
        __syncthreads();
        if (tid == 1023) carry = inc;
        __syncthreads();
    }
    if (tid == 0) counts[a] = carry;
}

__global__ void group_fill_kernel(const int32_t* __restrict__ probe, int P, int w,
                                  const uint8_t* __restrict__ exact_only,
                                  int use8, int use64, int c, const uint32_t* __restrict__ list_np,
                                  const uint32_t* __restrict__ gpre, uint32_t* __restrict__ cur,
                                  uint32_t* __restrict__ unit8_pairs, uint32_t* __restrict__ unit4_pairs,
                                  uint32_t* __restrict__ unit2_pairs, uint32_t* __restrict__ lo_pairs,
                                  uint32_t* __restrict__ unit64_pairs) {
    int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const int l = probe[p];
    const int cls = (use8 && !exact_only[p / w]) ? 0 : 1;
    const ListSplit sp = split_units(list_np[2 * l], list_np[2 * l + 1], use64);
    uint32_t i = atomicAdd(&cur[2 * l + cls], 1u);
    if (cls == 0) {
        if (i < sp.in64) {
            unit64_pairs[((int64_t)gpre[4 * (int64_t)c + l] + i / 64) * 64 + (i & 63)] = (uint32_t)p;
            return;
        }
        i -= sp.in64;
    }
    if (cls == 0 && i < sp.in8) {
        unit8_pairs[((int64_t)gpre[l] + i / 8) * 8 + (i & 7)] = (uint32_t)p;
        return;
    }
    const uint32_t k = cls == 0 ? i - sp.in8 : sp.restA + i;   // index in the list's pool
    if (k < sp.in4) unit4_pairs[((int64_t)gpre[(int64_t)c + l] + k / 4) * 4 + (k & 3)] = (uint32_t)p;
    else if (sp.n2) unit2_pairs[(int64_t)gpre[2 * (int64_t)c + l] * 2 + (k - sp.in4)] = (uint32_t)p;
    else lo_pairs[gpre[3 * (int64_t)c + l]] = (uint32_t)p;
}

// block prefixes over the units of one kind and its work total; one workgroup per kind (blockIdx.x:
// 0 = units of eight, 1 = of four, 2 = of two, 3 = single pairs, 4 = units of 64); work[0] must be zero on entry
__global__ __launch_bounds__(1024) void group_scan_units_kernel(const uint32_t* __restrict__ counts, GroupBuffers gb,
                                                                const uint32_t* __restrict__ pair_len) {
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t carry;
    __shared__ unsigned long long s_read, s_est;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int which = blockIdx.x;
    const int n = (int)counts[which];
    const uint32_t* ids = which == 0 ? gb.unit8_pairs : (which == 1 ? gb.unit4_pairs : (which == 2 ? gb.unit2_pairs : (which == 3 ? gb.lo_pairs : gb.unit64_pairs)));
    uint32_t* out = which == 0 ? gb.blk8 : (which == 1 ? gb.blk4 : (which == 2 ? gb.blk2 : (which == 3 ? gb.blklo : gb.blk64)));
    const int step = which == 0 ? 8 : (which == 1 ? 4 : (which == 2 ? 2 : (which == 3 ? 1 : 64)));
    if (tid == 0) { s_read = 0; s_est = 0; carry = 0; }
    __syncthreads();
    unsigned long long my_read = 0, my_est = 0;
    // four consecutive units per thread and step: their loads (pair ids, then the list length behind the first id)
    // are independent chains and in flight together
    for (int base = 0; base < n; base += 4096) {
        const int u0 = base + 4 * tid;
        uint32_t len[4], v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int u = u0 + i;
            len[i] = u < n ? pair_len[ids[(int64_t)u * step]] : 0u;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int u = u0 + i;
            if (u < n) {
                uint32_t members = 0;
                for (int x = 0; x < step; ++x) members += ids[(int64_t)u * step + x] != IVFR_NO_PAIR ? 1u : 0u;
                my_read += len[i];
                my_est += (unsigned long long)len[i] * members;
            }
            v[i] = (len[i] + IVFR_BLOCK - 1) / IVFR_BLOCK;
        }
        const uint32_t vsum = v[0] + v[1] + v[2] + v[3];
        uint32_t inc = wave_incl_scan(vsum, lane);
        if (lane == 63) wtot[wv] = inc;
        __syncthreads();
        uint32_t add = carry;
        for (int x = 0; x < wv; ++x) add += wtot[x];
        inc += add;
        uint32_t run = inc - vsum;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (u0 + i < n) out[u0 + i] = run;
            run += v[i];
        }
        __syncthreads();
        if (tid == 1023) carry = inc;
        __syncthreads();
    }
    // one LDS atomic per wavefront (1024 threads adding 64-bit words to one address would queue up behind one another)
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        my_read += __shfl_xor(my_read, off, 64);
        my_est += __shfl_xor(my_est, off, 64);
    }
    if (lane == 0) {
        atomicAdd(&s_read, my_read);
        atomicAdd(&s_est, my_est);
    }
    __syncthreads();
    if (tid == 0) {
        out[n] = carry;
        atomicAdd(&gb.work[0], s_read);
        gb.work[1 + which] = s_est;
    }
}

int ivfr_launch_group_plan(const int32_t* probe, int P, int w, int c, const uint8_t* exact_only, bool use8, bool use64,
                           const uint32_t* pair_len, const GroupBuffers& gb, hipStream_t st) {
    const int u64 = (use8 && use64) ? 1 : 0;
    hipLaunchKernelGGL(group_count_kernel, dim3((P + 255) / 256), dim3(256), 0, st, probe, P, w, exact_only, use8 ? 1 : 0,
                       gb.list_np);
    hipLaunchKernelGGL(group_scan_lists_kernel, dim3(5), dim3(1024), 0, st, c, u64, gb.list_np, gb.gpre, gb.cur, gb.counts);
    hipLaunchKernelGGL(group_fill_kernel, dim3((P + 255) / 256), dim3(256), 0, st, probe, P, w, exact_only, use8 ? 1 : 0, u64,
                       c, gb.list_np, gb.gpre, gb.cur, gb.unit8_pairs, gb.unit4_pairs, gb.unit2_pairs, gb.lo_pairs,
                       gb.unit64_pairs);
    hipLaunchKernelGGL(group_scan_units_kernel, dim3(5), dim3(1024), 0, st, gb.counts, gb, pair_len);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// Codes of entries e and e+1 of the list that starts at `start` (two M-byte codes = one 16-byte load at
// M = 8), zeros when the block is not part of the pass or the entry lies beyond the list.
template <int M>
__device__ __forceinline__ void load_code_pair(const uint8_t* __restrict__ codes, uint32_t start, uint32_t e, bool live,
                                               uint32_t len, uint32_t (&w0)[M / 4], uint32_t (&w1)[M / 4]) {
    if (live && e < len) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + e) * M);
        if (M == 8) {
            const uint4 c4 = *reinterpret_cast<const uint4*>(src);
            w0[0] = c4.x; w0[1] = c4.y; w1[0] = c4.z; w1[1] = c4.w;
        } else {
#pragma unroll
            for (int t2 = 0; t2 < M / 4; ++t2) { w0[t2] = src[t2]; w1[t2] = src[M / 4 + t2]; }
        }
    } else {
#pragma unroll
        for (int t2 = 0; t2 < M / 4; ++t2) { w0[t2] = 0; w1[t2] = 0; }
    }
}

// The M code bytes rotated down by r (0 <= r < M): byte i of the result is byte (i + r) mod M of the code.
template <int M>
__device__ __forceinline__ void rotate_code_bytes(uint32_t (&w)[M / 4], uint32_t r) {
    const uint32_t r3 = r & 3u;
    if (M == 4) {
        w[0] = __builtin_amdgcn_alignbyte(w[0], w[0], r3);
    } else if (M == 8) {
        const bool sw = (r & 4u) != 0;
        const uint32_t lo = sw ? w[1] : w[0], hi = sw ? w[0] : w[1];
        w[0] = __builtin_amdgcn_alignbyte(hi, lo, r3);
        w[1] = __builtin_amdgcn_alignbyte(lo, hi, r3);
    } else {
        static_assert(M == 4 || M == 8 || M == 16, "code sizes of the shared scans");
        uint32_t t[4], u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = (r & 4u) ? w[(i + 1) & 3] : w[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = (r & 8u) ? t[(i + 2) & 3] : t[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = __builtin_amdgcn_alignbyte(u[(i + 1) & 3], u[i], r3);
    }
}

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));

template <int G> struct LutVec;
template <> struct LutVec<4> { typedef float4 type; };
template <> struct LutVec<2> { typedef float2 type; };

__device__ __forceinline__ void vadd(float4& a, const float4& x) { a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w; }
__device__ __forceinline__ void vadd(float2& a, const float2& x) { a.x += x.x; a.y += x.y; }
__device__ __forceinline__ float vget(const float4& a, int i) { return i == 0 ? a.x : (i == 1 ? a.y : (i == 2 ? a.z : a.w)); }
__device__ __forceinline__ float vget(const float2& a, int i) { return i == 0 ? a.x : a.y; }
__device__ __forceinline__ void vzero(float4& a) { a = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void vzero(float2& a) { a = make_float2(0.f, 0.f); }
__device__ __forceinline__ void vload(float4& a, const float* v) { a = make_float4(v[0], v[1], v[2], v[3]); }
__device__ __forceinline__ void vload(float2& a, const float* v) { a = make_float2(v[0], v[1]); }


// One unit of four queries on half-precision tables (the scheme of the units of eight, documented at
// adc_scan_shared8h_kernel: scaled fp16 tables, packed fp16 sums, an int16 sign test against the rounded-up
// bounds, and an exact fp32 re-evaluation of the queued candidates, which alone is compared and recorded).
// Called by all 256 threads after the barrier that retires the previous unit's tables; blocks [b, stop)
// of the unit whose first block is pb0.  wq's arrays serve as the candidate queue (entry, query mask).
template <int M>
__device__ __forceinline__ void half_unit_pass(const uint8_t* __restrict__ codes, const PairTable (&pt)[4],
                                               const float* __restrict__ lut_scale,
                                               const uint32_t* __restrict__ unit, const int64_t (&pid)[4],
                                               const float (&t)[4], uint2* const (&qc)[4], uint32_t* const (&cnt)[4],
                                               const uint32_t (&cap)[4], uint32_t start, uint32_t len, uint32_t b,
                                               uint32_t stop, uint32_t pb0, float* s_raw, WaveQueue& wq) {
    half4* s_lut4 = reinterpret_cast<half4*>(s_raw);   // [M * 256] x 4 halves
    const int tid = threadIdx.x, lane = tid & 63;
    float sc[4];
    half4 tsh;
    short4v tshi;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const bool real = unit[x] != IVFR_NO_PAIR;
        sc[x] = lut_scale[pid[x]];
        const float ts = real ? t[x] * sc[x] * (1.f + (M + 1.2f) * 4.8828125e-4f) + 4e-3f : 0.f;
        tsh[x] = (_Float16)(real ? ts * 1.001f + 1e-4f : 0.f);
    }
    tshi = __builtin_bit_cast(short4v, tsh);
#pragma unroll
    for (int x = 0; x < 4; ++x)
        if (unit[x] == IVFR_NO_PAIR) tshi[x] = (short)-1;
    for (int e = tid; e < M * IVFR_KS; e += 256) {
        half4 h;
        float v[4];
        unit_table_entries<4>(pt, e, v);
#pragma unroll
        for (int x = 0; x < 4; ++x) h[x] = (_Float16)(v[x] * sc[x]);
        s_lut4[e] = h;
    }
    __syncthreads();
    // exact re-evaluation of the queued candidates, one per lane; one append atomic per query and round
    auto drain = [&]() {
        for (uint32_t base = 0; base < wq.n; base += 64) {
            const uint32_t i = base + lane;
            uint32_t e = 0, mask = 0;
            uint32_t wd[M / 4];
#pragma unroll
            for (int t2 = 0; t2 < M / 4; ++t2) wd[t2] = 0;
            if (i < wq.n) {
                e = wq.est[i];
                mask = wq.pos[i];
                const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + e) * M);
#pragma unroll
                for (int t2 = 0; t2 < M / 4; ++t2) wd[t2] = src[t2];
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const bool mine = ((mask >> x) & 1u) != 0;
                if (__ballot(mine) == 0) continue;
                float est = 0.f;
                bool keep = false;
                if (mine) {
                    est = adc_sum_pair<M>(pt[x], wd);
                    keep = est <= t[x];
                }
                const uint64_t kb = __ballot(keep);
                if (kb == 0) continue;
                const int leader = __ffsll((long long)kb) - 1;
                uint32_t first = 0;
                if (lane == leader) first = atomicAdd(cnt[x], (uint32_t)__popcll(kb));
                first = __builtin_amdgcn_readlane(first, leader);
                if (keep) {
                    const uint32_t slot = first + __builtin_amdgcn_mbcnt_hi((uint32_t)(kb >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)kb, 0u));
                    if (slot < cap[x]) qc[x][slot] = make_uint2(__float_as_uint(est), start + e);
                }
            }
        }
        wq.n = 0;
    };
    for (uint32_t bb = b; bb < stop; bb += 2) {
        uint32_t wds[2][2][M / 4];
        uint32_t e0[2];
        bool in0[2], in1[2];
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            e0[v] = (bb + v - pb0) * IVFR_BLOCK + 2u * tid;
            in0[v] = bb + v < stop && e0[v] < len;
            in1[v] = bb + v < stop && e0[v] + 1 < len;
            load_code_pair<M>(codes, start, e0[v], bb + v < stop, len, wds[v][0], wds[v][1]);
        }
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            half4 ha, hb;
#pragma unroll
            for (int t2 = 0; t2 < M / 4; ++t2) {
                const uint32_t wa = wds[v][0][t2], wb = wds[v][1][t2];
                const half4* L = s_lut4 + t2 * 4 * IVFR_KS;
                if (t2 == 0) { ha = L[wa & 0xff]; hb = L[wb & 0xff]; }
                else { ha += L[wa & 0xff]; hb += L[wb & 0xff]; }
                ha += L[IVFR_KS + ((wa >> 8) & 0xff)];
                hb += L[IVFR_KS + ((wb >> 8) & 0xff)];
                ha += L[2 * IVFR_KS + ((wa >> 16) & 0xff)];
                hb += L[2 * IVFR_KS + ((wb >> 16) & 0xff)];
                ha += L[3 * IVFR_KS + (wa >> 24)];
                hb += L[3 * IVFR_KS + (wb >> 24)];
            }
            const short4v da = tshi - __builtin_bit_cast(short4v, ha), db = tshi - __builtin_bit_cast(short4v, hb);
            const uint2 ua = __builtin_bit_cast(uint2, da), ub = __builtin_bit_cast(uint2, db);
            const bool none0 = !in0[v] || ((ua.x & ua.y & 0x80008000u) == 0x80008000u);
            const bool none1 = !in1[v] || ((ub.x & ub.y & 0x80008000u) == 0x80008000u);
            if (__ballot(!(none0 && none1)) == 0) continue;
            // bit x: the difference of query x is not negative
            const uint32_t m0 = none0 ? 0u : (~(((ua.x >> 15) & 1u) | ((ua.x >> 30) & 2u) | ((ua.y >> 13) & 4u) | ((ua.y >> 28) & 8u)) & 0xfu);
            const uint32_t m1 = none1 ? 0u : (~(((ub.x >> 15) & 1u) | ((ub.x >> 30) & 2u) | ((ub.y >> 13) & 4u) | ((ub.y >> 28) & 8u)) & 0xfu);
            const uint64_t b0 = __ballot(m0 != 0), b1 = __ballot(m1 != 0);
            const uint64_t below = (1ull << lane) - 1ull;
            const uint32_t n0 = __popcll(b0);
            if (m0) {
                const uint32_t slot = wq.n + __popcll(b0 & below);
                wq.est[slot] = e0[v];
                wq.pos[slot] = m0;
            }
            if (m1) {
                const uint32_t slot = wq.n + n0 + __popcll(b1 & below);
                wq.est[slot] = e0[v] + 1;
                wq.pos[slot] = m1;
            }
            wq.n += n0 + __popcll(b1);
            if (wq.n > WQ_CAP - 128) drain();
        }
    }
    drain();
}

template <int M, int G>
__global__ __launch_bounds__(256) void adc_scan_shared_kernel(const uint8_t* __restrict__ codes,
                                                              TableSrc ts,
                                                              const uint32_t* __restrict__ pair_start,
                                                              const uint32_t* __restrict__ pair_len,
                                                              const uint32_t* __restrict__ blkpre,
                                                              const uint32_t* __restrict__ unit_pairs, int n_host,
                                                              const uint32_t* __restrict__ n_dev, uint32_t bpg,
                                                              uint32_t g_min,
                                                              int w, const float* __restrict__ tau,
                                                              uint2* __restrict__ cand,
                                                              uint32_t* __restrict__ cand_cnt, CandLayout lay,
                                                              const float* __restrict__ lut_scale,
                                                              const uint8_t* __restrict__ exact_only,
                                                              DirectPlace direct) {
    typedef typename LutVec<G>::type vec_t;
    extern __shared__ float s_raw[];
    vec_t* s_lutv = reinterpret_cast<vec_t*>(s_raw);   // [M * 256] vectors: component x = query x of the unit
    WaveQueue wq;                                      // behind the tables: the wavefronts' append queues
    wq.est = reinterpret_cast<uint32_t*>(s_raw) + M * IVFR_KS * G + (threadIdx.x >> 6) * WQ_WORDS;
    wq.pos = wq.est + WQ_CAP;
    wq.tag = wq.pos + WQ_CAP;
    wq.n = 0;
    const int nunits = n_dev ? (int)*n_dev : n_host;
    uint32_t b, b_end;
    if (nunits <= 0 || !scan_share(blkpre, nunits, bpg, g_min, 1u, 0u, b, b_end)) return;
    int lo = 0, hi = nunits;   // last unit u with blkpre[u] <= b
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (blkpre[mid] <= b) lo = mid; else hi = mid;
    }
    int u = lo;
    const int tid = threadIdx.x;
    while (b < b_end) {
        while (blkpre[u + 1] <= b) ++u;
        const uint32_t pb0 = blkpre[u], pb1 = blkpre[u + 1];
        const uint32_t stop = pb1 < b_end ? pb1 : b_end;
        int64_t pid[G];
        PairTable pt[G];
        float t[G];
        uint2* qc[G];
        uint32_t* cnt[G];
        uint32_t cap[G];
        bool placed[G];      // the query keeps everything and every entry has its own place in its buffer
        uint32_t place0[G];
#pragma unroll
        for (int x = 0; x < G; ++x) {
            const uint32_t raw = unit_pairs[(int64_t)u * G + x];
            const bool real = raw != IVFR_NO_PAIR;
            pid[x] = real ? (int64_t)raw : (int64_t)unit_pairs[(int64_t)u * G];   // an empty slot reads slot 0's table
            pt[x] = ts.pair(pid[x]);
            const int q = (int)(pid[x] / w);
            t[x] = real ? tau[q] : -1.f;                                         // ... and never keeps anything
            placed[x] = real && direct.fully && direct.fully[q];
            place0[x] = placed[x] ? direct.off[pid[x]] : 0u;
            qc[x] = cand + lay.base(q);
            cap[x] = lay.cap(q);
            cnt[x] = cand_cnt + q;
        }
        const uint32_t start = pair_start[pid[0]], len = pair_len[pid[0]];   // the unit's pairs share the list
        // A unit of four whose queries all pass only a small share of their estimates runs on half-precision
        // tables with an exact re-evaluation of the few candidates, like the units of eight (see below).
        bool half_unit = false;
        if (G == 4 && exact_only != nullptr) {
            half_unit = true;
#pragma unroll
            for (int x = 0; x < G; ++x)
                if (unit_pairs[(int64_t)u * G + x] != IVFR_NO_PAIR && exact_only[(int)(pid[x] / w)]) half_unit = false;
        }
        __syncthreads();   // previous unit's tables no longer in use
        if constexpr (G == 4) {
            if (half_unit) {
                half_unit_pass<M>(codes, pt, lut_scale, unit_pairs + (int64_t)u * G, pid, t, qc, cnt, cap, start, len, b,
                                  stop, pb0, s_raw, wq);
                b = stop;
                continue;
            }
        }
        for (int e = tid; e < M * IVFR_KS; e += 256) {
            float v[G];
            unit_table_entries<G>(pt, e, v);
            vec_t packed;
            vload(packed, v);
            s_lutv[e] = packed;
        }
        __syncthreads();
        for (uint32_t bb = b; bb < stop; bb += 2) {
            uint32_t wds[2][2][M / 4];
            uint32_t e0[2];
            bool in0[2], in1[2];
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                e0[v] = (bb + v - pb0) * IVFR_BLOCK + 2u * tid;
                in0[v] = bb + v < stop && e0[v] < len;
                in1[v] = bb + v < stop && e0[v] + 1 < len;
                if (in0[v]) {
                    const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + e0[v]) * M);
                    if (M == 8) {
                        uint4 c4 = *reinterpret_cast<const uint4*>(src);
                        wds[v][0][0] = c4.x; wds[v][0][1] = c4.y; wds[v][1][0] = c4.z; wds[v][1][1] = c4.w;
                    } else {
#pragma unroll
                        for (int t2 = 0; t2 < M / 4; ++t2) { wds[v][0][t2] = src[t2]; wds[v][1][t2] = src[M / 4 + t2]; }
                    }
                } else {
#pragma unroll
                    for (int t2 = 0; t2 < M / 4; ++t2) { wds[v][0][t2] = 0; wds[v][1][t2] = 0; }
                }
            }
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                // per query the same two partial sums as adc_sum<M>: even and odd sub-quantizers
                vec_t a0, a1, b0, b1;
                vzero(a0); vzero(a1); vzero(b0); vzero(b1);
#pragma unroll
                for (int t2 = 0; t2 < M / 4; ++t2) {
                    const uint32_t wa = wds[v][0][t2], wb = wds[v][1][t2];
                    const vec_t* L = s_lutv + t2 * 4 * IVFR_KS;
                    vadd(a0, L[wa & 0xff]);
                    vadd(a1, L[IVFR_KS + ((wa >> 8) & 0xff)]);
                    vadd(a0, L[2 * IVFR_KS + ((wa >> 16) & 0xff)]);
                    vadd(a1, L[3 * IVFR_KS + (wa >> 24)]);
                    vadd(b0, L[wb & 0xff]);
                    vadd(b1, L[IVFR_KS + ((wb >> 8) & 0xff)]);
                    vadd(b0, L[2 * IVFR_KS + ((wb >> 16) & 0xff)]);
                    vadd(b1, L[3 * IVFR_KS + (wb >> 24)]);
                }
#pragma unroll
                for (int x = 0; x < G; ++x) {
                    const float ea = vget(a0, x) + vget(a1, x), eb = vget(b0, x) + vget(b1, x);
                    if (placed[x]) {
                        const uint32_t s0 = place0[x] + e0[v];
                        if (in0[v] && s0 < cap[x]) qc[x][s0] = make_uint2(__float_as_uint(ea), start + e0[v]);
                        if (in1[v] && s0 + 1 < cap[x]) qc[x][s0 + 1] = make_uint2(__float_as_uint(eb), start + e0[v] + 1);
                    } else if (t[x] == INFINITY) {   // nothing is filtered for this query: one atomic per pass
                        append_records(in0[v], ea, start + e0[v], in1[v], eb, start + e0[v] + 1, qc[x], cnt[x], cap[x]);
                    } else {
                        if (wq.n > WQ_CAP - 128) wq_flush<G>(wq, qc, cnt, cap);
                        wq_push(wq, in0[v] && ea <= t[x], ea, start + e0[v], in1[v] && eb <= t[x], eb,
                                start + e0[v] + 1, (uint32_t)x);
                    }
                }
            }
        }
        wq_flush<G>(wq, qc, cnt, cap);   // the queue refers to this unit's queries
        b = stop;
    }
}

template <int M, int G>
static size_t shared_lds_bytes() { return (size_t)(M * IVFR_KS * G + 4 * WQ_WORDS) * sizeof(float); }

template <int M, int G>
static int launch_shared_mg(const ivfr_index* ix, const TableSrc& ts, const uint32_t* pair_start,
                            const uint32_t* pair_len, const uint32_t* blkpre, const uint32_t* unit_pairs,
                            const ScanShape& sh, int w, const float* tau, uint2* cand, uint32_t* cand_cnt,
                            CandLayout lay, hipStream_t st, const float* lut_scale, const uint8_t* exact_only,
                            DirectPlace direct) {
    hipLaunchKernelGGL((adc_scan_shared_kernel<M, G>), dim3(sh.groups), dim3(256), (shared_lds_bytes<M, G>()), st,
                       ix->codes, ts, pair_start, pair_len, blkpre, unit_pairs, sh.n_host, sh.n_dev, sh.bpg, sh.g_min,
                       w, tau, cand, cand_cnt, lay, lut_scale, exact_only, direct);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

bool ivfr_shared_scan_supported(const ivfr_index* ix) { return ix->p.m <= 16; }

int ivfr_launch_scan_shared(const ivfr_index* ix, int G, const TableSrc& ts, const uint32_t* pair_start,
                            const uint32_t* pair_len, const uint32_t* blkpre, const uint32_t* unit_pairs,
                            ScanShape sh, int w, const float* tau, uint2* cand, uint32_t* cand_cnt, CandLayout lay,
                            hipStream_t st, const float* lut_scale, const uint8_t* exact_only, DirectPlace direct) {
    if (!sh.n_dev && sh.n_host <= 0) return IVFR_OK;
#define IVFR_SH_ARGS \
    ix, ts, pair_start, pair_len, blkpre, unit_pairs, sh, w, tau, cand, cand_cnt, lay, st, lut_scale, exact_only, direct
    if (G == 4) {
        switch (ix->p.m) {
            case 4: return launch_shared_mg<4, 4>(IVFR_SH_ARGS);
            case 8: return launch_shared_mg<8, 4>(IVFR_SH_ARGS);
            case 16: return launch_shared_mg<16, 4>(IVFR_SH_ARGS);
        }
    } else if (G == 2) {
        switch (ix->p.m) {
            case 4: return launch_shared_mg<4, 2>(IVFR_SH_ARGS);
            case 8: return launch_shared_mg<8, 2>(IVFR_SH_ARGS);
            case 16: return launch_shared_mg<16, 2>(IVFR_SH_ARGS);
        }
    }
#undef IVFR_SH_ARGS
    ivfr_set_error("shared scan supports m <= 16 and units of 2 or 4; got m = %d, unit %d", ix->p.m, G);
    return IVFR_ERR_INVALID_ARG;
}

// ------------------------------------------------------------------------------------------
// Shared scan of eight queries with half-precision tables and an exact re-evaluation.
//
// LDS read bandwidth bounds the shared scan, so the tables of a unit of eight are kept as fp16:
// one 16-byte LDS read then serves eight queries.  Table x is scaled by s_x (chosen so that no
// sum of m entries can overflow fp16) and the m entries are added in packed fp16.  All terms
// are non-negative, so the result H satisfies H <= s_x E (1 + 2^-11)^m + m 2^-14 for the fp32
// estimate E (one rounding per table entry, one per add; an entry below the smallest normal
// 2^-14 may round up to it or be flushed to zero).
// An entry can only belong to the short-list if E <= tau, hence only if
//     H <= s_x tau (1 + (m + 1.2) 2^-11) + 4e-3     (1.0045 at m = 8, 1.0084 at m = 16),
// and exactly those few (a fraction of a percent of the scanned entries) are re-evaluated in
// fp32 from the query's table in global memory, with the same summation order as everywhere
// else; only that exact value is compared with tau and recorded.  The records, and therefore
// the search results, are bit-identical to the fp32 kernels' (tested).
// The candidates are not re-evaluated where they are found (every second or third pass of the
// scan loop has one somewhere in the wavefront, and its global reads and atomic would stall
// all 64 lanes): a wavefront queues them in LDS as (entry, query mask) and works the queue off
// when it is full or the unit ends, one candidate per lane, so the latencies overlap.
// ------------------------------------------------------------------------------------------
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef short short8 __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------------
// Sample pass: the first len_s[p] entries of every pair, all estimates kept (the values only), each at its own place
// in the query's buffer (the plan's prefix sums give the place, no counter is touched).  The prefixes are
// short (a few hundred entries, a few chunks of IVFR_SAMPLE_CHUNK for the longest lists) and there
// are tens of thousands of pairs, so the work is table loads and latency: a small workgroup (two wavefronts
// at m <= 16) per chunk shares one table, so that a compute unit keeps sixteen independent chunks and all of its
// 32 wavefronts in flight, and a chunk is half as many steps long as with one wavefront.
// ------------------------------------------------------------------------------------------
template <int M, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void adc_sample_kernel(const uint8_t* __restrict__ codes,
                                                                TableSrc ts,
                                                                const uint32_t* __restrict__ pair_start,
                                                                const uint32_t* __restrict__ len_s,
                                                                const uint32_t* __restrict__ chunk_pre,
                                                                const uint32_t* __restrict__ items,
                                                                const uint32_t* __restrict__ n_items_dev,
                                                                const uint32_t* __restrict__ soff, int w,
                                                                uint2* __restrict__ cand, CandLayout lay) {
    extern __shared__ float s_lut[];   // one table of M * 256 floats, shared by the workgroup's WAVES wavefronts
    const int tid = threadIdx.x;
    const uint32_t n_items = *n_items_dev;
    float* T = s_lut;
    // the workgroup walks over the chunks (item is uniform over it: every barrier is reached by all its threads)
    for (uint32_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const uint32_t p = items[item];
        const uint32_t first = (item - chunk_pre[p]) * IVFR_SAMPLE_CHUNK;
        const uint32_t n = len_s[p];
        const uint32_t last = n - first < IVFR_SAMPLE_CHUNK ? n : first + IVFR_SAMPLE_CHUNK;   // exclusive
        __syncthreads();   // the previous chunk's table is no longer read
        {
            const PairTable pt = ts.pair((int64_t)p);
            float4* dst = reinterpret_cast<float4*>(T);
            for (int i = tid; i < M * IVFR_KS / 4; i += 64 * WAVES) dst[i] = pt.get4(4 * i);
        }
        __syncthreads();
        const uint32_t start = pair_start[p];
        const int q = (int)(p / (uint32_t)w);
        // bare estimates: the buffer (records of 8 bytes) holds at least the query's whole sample
        float* out = reinterpret_cast<float*>(cand + lay.base(q)) + soff[p];
        for (uint32_t e = first + 2u * tid; e < last; e += 128u * WAVES) {
            uint32_t w0[M / 4], w1[M / 4];
            load_code_pair<M>(codes, start, e, true, last, w0, w1);
            out[e] = adc_sum<M>(T, w0);
            if (e + 1 < last) out[e + 1] = adc_sum<M>(T, w1);
        }
    }
}

template <int M, int WAVES>
static size_t sample_lds_bytes() { return (size_t)M * IVFR_KS * sizeof(float); }

template <int M, int WAVES>
static int launch_sample_m(const ivfr_index* ix, const TableSrc& ts, const uint32_t* pair_start, const uint32_t* len_s,
                           const uint32_t* chunk_pre, const uint32_t* items, const uint32_t* n_items, size_t max_items,
                           const uint32_t* soff, int w, uint2* cand, CandLayout lay, hipStream_t st) {
    const size_t lds = sample_lds_bytes<M, WAVES>();
    // four times the workgroups that a compute unit holds at once (its LDS or its 32 wavefronts), or one workgroup per
    // chunk when there are fewer
    const size_t per_cu = std::max<size_t>(1, std::min<size_t>((size_t)(160 * 1024) / lds, (size_t)32 / WAVES));
    const size_t grid = std::max<size_t>(1, std::min(max_items, (size_t)ix->n_cu * per_cu * 4));
    hipLaunchKernelGGL((adc_sample_kernel<M, WAVES>), dim3((unsigned)grid), dim3(64 * WAVES), lds, st, ix->codes, ts,
                       pair_start, len_s, chunk_pre, items, n_items, soff, w, cand, lay);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

int ivfr_launch_sample_scan(const ivfr_index* ix, const TableSrc& ts, const uint32_t* pair_start, const uint32_t* len_s,
                            const uint32_t* chunk_pre, const uint32_t* items, const uint32_t* n_items, size_t max_items,
                            const uint32_t* soff, int w, uint2* cand, CandLayout lay, hipStream_t st) {
    if (max_items == 0) return IVFR_OK;
#define IVFR_SAMPLE_ARGS ix, ts, pair_start, len_s, chunk_pre, items, n_items, max_items, soff, w, cand, lay, st
    switch (ix->p.m) {
        case 4: return launch_sample_m<4, 2>(IVFR_SAMPLE_ARGS);
        case 8: return launch_sample_m<8, 2>(IVFR_SAMPLE_ARGS);
        case 16: return launch_sample_m<16, 2>(IVFR_SAMPLE_ARGS);
        case 32: return launch_sample_m<32, 4>(IVFR_SAMPLE_ARGS);
        case 64: return launch_sample_m<64, 4>(IVFR_SAMPLE_ARGS);
        default:
            ivfr_set_error("list scan supports m in {4, 8, 16, 32, 64}; got %d", ix->p.m);
            return IVFR_ERR_INVALID_ARG;
    }
#undef IVFR_SAMPLE_ARGS
}

// Threads per workgroup of the half-precision scan of eight: eight wavefronts share one 32 KB set of tables,
// three workgroups (24 wavefronts) fit a compute unit; measured best against 256 and 1024.
#define H8_T 512
#define Q8H_CAP 192   // queued candidates per wavefront (two LDS words each)

// bit x set when 16-bit lane x of the four words is not negative (lane 0 = low half of u.x)
__device__ __forceinline__ uint32_t sign_free_mask(uint4 u) {
    const uint32_t neg = ((u.x >> 15) & 1u) | ((u.x >> 30) & 2u) | ((u.y >> 13) & 4u) | ((u.y >> 28) & 8u) |
                         ((u.z >> 11) & 16u) | ((u.z >> 26) & 32u) | ((u.w >> 9) & 64u) | ((u.w >> 24) & 128u);
    return ~neg & 0xffu;
}

template <int M>
__global__ __launch_bounds__(H8_T) void adc_scan_shared8h_kernel(const uint8_t* __restrict__ codes,
                                                                TableSrc ts,
                                                                const float* __restrict__ lut_scale,
                                                                const uint32_t* __restrict__ pair_start,
                                                                const uint32_t* __restrict__ pair_len,
                                                                const uint32_t* __restrict__ blkpre,
                                                                const uint32_t* __restrict__ unit_pairs, int n_host,
                                                                const uint32_t* __restrict__ n_dev, uint32_t bpg,
                                                                uint32_t g_min,
                                                                int w, const float* __restrict__ tau,
                                                                uint2* __restrict__ cand,
                                                                uint32_t* __restrict__ cand_cnt, CandLayout lay) {
    extern __shared__ float s_raw[];
    half8* s_lut8 = reinterpret_cast<half8*>(s_raw);   // [M * 256] x 8 halves: component x = query x of the unit
    // behind the tables: per wavefront a queue of Q8H_CAP (entry, query mask) candidates, then the unit's pairs and bounds
    uint32_t* q_entry = reinterpret_cast<uint32_t*>(s_raw) + M * IVFR_KS * 4 + (threadIdx.x >> 6) * (2 * Q8H_CAP);
    uint32_t* q_mask = q_entry + Q8H_CAP;
    uint32_t* s_pid = reinterpret_cast<uint32_t*>(s_raw) + M * IVFR_KS * 4 + (H8_T / 64) * (2 * Q8H_CAP);
    float* s_tau = reinterpret_cast<float*>(s_pid + 8);
    const int nunits = n_dev ? (int)*n_dev : n_host;
    uint32_t b, b_end;
    if (nunits <= 0 || !scan_share(blkpre, nunits, bpg, g_min, 1u, 0u, b, b_end)) return;
    int lo = 0, hi = nunits;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (blkpre[mid] <= b) lo = mid; else hi = mid;
    }
    int u = lo;
    const int tid = threadIdx.x, lane = tid & 63;
    // Table entry (j, byte) lives at [byte][j], and lane l looks its code's sub-quantizers up in the order
    // l, l + 1, ... (mod M): the lanes of a wavefront that the LDS serves together (eight consecutive ones for
    // 16-byte reads) then always read different j, hence different banks whatever the code bytes are.  Random
    // 16-byte gathers cost 12.7 cycles per wavefront read, these 8.6 (8 is the LDS rate).
    const uint32_t rot = (uint32_t)lane & (M - 1);
    const char* s_lut_bytes = reinterpret_cast<const char*>(s_lut8);
    uint32_t joff[M];
#pragma unroll
    for (int s2 = 0; s2 < M; ++s2) joff[s2] = ((rot + (uint32_t)s2) & (M - 1)) * 16u;
    uint32_t qn = 0;   // candidates queued by this wavefront (uniform over its lanes)
    uint32_t start = 0;
    // Exact fp32 re-evaluation of the queued candidates, one per lane: every lane works on its own
    // (entry, query) combinations, so the table reads of a whole queue overlap.  What is kept is appended with
    // one atomic per query and round (the lanes that keep something for the same query share it): the counters
    // of a batch sit in a few cache lines, and an atomic per record would queue up behind them.
    auto drain = [&]() {
        for (uint32_t base = 0; base < qn; base += 64) {
            const uint32_t i = base + lane;
            uint32_t e = 0, mask = 0;
            uint32_t wd[M / 4];
#pragma unroll
            for (int t2 = 0; t2 < M / 4; ++t2) wd[t2] = 0;
            if (i < qn) {
                e = q_entry[i];
                mask = q_mask[i];
                const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + e) * M);
#pragma unroll
                for (int t2 = 0; t2 < M / 4; ++t2) wd[t2] = src[t2];
            }
            while (__ballot(mask != 0) != 0) {   // one query per lane and round
                int x = -1;
                float est = 0.f;
                bool keep = false;
                if (mask) {
                    x = __ffs(mask) - 1;
                    mask &= mask - 1;
                    est = adc_sum_pair<M>(ts.pair((int64_t)s_pid[x]), wd);
                    keep = est <= s_tau[x];
                }
                uint64_t todo = __ballot(keep);
                while (todo) {   // one round per query that has records in this wavefront
                    const int leader = __ffsll((long long)todo) - 1;
                    const int xl = __builtin_amdgcn_readlane(x, leader);
                    const uint64_t same = __ballot(keep && x == xl);
                    const int q = (int)(s_pid[xl] / (uint32_t)w);
                    uint32_t first = 0;
                    if (lane == leader) first = atomicAdd(cand_cnt + q, (uint32_t)__popcll(same));
                    first = __builtin_amdgcn_readlane(first, leader);
                    if (keep && x == xl) {
                        const uint32_t slot = first + __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
                        if (slot < lay.cap(q)) cand[lay.base(q) + slot] = make_uint2(__float_as_uint(est), start + e);
                    }
                    todo &= ~same;
                }
            }
        }
        qn = 0;
    };
    while (b < b_end) {
        while (blkpre[u + 1] <= b) ++u;
        const uint32_t pb0 = blkpre[u], pb1 = blkpre[u + 1];
        const uint32_t stop = pb1 < b_end ? pb1 : b_end;
        int64_t pid[8];
        PairTable pt[8];
        float t[8], tsc[8], sc[8];
        half8 tsh;   // the thresholds in half precision, rounded up (bit pattern 0xFFFF for an empty slot)
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const uint32_t raw = unit_pairs[(int64_t)u * 8 + x];
            const bool real = raw != IVFR_NO_PAIR;
            pid[x] = real ? (int64_t)raw : (int64_t)unit_pairs[(int64_t)u * 8];
            pt[x] = ts.pair(pid[x]);
            sc[x] = lut_scale[pid[x]];
            t[x] = real ? tau[(int)(pid[x] / w)] : -1.f;
            tsc[x] = real ? t[x] * sc[x] * (1.f + (M + 1.2f) * 4.8828125e-4f) + 4e-3f : -1.f;
            tsh[x] = (_Float16)(real ? tsc[x] * 1.001f + 1e-4f : 0.f);   // 2^-10 > the 2^-11 of the conversion
        }
        short8 tshi = __builtin_bit_cast(short8, tsh);
#pragma unroll
        for (int x = 0; x < 8; ++x)
            if (unit_pairs[(int64_t)u * 8 + x] == IVFR_NO_PAIR) tshi[x] = (short)-1;
        start = pair_start[pid[0]];
        const uint32_t len = pair_len[pid[0]];
        __syncthreads();   // every wavefront has drained its queue and left the previous unit's tables
        if (tid < 8) {
            const uint32_t raw = unit_pairs[(int64_t)u * 8 + tid];
            s_pid[tid] = raw != IVFR_NO_PAIR ? raw : unit_pairs[(int64_t)u * 8];
            s_tau[tid] = raw != IVFR_NO_PAIR ? tau[(int)(raw / (uint32_t)w)] : -1.f;
        }
        for (int e = tid; e < M * IVFR_KS; e += H8_T) {   // e = j * 256 + byte; stored at [byte][j]
            half8 h;
            float v[8];
            unit_table_entries<8>(pt, e, v);
#pragma unroll
            for (int x = 0; x < 8; ++x) h[x] = (_Float16)(v[x] * sc[x]);
            s_lut8[(e & (IVFR_KS - 1)) * M + (e >> 8)] = h;
        }
        __syncthreads();
        constexpr uint32_t BPV = H8_T / 256;   // blocks covered by the workgroup per v
        for (uint32_t bb = b; bb < stop; bb += 2 * BPV) {
            uint32_t wds[2][2][M / 4];
            uint32_t e0[2];
            bool in0[2], in1[2];
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const uint32_t blk = bb + v * BPV + (uint32_t)(tid >> 8);
                e0[v] = (blk - pb0) * IVFR_BLOCK + 2u * (uint32_t)(tid & 255);
                in0[v] = blk < stop && e0[v] < len;
                in1[v] = blk < stop && e0[v] + 1 < len;
                load_code_pair<M>(codes, start, e0[v], blk < stop, len, wds[v][0], wds[v][1]);
            }
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                half8 ha, hb;
                rotate_code_bytes<M>(wds[v][0], rot);
                rotate_code_bytes<M>(wds[v][1], rot);
#pragma unroll
                for (int s2 = 0; s2 < M; ++s2) {
                    const uint32_t ba = (wds[v][0][s2 / 4] >> (8 * (s2 % 4))) & 0xffu;
                    const uint32_t bb = (wds[v][1][s2 / 4] >> (8 * (s2 % 4))) & 0xffu;
                    const half8 xa = *reinterpret_cast<const half8*>(s_lut_bytes + ba * (M * 16) + joff[s2]);
                    const half8 xb = *reinterpret_cast<const half8*>(s_lut_bytes + bb * (M * 16) + joff[s2]);
                    if (s2 == 0) { ha = xa; hb = xb; }
                    else { ha += xa; hb += xb; }
                }
                // fast reject: sums and thresholds are non-negative, so their fp16 bit patterns order like
                // 16-bit integers; threshold minus sum in packed int16 is negative in all eight lanes of both
                // codes when no query can keep either entry (an empty slot's -1 minus a sum is always negative)
                const short8 da = tshi - __builtin_bit_cast(short8, ha), db = tshi - __builtin_bit_cast(short8, hb);
                const uint4 ua = __builtin_bit_cast(uint4, da), ub = __builtin_bit_cast(uint4, db);
                const bool none0 = !in0[v] || ((ua.x & ua.y & ua.z & ua.w & 0x80008000u) == 0x80008000u);
                const bool none1 = !in1[v] || ((ub.x & ub.y & ub.z & ub.w & 0x80008000u) == 0x80008000u);
                if (__ballot(!(none0 && none1)) == 0) continue;
                // bit x of the mask: query x may keep the entry (its difference is not negative)
                const uint32_t m0 = none0 ? 0u : sign_free_mask(ua), m1 = none1 ? 0u : sign_free_mask(ub);
                const uint64_t b0 = __ballot(m0 != 0), b1 = __ballot(m1 != 0);
                const uint64_t below = (1ull << lane) - 1ull;
                const uint32_t n0 = __popcll(b0);
                if (m0) {
                    const uint32_t slot = qn + __popcll(b0 & below);
                    q_entry[slot] = e0[v];
                    q_mask[slot] = m0;
                }
                if (m1) {
                    const uint32_t slot = qn + n0 + __popcll(b1 & below);
                    q_entry[slot] = e0[v] + 1;
                    q_mask[slot] = m1;
                }
                qn += n0 + __popcll(b1);
                if (qn > Q8H_CAP - 128) drain();   // room for the next 64 x 2 entries
            }
        }
        drain();   // the queue refers to this unit's pairs
        b = stop;
    }
}

template <int M>
static size_t shared8h_lds_bytes() {
    return (size_t)M * IVFR_KS * 16 + (H8_T / 64) * 2 * Q8H_CAP * sizeof(uint32_t) + 16 * sizeof(uint32_t);
}

template <int M>
static int launch_shared8h_m(const ivfr_index* ix, const TableSrc& ts, const float* lut_scale,
                             const uint32_t* pair_start, const uint32_t* pair_len, const uint32_t* blkpre,
                             const uint32_t* unit_pairs, const ScanShape& sh, int w, const float* tau, uint2* cand,
                             uint32_t* cand_cnt, CandLayout lay, hipStream_t st) {
    hipLaunchKernelGGL(adc_scan_shared8h_kernel<M>, dim3(sh.groups), dim3(H8_T), shared8h_lds_bytes<M>(), st, ix->codes,
                       ts, lut_scale, pair_start, pair_len, blkpre, unit_pairs, sh.n_host, sh.n_dev, sh.bpg, sh.g_min,
                       w, tau, cand, cand_cnt, lay);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

bool ivfr_shared8h_supported(const ivfr_index* ix) { return ix->p.m <= 16; }

int ivfr_launch_scan_shared8h(const ivfr_index* ix, const TableSrc& ts, const float* lut_scale,
                              const uint32_t* pair_start, const uint32_t* pair_len, const uint32_t* blkpre,
                              const uint32_t* unit_pairs, ScanShape sh, int w, const float* tau, uint2* cand,
                              uint32_t* cand_cnt, CandLayout lay, hipStream_t st) {
    if (!sh.n_dev && sh.n_host <= 0) return IVFR_OK;
    switch (ix->p.m) {
        case 4: return launch_shared8h_m<4>(ix, ts, lut_scale, pair_start, pair_len, blkpre, unit_pairs, sh, w, tau, cand, cand_cnt, lay, st);
        case 8: return launch_shared8h_m<8>(ix, ts, lut_scale, pair_start, pair_len, blkpre, unit_pairs, sh, w, tau, cand, cand_cnt, lay, st);
        case 16: return launch_shared8h_m<16>(ix, ts, lut_scale, pair_start, pair_len, blkpre, unit_pairs, sh, w, tau, cand, cand_cnt, lay, st);
        default:
            ivfr_set_error("half-precision shared scan supports m <= 16; got %d", ix->p.m);
            return IVFR_ERR_INVALID_ARG;
    }
}

// ------------------------------------------------------------------------------------------
// Matrix-core scan for lists that 64 queries of the batch visit together.
//
// With that many queries on one list the estimate of Eq. (5) is cheaper as a contraction than as table
// look-ups: for query residual r and the entry's decoded vector y = (pq[0][b_0], ..., pq[m-1][b_{m-1}])
//     estimate = ||r||^2 - 2 r . y + ||y||^2 ,
// so a tile of 32 entries against 64 queries is a [64 x d] . [d x 32] product.  The decoded vectors are
// gathered, 16 bytes per lane and 16-dimension step, from one fp16 copy of the PQ codebook that stays in LDS for
// the whole launch (it depends on neither list nor query, so nothing is rebuilt between units); the queries'
// -2 r, in fp16, stay in registers; v_mfma_f32_32x32x16_f16 accumulates in fp32 on top of a per-query constant
//     c0 = S (||r||^2 - tau) - margin,
// and an entry can be kept by query x only if c0[x] + (product) + S ||y||^2 <= 0 (S: the power-of-two scale
// that brings both fp16 operands into range).  The margin bounds every rounding of this filter against the fp32
// table sum, so nothing the exact test would keep is dropped: fp16 rounding of both operands changes
// the product by at most 2^-10 sum_j 2 ||r^j|| max_k ||pq[j][k]||, the tables themselves and the fp32 sums are
// accurate to a few 2^-22 of sum_j (||r^j|| + max_k ||pq[j][k]||)^2.  Whatever passes is queued per wavefront
// and re-evaluated exactly like in the half-precision scan of eight: the same fp32 sum of the same table
// entries, compared with tau, appended to the query's buffer.  Wavefronts work independently (no barrier after
// the codebook is staged); each takes an equal share of the launch's block stream.
// ------------------------------------------------------------------------------------------
#define MF_T 512      // threads per workgroup: eight wavefronts share the LDS codebook, one workgroup per CU
#define MF_ROWS 64    // queries per unit
#define MFQ_CAP 128   // queued candidates per wavefront; a tile adds at most 64

template <int M, int DSUB>
__global__ __launch_bounds__(MF_T) void adc_scan_mfma64_kernel(const uint8_t* __restrict__ codes,
                                                              const float* __restrict__ queries,
                                                              const int32_t* __restrict__ probe,
                                                              const float* __restrict__ coarse,
                                                              const float* __restrict__ pq,
                                                              const float* __restrict__ pq_norm,
                                                              const float* __restrict__ pq_maxnorm,
                                                              TableSrc ts,
                                                              const float* __restrict__ lut_scale,
                                                              const uint32_t* __restrict__ pair_start,
                                                              const uint32_t* __restrict__ pair_len,
                                                              const uint32_t* __restrict__ blkpre,
                                                              const uint32_t* __restrict__ unit_pairs, int n_host,
                                                              const uint32_t* __restrict__ n_dev, uint32_t bpg,
                                                              uint32_t g_min,
                                                              int w, const float* __restrict__ tau,
                                                              uint2* __restrict__ cand,
                                                              uint32_t* __restrict__ cand_cnt, CandLayout lay) {
    constexpr int D = M * DSUB;          // dimensions
    constexpr int KSTEPS = D / 16;       // matrix instructions per tile and 32 queries
    constexpr int CENT_BYTES = IVFR_KS * D * 2;
    constexpr int WAVE_WORDS = 2 * MFQ_CAP + 3 * MF_ROWS;
    extern __shared__ float s_raw[];
    char* s_cent = reinterpret_cast<char*>(s_raw);                                  // fp16 [M][256][DSUB], scaled
    float* s_norm = reinterpret_cast<float*>(s_cent + CENT_BYTES);                  // [M][256] ||pq[j][k]||^2
    uint32_t* s_wave = reinterpret_cast<uint32_t*>(s_norm + M * IVFR_KS) + (threadIdx.x >> 6) * WAVE_WORDS;
    uint32_t* q_entry = s_wave;                  // entry | (lane half << 31)
    uint32_t* q_mask = s_wave + MFQ_CAP;         // bit rb*16 + i: accumulator i of query block rb passed
    uint32_t* s_pid = s_wave + 2 * MFQ_CAP;      // [64] pair of every row
    float* s_tau = reinterpret_cast<float*>(s_pid + MF_ROWS);
    float* s_c0 = s_tau + MF_ROWS;
    const int tid = threadIdx.x, lane = tid & 63, row = lane & 31, h = lane >> 5;

    const int nunits = n_dev ? (int)*n_dev : n_host;   // uniform over the workgroup: no unit, no work, no barrier
    if (nunits <= 0 || blkpre[nunits] == blkpre[0]) return;
    // codebook scale: a power of two that brings the largest component below 128
    float cmax = 0.f, nmax = 0.f;
#pragma unroll
    for (int j = 0; j < M; ++j) { const float v = pq_maxnorm[j]; cmax = fmaxf(cmax, v); nmax = fmaf(v, v, nmax); }
    int ce = 0;
    if (cmax > 0.f) (void)frexpf(cmax, &ce);
    const float s_c = cmax > 0.f ? ldexpf(1.f, 7 - ce) : 1.f;
    for (int i = tid; i < IVFR_KS * D / 8; i += MF_T) {
        const float4 v0 = *reinterpret_cast<const float4*>(pq + (int64_t)i * 8);
        const float4 v1 = *reinterpret_cast<const float4*>(pq + (int64_t)i * 8 + 4);
        half8 hv;
        hv[0] = (_Float16)(v0.x * s_c); hv[1] = (_Float16)(v0.y * s_c); hv[2] = (_Float16)(v0.z * s_c); hv[3] = (_Float16)(v0.w * s_c);
        hv[4] = (_Float16)(v1.x * s_c); hv[5] = (_Float16)(v1.y * s_c); hv[6] = (_Float16)(v1.z * s_c); hv[7] = (_Float16)(v1.w * s_c);
        reinterpret_cast<half8*>(s_cent)[i] = hv;
    }
    for (int i = tid; i < M * IVFR_KS; i += MF_T) s_norm[i] = pq_norm[i];
    __syncthreads();   // the only barrier: from here on every wavefront works alone

    uint32_t b, b_end;
    if (!scan_share(blkpre, nunits, bpg, g_min, MF_T / 64, (uint32_t)(tid >> 6), b, b_end)) return;
    int lo = 0, hi = nunits;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (blkpre[mid] <= b) lo = mid; else hi = mid;
    }
    int u = lo;
    uint32_t qn = 0, start = 0;
    // per-lane parts of the LDS addresses
    const uint32_t cent_lane = DSUB == 8 ? (uint32_t)h * (IVFR_KS * 16) : (uint32_t)h * 16;
    const uint32_t norm_lane = (uint32_t)h * (M / 2) * (IVFR_KS * 4);
    const uint32_t hmask = h ? 0xffffffffu : 0u;

    // exact re-evaluation of the queued candidates, one per lane; one append atomic per query and round
    auto drain = [&]() {
        for (uint32_t base = 0; base < qn; base += 64) {
            const uint32_t i = base + lane;
            uint32_t e = 0, hh = 0, mask = 0;
            uint32_t wd[M / 4];
#pragma unroll
            for (int t2 = 0; t2 < M / 4; ++t2) wd[t2] = 0;
            if (i < qn) {
                e = q_entry[i] & 0x7fffffffu;
                hh = q_entry[i] >> 31;
                mask = q_mask[i];
                const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + e) * M);
#pragma unroll
                for (int t2 = 0; t2 < M / 4; ++t2) wd[t2] = src[t2];
            }
            while (__ballot(mask != 0) != 0) {   // one row per lane and round
                int r64 = -1;
                float est = 0.f;
                bool keep = false;
                if (mask) {
                    const int x = __ffs(mask) - 1;
                    mask &= mask - 1;
                    r64 = (x >> 4) * 32 + 8 * ((x & 15) >> 2) + 4 * (int)hh + (x & 3);
                    est = adc_sum_pair<M>(ts.pair((int64_t)s_pid[r64]), wd);
                    keep = est <= s_tau[r64];
                }
                uint64_t todo = __ballot(keep);
                while (todo) {   // one round per row that has records in this wavefront
                    const int leader = __ffsll((long long)todo) - 1;
                    const int rl = __builtin_amdgcn_readlane(r64, leader);
                    const uint64_t same = __ballot(keep && r64 == rl);
                    const int q = (int)(s_pid[rl] / (uint32_t)w);
                    uint32_t first = 0;
                    if (lane == leader) first = atomicAdd(cand_cnt + q, (uint32_t)__popcll(same));
                    first = __builtin_amdgcn_readlane(first, leader);
                    if (keep && r64 == rl) {
                        const uint32_t slot = first + __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
                        if (slot < lay.cap(q)) cand[lay.base(q) + slot] = make_uint2(__float_as_uint(est), start + e);
                    }
                    todo &= ~same;
                }
            }
        }
        qn = 0;
    };

    while (b < b_end) {
        while (blkpre[u + 1] <= b) ++u;
        const uint32_t pb0 = blkpre[u], pb1 = blkpre[u + 1];
        const uint32_t stop = pb1 < b_end ? pb1 : b_end;
        // ---- the unit's 64 queries: residuals -> fp16 operand, per-row constants ----
        uint32_t pidx[2];
        bool real[2];
        const float* xr[2];
        const float* cr[2];
        float rr[2] = {0.f, 0.f}, amax = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const uint32_t raw = unit_pairs[(int64_t)u * MF_ROWS + rb * 32 + row];
            real[rb] = raw != IVFR_NO_PAIR;
            pidx[rb] = real[rb] ? raw : unit_pairs[(int64_t)u * MF_ROWS];
            xr[rb] = queries + (int64_t)(pidx[rb] / (uint32_t)w) * D + 8 * h;
            cr[rb] = coarse + (int64_t)probe[pidx[rb]] * D + 8 * h;
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const float4 x0 = *reinterpret_cast<const float4*>(xr[rb] + 16 * s), x1 = *reinterpret_cast<const float4*>(xr[rb] + 16 * s + 4);
                const float4 c0 = *reinterpret_cast<const float4*>(cr[rb] + 16 * s), c1 = *reinterpret_cast<const float4*>(cr[rb] + 16 * s + 4);
                const float v[8] = {x0.x - c0.x, x0.y - c0.y, x0.z - c0.z, x0.w - c0.w, x1.x - c1.x, x1.y - c1.y, x1.z - c1.z, x1.w - c1.w};
#pragma unroll
                for (int x = 0; x < 8; ++x) { rr[rb] = fmaf(v[x], v[x], rr[rb]); amax = fmaxf(amax, fabsf(v[x])); }
            }
            rr[rb] += __shfl_xor(rr[rb], 32);
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
        int ae = 0;
        if (amax > 0.f) (void)frexpf(2.f * amax, &ae);
        const float s_a = amax > 0.f ? ldexpf(1.f, 9 - ae) : 1.f;   // largest |2 r s_a| in [256, 512)
        const float S = s_a * s_c;
        half8 a[2][KSTEPS];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const float f = -2.f * s_a;
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const float4 x0 = *reinterpret_cast<const float4*>(xr[rb] + 16 * s), x1 = *reinterpret_cast<const float4*>(xr[rb] + 16 * s + 4);
                const float4 c0 = *reinterpret_cast<const float4*>(cr[rb] + 16 * s), c1 = *reinterpret_cast<const float4*>(cr[rb] + 16 * s + 4);
                half8 hv;
                hv[0] = (_Float16)((x0.x - c0.x) * f); hv[1] = (_Float16)((x0.y - c0.y) * f);
                hv[2] = (_Float16)((x0.z - c0.z) * f); hv[3] = (_Float16)((x0.w - c0.w) * f);
                hv[4] = (_Float16)((x1.x - c1.x) * f); hv[5] = (_Float16)((x1.y - c1.y) * f);
                hv[6] = (_Float16)((x1.z - c1.z) * f); hv[7] = (_Float16)((x1.w - c1.w) * f);
                a[rb][s] = hv;
            }
            const float t = tau[(int)(pidx[rb] / (uint32_t)w)];
            const float ub = 60000.f / lut_scale[pidx[rb]];
            // unscaled margin: fp16 rounding of both operands + the tables' own fp32 round-off
            const float mg = 1.05f * 9.765625e-4f * fmaxf(ub - rr[rb] - nmax, 0.f) + 7.62939453125e-6f * ub;
            const float c0v = real[rb] ? S * (rr[rb] - t) - S * mg - 5.f : INFINITY;
            if (h == 0) {
                s_pid[rb * 32 + row] = pidx[rb];
                s_tau[rb * 32 + row] = real[rb] ? t : -1.f;
                s_c0[rb * 32 + row] = c0v;
            }
        }
        floatx16 c0[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int i = 0; i < 16; ++i) c0[rb][i] = s_c0[rb * 32 + 8 * (i >> 2) + 4 * h + (i & 3)];
        start = pair_start[pidx[0]];
        start = __builtin_amdgcn_readfirstlane(start);
        const uint32_t len = __builtin_amdgcn_readfirstlane(pair_len[pidx[0]]);

        // ---- tiles of 32 entries ----
        const uint32_t t0 = (b - pb0) * (IVFR_BLOCK / 32);
        uint32_t t1 = (stop - pb0) * (IVFR_BLOCK / 32);
        const uint32_t tl = (len + 31) / 32;
        if (t1 > tl) t1 = tl;
        uint32_t wn[M / 4];   // code words of the next tile
        {
            const uint32_t e = t0 * 32 + row;
            const bool in = t0 < t1 && e < len;
            const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + (in ? e : 0u)) * M);
#pragma unroll
            for (int t2 = 0; t2 < M / 4; ++t2) wn[t2] = in ? src[t2] : 0u;
        }
        for (uint32_t tile = t0; tile < t1; ++tile) {
            uint32_t wc[M / 4];
#pragma unroll
            for (int t2 = 0; t2 < M / 4; ++t2) wc[t2] = wn[t2];
            const uint32_t e = tile * 32 + row;
            const bool valid = e < len;
            {
                const uint32_t en = e + 32;
                const bool in = tile + 1 < t1 && en < len;
                const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + ((uint64_t)start + (in ? en : 0u)) * M);
#pragma unroll
                for (int t2 = 0; t2 < M / 4; ++t2) wn[t2] = in ? src[t2] : 0u;
            }
            // decoded operand: 8 dimensions of this lane's entry per step
            half8 bv[KSTEPS];
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                uint32_t byte, off;
                if (DSUB == 8) {
                    const uint32_t wsel = wc[(2 * s) / 4] >> (8 * ((2 * s) % 4) + 8 * h);   // sub-quantizer 2s + h
                    byte = wsel & 0xffu;
                    off = (uint32_t)(2 * s) * (IVFR_KS * 16) + byte * 16;
                } else {
                    const int j = (16 * s) / DSUB;
                    byte = (wc[j / 4] >> (8 * (j % 4))) & 0xffu;
                    off = (uint32_t)j * (IVFR_KS * DSUB * 2) + byte * (DSUB * 2) + (uint32_t)((16 * s) % DSUB) * 2;
                }
                bv[s] = *reinterpret_cast<const half8*>(s_cent + cent_lane + off);
            }
            floatx16 acc[2];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[rb][0], bv[0], c0[rb], 0, 0, 0);
#pragma unroll
                for (int s = 1; s < KSTEPS; ++s) acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[rb][s], bv[s], acc[rb], 0, 0, 0);
            }
            // ||y||^2: each lane half sums half of the sub-quantizers (its words picked without indexing by h)
            float ns = 0.f;
            {
                constexpr int NWH = M >= 8 ? M / 8 : 1;
                uint32_t wh[NWH];
                if (M == 4) wh[0] = wc[0] >> (16 * h);
                else {
#pragma unroll
                    for (int t2 = 0; t2 < NWH; ++t2) wh[t2] = wc[t2] ^ ((wc[t2] ^ wc[M / 8 + t2]) & hmask);
                }
#pragma unroll
                for (int jj = 0; jj < M / 2; ++jj) {
                    const uint32_t byte = (wh[jj / 4] >> (8 * (jj % 4))) & 0xffu;
                    ns += *reinterpret_cast<const float*>(reinterpret_cast<const char*>(s_norm) + norm_lane + jj * (IVFR_KS * 4) + byte * 4);
                }
            }
            ns += __shfl_xor(ns, 32);
            const float lim = -S * ns;
            float mn = acc[0][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mn = fminf(mn, acc[0][i]);
#pragma unroll
            for (int i = 0; i < 16; ++i) mn = fminf(mn, acc[1][i]);
            const bool pass = valid && mn <= lim;
            const uint64_t bal = __ballot(pass);
            if (bal == 0) continue;
            if (pass) {
                // bit rb*16 + i = sign of lim - acc (clear: the row may keep the entry), shifted in from the top down
                uint32_t mask = 0;
#pragma unroll
                for (int x = 31; x >= 0; --x)
                    mask = __builtin_amdgcn_alignbit(mask, __float_as_uint(lim - acc[x >> 4][x & 15]), 31);
                mask = ~mask;
                // passing lanes below this one: counted in place (no 64-bit lane mask kept in registers)
                const uint32_t slot = qn + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
                q_entry[slot] = e | (hmask & 0x80000000u);
                q_mask[slot] = mask;
            }
            qn += __popcll(bal);
            if (qn > MFQ_CAP - 64) drain();
        }
        drain();   // the queue refers to this unit's rows
        b = stop;
    }
}

template <int M, int DSUB>
static size_t mfma64_lds_bytes() {
    return (size_t)IVFR_KS * M * DSUB * 2 + (size_t)M * IVFR_KS * 4 +
           (size_t)(MF_T / 64) * (2 * MFQ_CAP + 3 * MF_ROWS) * sizeof(uint32_t);
}

template <int M, int DSUB>
static int launch_mfma64_md(const ivfr_index* ix, const float* queries, const int32_t* probe, const TableSrc& ts,
                            const float* lut_scale, const uint32_t* pair_start, const uint32_t* pair_len,
                            const uint32_t* blkpre, const uint32_t* unit_pairs, const ScanShape& sh, int w,
                            const float* tau, uint2* cand, uint32_t* cand_cnt, CandLayout lay, hipStream_t st) {
    hipLaunchKernelGGL((adc_scan_mfma64_kernel<M, DSUB>), dim3(sh.groups), dim3(MF_T), (mfma64_lds_bytes<M, DSUB>()), st,
                       ix->codes, queries, probe, ix->coarse, ix->pq, ix->pq_norm, ix->pq_maxnorm, ts, lut_scale,
                       pair_start, pair_len, blkpre, unit_pairs, sh.n_host, sh.n_dev, sh.bpg, sh.g_min, w, tau, cand,
                       cand_cnt, lay);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// sub-vectors of 8, 16 or 32 dimensions, at most 128 dimensions (the fp16 codebook takes 512 d bytes of LDS)
bool ivfr_mfma_scan_supported(const ivfr_index* ix) {
    const int m = ix->p.m, ds = ix->dsub;
    return (m == 4 || m == 8 || m == 16) && (ds == 8 || ds == 16 || ds == 32) && m * ds <= 128;
}

int ivfr_launch_scan_mfma64(const ivfr_index* ix, const float* queries, const int32_t* probe, const TableSrc& ts,
                            const float* lut_scale, const uint32_t* pair_start, const uint32_t* pair_len,
                            const uint32_t* blkpre, const uint32_t* unit_pairs, ScanShape sh, int w, const float* tau,
                            uint2* cand, uint32_t* cand_cnt, CandLayout lay, hipStream_t st) {
    if (!sh.n_dev && sh.n_host <= 0) return IVFR_OK;
#define IVFR_MF_ARGS ix, queries, probe, ts, lut_scale, pair_start, pair_len, blkpre, unit_pairs, sh, w, tau, cand, cand_cnt, lay, st
    const int key = ix->p.m * 100 + ix->dsub;
    switch (key) {
        case 408: return launch_mfma64_md<4, 8>(IVFR_MF_ARGS);
        case 416: return launch_mfma64_md<4, 16>(IVFR_MF_ARGS);
        case 432: return launch_mfma64_md<4, 32>(IVFR_MF_ARGS);
        case 808: return launch_mfma64_md<8, 8>(IVFR_MF_ARGS);
        case 816: return launch_mfma64_md<8, 16>(IVFR_MF_ARGS);
        case 1608: return launch_mfma64_md<16, 8>(IVFR_MF_ARGS);
        default:
            ivfr_set_error("matrix-core scan does not support m = %d with %d-dimensional sub-vectors", ix->p.m, ix->dsub);
            return IVFR_ERR_INVALID_ARG;
    }
#undef IVFR_MF_ARGS
}

// ------------------------------------------------------------------------------------------
// Dynamic LDS beyond 48 KB has to be allowed per kernel and device.  Called by ivfr_create with the
// index's device current, for every instantiation the launchers above can pick.
// ------------------------------------------------------------------------------------------
template <class K>
static int allow_lds(K kernel, size_t bytes) {
    if (bytes <= 48 * 1024) return IVFR_OK;
    IVFR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)bytes));
    return IVFR_OK;
}

int ivfr_scan_init() {
    IVFR_TRY(allow_lds(adc_scan_kernel<4, false>, scan_lds_bytes<4>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<4, true>, scan_lds_bytes<4>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<8, false>, scan_lds_bytes<8>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<8, true>, scan_lds_bytes<8>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<16, false>, scan_lds_bytes<16>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<16, true>, scan_lds_bytes<16>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<32, false>, scan_lds_bytes<32>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<32, true>, scan_lds_bytes<32>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<64, false>, scan_lds_bytes<64>()));
    IVFR_TRY(allow_lds(adc_scan_kernel<64, true>, scan_lds_bytes<64>()));
    IVFR_TRY(allow_lds(adc_scan_shared_kernel<4, 4>, shared_lds_bytes<4, 4>()));
    IVFR_TRY(allow_lds(adc_scan_shared_kernel<8, 4>, shared_lds_bytes<8, 4>()));
    IVFR_TRY(allow_lds(adc_scan_shared_kernel<16, 4>, shared_lds_bytes<16, 4>()));
    IVFR_TRY(allow_lds(adc_scan_shared_kernel<4, 2>, shared_lds_bytes<4, 2>()));
    IVFR_TRY(allow_lds(adc_scan_shared_kernel<8, 2>, shared_lds_bytes<8, 2>()));
    IVFR_TRY(allow_lds(adc_scan_shared_kernel<16, 2>, shared_lds_bytes<16, 2>()));
    IVFR_TRY(allow_lds(adc_scan_shared8h_kernel<4>, shared8h_lds_bytes<4>()));
    IVFR_TRY(allow_lds(adc_scan_shared8h_kernel<8>, shared8h_lds_bytes<8>()));
    IVFR_TRY(allow_lds(adc_scan_shared8h_kernel<16>, shared8h_lds_bytes<16>()));
    IVFR_TRY(allow_lds(adc_sample_kernel<4, 2>, sample_lds_bytes<4, 2>()));
    IVFR_TRY(allow_lds(adc_sample_kernel<8, 2>, sample_lds_bytes<8, 2>()));
    IVFR_TRY(allow_lds(adc_sample_kernel<16, 2>, sample_lds_bytes<16, 2>()));
    IVFR_TRY(allow_lds(adc_sample_kernel<32, 4>, sample_lds_bytes<32, 4>()));
    IVFR_TRY(allow_lds(adc_sample_kernel<64, 4>, sample_lds_bytes<64, 4>()));
    IVFR_TRY(allow_lds(adc_scan_mfma64_kernel<4, 8>, mfma64_lds_bytes<4, 8>()));
    IVFR_TRY(allow_lds(adc_scan_mfma64_kernel<4, 16>, mfma64_lds_bytes<4, 16>()));
    IVFR_TRY(allow_lds(adc_scan_mfma64_kernel<4, 32>, mfma64_lds_bytes<4, 32>()));
    IVFR_TRY(allow_lds(adc_scan_mfma64_kernel<8, 8>, mfma64_lds_bytes<8, 8>()));
    IVFR_TRY(allow_lds(adc_scan_mfma64_kernel<8, 16>, mfma64_lds_bytes<8, 16>()));
    IVFR_TRY(allow_lds(adc_scan_mfma64_kernel<16, 8>, mfma64_lds_bytes<16, 8>()));
    return IVFR_OK;
}
