// Offline stage of section 3.2 (gfx950): residuals, product-quantizer encoding (Eq. (4), (8)),
// stable placement of encoded vectors into inverted lists, and the k-means updates used to
// learn the quantizers (step 1).
#include "ivfr_internal.h"

// X[i] -= C[assign[i]]   (Eq. (7) with the coarse quantizer: residual to the list's centroid)
__global__ __launch_bounds__(256) void residual_kernel(float* __restrict__ X, int64_t n, int d4,
                                                       const float* __restrict__ C,
                                                       const int32_t* __restrict__ assign) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * d4) return;
    int64_t row = i / d4;
    int e = (int)(i % d4);
    float4 x = reinterpret_cast<float4*>(X)[i];
    float4 c = reinterpret_cast<const float4*>(C)[(int64_t)assign[row] * d4 + e];
    reinterpret_cast<float4*>(X)[i] = make_float4(x.x - c.x, x.y - c.y, x.z - c.z, x.w - c.w);
}

int ivfr_launch_residual(float* X, int64_t n, int d, const float* C, const int32_t* assign, hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    int64_t total = n * (d / 4);
    hipLaunchKernelGGL(residual_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, X, n, d / 4, C,
                       assign);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// code[i][j] = argmin_k || R[i]^j - book[j][k] ||^2 (ties to the lowest k); with `subtract`
// the chosen reproduction value is removed from R in place, leaving the next-level residual.
// One thread per (vector, sub-quantizer); the sub-quantizer's 256 centroids sit in LDS and are
// read as broadcasts.
template <int DSUB>
__global__ __launch_bounds__(256) void pq_encode_kernel(float* __restrict__ R, int64_t n, int d,
                                                        const float* __restrict__ book, int parts,
                                                        uint8_t* __restrict__ codes, int subtract) {
    extern __shared__ float cb[];   // [256][DSUB]
    const int j = blockIdx.y;
    for (int i = threadIdx.x; i < IVFR_KS * DSUB; i += 256) cb[i] = book[(int64_t)j * IVFR_KS * DSUB + i];
    __syncthreads();
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float v[DSUB];
    float* src = R + i * d + j * DSUB;
#pragma unroll
    for (int t = 0; t < DSUB; ++t) v[t] = src[t];
    float best = INFINITY;
    int bi = 0;
    for (int k = 0; k < IVFR_KS; ++k) {
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) { float df = v[t] - cb[k * DSUB + t]; s = fmaf(df, df, s); }
        if (s < best) { best = s; bi = k; }
    }
    if (codes) codes[i * parts + j] = (uint8_t)bi;
    if (subtract) {
#pragma unroll
        for (int t = 0; t < DSUB; ++t) src[t] = v[t] - cb[bi * DSUB + t];
    }
}

int ivfr_launch_pq_encode(float* R, int64_t n, int d, const float* book, int parts, uint8_t* codes, bool subtract,
                          hipStream_t st) {
    if (n <= 0 || parts <= 0) return IVFR_OK;
    const int dsub = d / parts;
    dim3 grid((unsigned)((n + 255) / 256), parts);
    size_t lds = (size_t)IVFR_KS * dsub * sizeof(float);
#define IVFR_ENC_CASE(D)                                                                                  \
    case D:                                                                                               \
        hipLaunchKernelGGL(pq_encode_kernel<D>, grid, dim3(256), lds, st, R, n, d, book, parts, codes,    \
                           subtract ? 1 : 0);                                                             \
        break
    switch (dsub) {
        IVFR_ENC_CASE(1);
        IVFR_ENC_CASE(2);
        IVFR_ENC_CASE(4);
        IVFR_ENC_CASE(8);
        IVFR_ENC_CASE(16);
        IVFR_ENC_CASE(32);
        default:
            ivfr_set_error("sub-vector width d/m = %d not supported (1, 2, 4, 8, 16, 32)", dsub);
            return IVFR_ERR_INVALID_ARG;
    }
#undef IVFR_ENC_CASE
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// ---- stable rank of each vector inside its list ----------------------------------------------
// T threads each own a contiguous run of the batch.  cnt is a [T, c] matrix: (1) every thread
// counts its run per list, (2) a column scan turns the counts into each run's first rank in
// the list (continuing from the entries already in it), (3) every thread walks its run again
// and hands out consecutive ranks.  Insertion order, hence ascending id order, is kept.
__global__ void rank_count_kernel(const int32_t* __restrict__ list, int64_t n, int64_t run, int c,
                                  uint32_t* __restrict__ cnt) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t a = t * run, b = a + run < n ? a + run : n;
    uint32_t* row = cnt + t * c;
    for (int64_t i = a; i < b; ++i) row[list[i]] += 1;
}

__global__ void rank_colscan_kernel(uint32_t* __restrict__ cnt, int T, int c,
                                    unsigned long long* __restrict__ list_fill) {
    int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= c) return;
    unsigned long long running = list_fill[l];
    for (int t = 0; t < T; ++t) {
        uint32_t v = cnt[(int64_t)t * c + l];
        cnt[(int64_t)t * c + l] = (uint32_t)running;
        running += v;
    }
    list_fill[l] = running;
}

__global__ void rank_assign_kernel(const int32_t* __restrict__ list, int64_t n, int64_t run, int c,
                                   uint32_t* __restrict__ cnt, uint32_t* __restrict__ rank) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t a = t * run, b = a + run < n ? a + run : n;
    uint32_t* row = cnt + t * c;
    for (int64_t i = a; i < b; ++i) rank[i] = row[list[i]]++;
}

int ivfr_launch_list_ranks(const int32_t* list, int64_t n, int c, unsigned long long* list_fill, uint32_t* cnt,
                           int T, uint32_t* rank, hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    int64_t run = (n + T - 1) / T;
    IVFR_HIP(hipMemsetAsync(cnt, 0, (size_t)T * c * sizeof(uint32_t), st));
    hipLaunchKernelGGL(rank_count_kernel, dim3((T + 63) / 64), dim3(64), 0, st, list, n, run, c, cnt);
    hipLaunchKernelGGL(rank_colscan_kernel, dim3((c + 63) / 64), dim3(64), 0, st, cnt, T, c, list_fill);
    hipLaunchKernelGGL(rank_assign_kernel, dim3((T + 63) / 64), dim3(64), 0, st, list, n, run, c, cnt, rank);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// Move one staged batch into the finished, list-sorted arrays: the dense code stream of the list scan and the
// per-entry record (id, list, code, refinement code) that the re-rank and the tie-breaks by id read.
__global__ __launch_bounds__(256) void scatter_kernel(const int32_t* __restrict__ list,
                                                      const uint32_t* __restrict__ rank,
                                                      const int32_t* __restrict__ ids_in,
                                                      const uint8_t* __restrict__ codes_in,
                                                      const uint8_t* __restrict__ rcodes_in, int64_t n, int m, int mr,
                                                      const uint32_t* __restrict__ list_start,
                                                      uint8_t* __restrict__ codes, uint8_t* __restrict__ rec,
                                                      int rec_stride) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int l = list[i];
    uint64_t dst = (uint64_t)list_start[l] + rank[i];
    const uint32_t* s = reinterpret_cast<const uint32_t*>(codes_in + i * m);
    uint32_t* o = reinterpret_cast<uint32_t*>(codes + dst * m);
    uint32_t* r = reinterpret_cast<uint32_t*>(rec + dst * rec_stride);
    r[0] = (uint32_t)ids_in[i];
    r[1] = (uint32_t)l;
    for (int t = 0; t < m / 4; ++t) { o[t] = s[t]; r[2 + t] = s[t]; }
    if (mr > 0) {
        const uint32_t* sr = reinterpret_cast<const uint32_t*>(rcodes_in + i * mr);
        for (int t = 0; t < mr / 4; ++t) r[2 + m / 4 + t] = sr[t];
    }
}

int ivfr_launch_scatter(const StagedChunk& ch, int m, int mr, const uint32_t* list_start, uint8_t* codes,
                        uint8_t* rec, int rec_stride, hipStream_t st) {
    if (ch.n <= 0) return IVFR_OK;
    hipLaunchKernelGGL(scatter_kernel, dim3((unsigned)((ch.n + 255) / 256)), dim3(256), 0, st, ch.list, ch.rank,
                       ch.ids, ch.codes, ch.rcodes, ch.n, m, mr, list_start, codes, rec, rec_stride);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// Records <-> dense per-slot arrays, for import and export.  Slots [slot0, slot0 + n) of the padded layout;
// ids_st [n], rcodes_st [n, mr] are indexed by slot - slot0.  pack: the list of a slot is the last one that
// starts at or before it (binary search); slots past the end of their list are padding and are left alone.
__global__ __launch_bounds__(256) void pack_records_kernel(uint64_t slot0, int64_t n, int m, int mr, int c,
                                                           const uint32_t* __restrict__ list_start,
                                                           const uint32_t* __restrict__ list_len,
                                                           const int32_t* __restrict__ ids_st,
                                                           const uint8_t* __restrict__ rcodes_st,
                                                           const uint8_t* __restrict__ codes,
                                                           uint8_t* __restrict__ rec, int rec_stride) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint64_t slot = slot0 + (uint64_t)i;
    int lo = 0, hi = c;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if ((uint64_t)list_start[mid] <= slot) lo = mid; else hi = mid;
    }
    if (slot - list_start[lo] >= list_len[lo]) return;
    uint32_t* r = reinterpret_cast<uint32_t*>(rec + slot * rec_stride);
    r[0] = (uint32_t)ids_st[i];
    r[1] = (uint32_t)lo;
    const uint32_t* s = reinterpret_cast<const uint32_t*>(codes + slot * m);
    for (int t = 0; t < m / 4; ++t) r[2 + t] = s[t];
    const uint32_t* sr = reinterpret_cast<const uint32_t*>(rcodes_st + i * mr);
    for (int t = 0; t < mr / 4; ++t) r[2 + m / 4 + t] = sr[t];
}

__global__ __launch_bounds__(256) void unpack_records_kernel(uint64_t slot0, int64_t n, int m, int mr,
                                                             const uint8_t* __restrict__ rec, int rec_stride,
                                                             int32_t* __restrict__ ids_st,
                                                             uint8_t* __restrict__ rcodes_st) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t* r = reinterpret_cast<const uint32_t*>(rec + (slot0 + (uint64_t)i) * rec_stride);
    ids_st[i] = (int32_t)r[0];
    uint32_t* o = reinterpret_cast<uint32_t*>(rcodes_st + i * mr);
    for (int t = 0; t < mr / 4; ++t) o[t] = r[2 + m / 4 + t];
}

int ivfr_launch_pack_records(const ivfr_index* ix, uint64_t slot0, int64_t n, const int32_t* ids_st,
                             const uint8_t* rcodes_st, hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    hipLaunchKernelGGL(pack_records_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, slot0, n, ix->p.m,
                       ix->p.m_refine, ix->p.c, ix->list_start, ix->list_len, ids_st, rcodes_st, ix->codes, ix->rec,
                       ix->rec_stride);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

int ivfr_launch_unpack_records(const ivfr_index* ix, uint64_t slot0, int64_t n, int32_t* ids_st, uint8_t* rcodes_st,
                               hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    hipLaunchKernelGGL(unpack_records_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, slot0, n, ix->p.m,
                       ix->p.m_refine, ix->rec, ix->rec_stride, ids_st, rcodes_st);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

__global__ __launch_bounds__(256) void iota_ids_kernel(int32_t* ids, int64_t n, int64_t base) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) ids[i] = (int32_t)(base + i);
}

int ivfr_launch_iota(int32_t* ids, int64_t n, int64_t base, hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    hipLaunchKernelGGL(iota_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ids, n, base);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// ---- k-means update (Lloyd): centroid = mean of its assigned points ---------------------------
// Sums are accumulated as 64-bit fixed point (2^-20 resolution) with integer atomics, so the
// result does not depend on the order in which threads arrive.
#define KM_SCALE 1048576.0f

__global__ __launch_bounds__(256) void km_accum_rows_kernel(const float* __restrict__ X, int64_t n, int d,
                                                            const int32_t* __restrict__ assign,
                                                            unsigned long long* __restrict__ sums,
                                                            unsigned long long* __restrict__ counts) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * d) return;
    int64_t row = i / d;
    int e = (int)(i % d);
    int l = assign[row];
    long long v = __float2ll_rn(X[i] * KM_SCALE);
    atomicAdd(&sums[(int64_t)l * d + e], (unsigned long long)v);
    if (e == 0) atomicAdd(&counts[l], 1ull);
}

// product-quantizer variant: point i, sub-quantizer j is assigned to centroid codes[i][j]
__global__ __launch_bounds__(256) void km_accum_pq_kernel(const float* __restrict__ R, int64_t n, int d, int parts,
                                                          const uint8_t* __restrict__ codes,
                                                          unsigned long long* __restrict__ sums,
                                                          unsigned long long* __restrict__ counts) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * d) return;
    int64_t row = i / d;
    int e = (int)(i % d);
    int dsub = d / parts;
    int j = e / dsub, t = e % dsub;
    int k = codes[row * parts + j];
    long long v = __float2ll_rn(R[i] * KM_SCALE);
    atomicAdd(&sums[((int64_t)j * IVFR_KS + k) * dsub + t], (unsigned long long)v);
    if (t == 0) atomicAdd(&counts[j * IVFR_KS + k], 1ull);
}

// cent[g][t] = sums / counts where counts > 0 (an empty cluster keeps its centroid); width = floats per centroid
__global__ __launch_bounds__(256) void km_update_kernel(float* __restrict__ cent, int64_t total, int width,
                                                        const unsigned long long* __restrict__ sums,
                                                        const unsigned long long* __restrict__ counts) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    unsigned long long cn = counts[i / width];
    if (cn == 0) return;
    double s = (double)(long long)sums[i] / (double)KM_SCALE;
    cent[i] = (float)(s / (double)cn);
}

int ivfr_launch_km_accum_rows(const float* X, int64_t n, int d, const int32_t* assign, unsigned long long* sums,
                              unsigned long long* counts, hipStream_t st) {
    int64_t total = n * d;
    hipLaunchKernelGGL(km_accum_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, X, n, d, assign,
                       sums, counts);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

int ivfr_launch_km_accum_pq(const float* R, int64_t n, int d, int parts, const uint8_t* codes,
                            unsigned long long* sums, unsigned long long* counts, hipStream_t st) {
    int64_t total = n * d;
    hipLaunchKernelGGL(km_accum_pq_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, R, n, d, parts,
                       codes, sums, counts);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

int ivfr_launch_km_update(float* cent, int64_t total, int width, const unsigned long long* sums,
                          const unsigned long long* counts, hipStream_t st) {
    hipLaunchKernelGGL(km_update_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, cent, total, width,
                       sums, counts);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// rows of X selected by idx -> out (initial centroids); sub-vector variant for product quantizers
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ X, int d, int col0, int width,
                                                          const int64_t* __restrict__ idx, int count,
                                                          float* __restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)count * width) return;
    int r = (int)(i / width), t = (int)(i % width);
    out[i] = X[idx[r] * d + col0 + t];
}

int ivfr_launch_gather_rows(const float* X, int d, int col0, int width, const int64_t* idx, int count, float* out,
                            hipStream_t st) {
    int64_t total = (int64_t)count * width;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, X, d, col0, width,
                       idx, count, out);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}
