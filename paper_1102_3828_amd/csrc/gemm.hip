// fp32 MFMA distance GEMM for gfx950: rows X [n, d] against centroids C [c, d].
//
// Used for the coarse-quantizer distances of the search (section 3.3: the w nearest of c
// reproduction values) and for nearest-centroid assignment when vectors are encoded or a
// k-means iteration runs (offline steps 1-2 of section 3.2).  ||x - c||^2 is expanded as
// ||x||^2 + ||c||^2 - 2 x.c so that the O(n c d) part is a dense contraction on the matrix
// cores; fp32 inputs and fp32 accumulation (v_mfma_f32_32x32x2_f32) keep the result within
// a few ulp of the direct form.
//
// Tiling: a 256-thread workgroup (4 wavefronts, 2x2) owns a 128x128 output tile; each
// wavefront owns 64x64 = 2x2 MFMA tiles of 32x32 (64 accumulator VGPRs).  K is consumed in
// slabs of 32 staged through LDS (rows padded to 36 floats so that 16-byte fragment reads of
// 8 consecutive rows cover all 32 banks).  A lane reads one float4 per 32-row fragment and
// k-group of 8: lanes 0-31 take k+0..3, lanes 32-63 take k+4..7, and the four MFMAs of the
// group pair element t of A's float4 with element t of B's, so both operands see the same k.
#include "ivfr_internal.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));

#define TM 128
#define TN 128
#define KT 32
#define LDS_STRIDE (KT + 4)

// bad (optional, zero on entry): raised to row + 1 for a row whose squared norm is not a finite number
__global__ __launch_bounds__(256) void row_norms_kernel(const float* __restrict__ X, int64_t n, int dim,
                                                        float* __restrict__ out, uint32_t* __restrict__ bad) {
    int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= n) return;
    const float* x = X + row * dim;
    float s = 0.f;
    for (int e = 0; e < dim; ++e) s = fmaf(x[e], x[e], s);
    out[row] = s;
    if (bad && !(s <= 3.0e38f)) atomicMax(bad, (uint32_t)row + 1u);
}

// out[j] = max over the `per` rows of group j of sqrt(norm2[j * per + k])
__global__ __launch_bounds__(256) void group_max_norm_kernel(const float* __restrict__ norm2, int per,
                                                             float* __restrict__ out) {
    __shared__ float red[256];
    float m = 0.f;
    for (int k = threadIdx.x; k < per; k += 256) m = fmaxf(m, norm2[(int64_t)blockIdx.x * per + k]);
    red[threadIdx.x] = m;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x] = sqrtf(red[0]);
}

int ivfr_launch_group_max_norm(const float* norm2, int groups, int per, float* out, hipStream_t st) {
    hipLaunchKernelGGL(group_max_norm_kernel, dim3(groups), dim3(256), 0, st, norm2, per, out);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// Rows of at least 32 floats: eight lanes per row, 16 bytes per lane and step (coalesced), partial sums combined
// with three xor-shuffles.
__global__ __launch_bounds__(256) void row_norms8_kernel(const float* __restrict__ X, int64_t n, int dim,
                                                         float* __restrict__ out, uint32_t* __restrict__ bad) {
    const int64_t row = (int64_t)blockIdx.x * 32 + (threadIdx.x >> 3);
    const int t = threadIdx.x & 7;
    float s = 0.f;
    if (row < n) {
        const float* x = X + row * dim;
        for (int e = 4 * t; e < dim; e += 32) {
            const float4 v = *reinterpret_cast<const float4*>(x + e);
            s = fmaf(v.x, v.x, s); s = fmaf(v.y, v.y, s); s = fmaf(v.z, v.z, s); s = fmaf(v.w, v.w, s);
        }
    }
    s += __shfl_xor(s, 4, 64);
    s += __shfl_xor(s, 2, 64);
    s += __shfl_xor(s, 1, 64);
    if (row < n && t == 0) {
        out[row] = s;
        if (bad && !(s <= 3.0e38f)) atomicMax(bad, (uint32_t)row + 1u);
    }
}

int ivfr_launch_row_norms(const float* X, int64_t n, int dim, float* out, hipStream_t st, uint32_t* bad) {
    if (n <= 0) return IVFR_OK;
    if (dim >= 32 && dim % 4 == 0) {
        hipLaunchKernelGGL(row_norms8_kernel, dim3((unsigned)((n + 31) / 32)), dim3(256), 0, st, X, n, dim, out, bad);
        IVFR_HIP(hipGetLastError());
        return IVFR_OK;
    }
    hipLaunchKernelGGL(row_norms_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, X, n, dim, out, bad);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

__global__ __launch_bounds__(256) void u8_to_f32_kernel(const uint8_t* __restrict__ x, int64_t count4,
                                                        float* __restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < count4; i += stride) {
        uint32_t v = reinterpret_cast<const uint32_t*>(x)[i];
        float4 f = make_float4((float)(v & 0xff), (float)((v >> 8) & 0xff), (float)((v >> 16) & 0xff),
                               (float)(v >> 24));
        reinterpret_cast<float4*>(out)[i] = f;
    }
}

int ivfr_launch_u8_to_f32(const uint8_t* x, int64_t count, float* out, hipStream_t st) {
    if (count <= 0) return IVFR_OK;
    int64_t c4 = count / 4;   // count is n*d with d % 8 == 0
    int64_t blocks = (c4 + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(u8_to_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, c4, out);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// Stage a [128 x KT] slab of a row-major [rows, d] matrix into LDS (zero fill past `rows` and past d;
// d % 4 == 0).
__device__ __forceinline__ void stage_slab(const float* __restrict__ M, int64_t rows, int d, int64_t row0, int k0,
                                           float* lds) {
    const int tid = threadIdx.x;
    const int kc = (tid & 7) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = (tid >> 3) + 32 * i;
        int64_t gr = row0 + r;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gr < rows && k0 + kc < d) v = *reinterpret_cast<const float4*>(M + gr * d + k0 + kc);
        *reinterpret_cast<float4*>(lds + r * LDS_STRIDE + kc) = v;
    }
}

// Accumulate one KT slab: acc[a][b] += A(rows 64*wm + 32a ..) . B(cols 64*wn + 32b ..)
__device__ __forceinline__ void mma_slab(const float* As, const float* Bs, int wm, int wn, floatx16 acc[2][2]) {
    const int lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < KT / 8; ++kk) {
        float4 a[2], b[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            a[t] = *reinterpret_cast<const float4*>(As + (64 * wm + 32 * t + r) * LDS_STRIDE + kk * 8 + 4 * h);
            b[t] = *reinterpret_cast<const float4*>(Bs + (64 * wn + 32 * t + r) * LDS_STRIDE + kk * 8 + 4 * h);
        }
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].x, b[tb].x, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].y, b[tb].y, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].z, b[tb].z, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].w, b[tb].w, acc[ta][tb], 0, 0, 0);
            }
    }
}

// Accumulator element v of a 32x32 MFMA tile sits at row 8*(v/4) + 4*(lane/32) + v%4, col lane%32.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// The same staging and accumulation for a workgroup tile of (64 T) x (64 T) outputs, T = 1 or 2: each of the
// 2x2 wavefronts owns T x T MFMA tiles.  The k order per output element does not depend on T, so both tile sizes
// give the same bits.
template <int T>
__device__ __forceinline__ void stage_rows(const float* __restrict__ M, int64_t rows, int d, int64_t row0, int k0,
                                           float* lds) {
    const int tid = threadIdx.x;
    const int kc = (tid & 7) * 4;
#pragma unroll
    for (int i = 0; i < 2 * T; ++i) {
        int r = (tid >> 3) + 32 * i;
        int64_t gr = row0 + r;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gr < rows && k0 + kc < d) v = *reinterpret_cast<const float4*>(M + gr * d + k0 + kc);
        *reinterpret_cast<float4*>(lds + r * LDS_STRIDE + kc) = v;
    }
}

template <int T>
__device__ __forceinline__ void mma_tiles(const float* As, const float* Bs, int wm, int wn, floatx16 (&acc)[T][T]) {
    const int lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < KT / 8; ++kk) {
        float4 a[T], b[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            a[t] = *reinterpret_cast<const float4*>(As + (32 * T * wm + 32 * t + r) * LDS_STRIDE + kk * 8 + 4 * h);
            b[t] = *reinterpret_cast<const float4*>(Bs + (32 * T * wn + 32 * t + r) * LDS_STRIDE + kk * 8 + 4 * h);
        }
#pragma unroll
        for (int ta = 0; ta < T; ++ta)
#pragma unroll
            for (int tb = 0; tb < T; ++tb) {
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].x, b[tb].x, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].y, b[tb].y, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].z, b[tb].z, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].w, b[tb].w, acc[ta][tb], 0, 0, 0);
            }
    }
}

template <int T>
__global__ __launch_bounds__(256) void dist_keys_kernel(const float* __restrict__ X, const float* __restrict__ xnorm,
                                                        int64_t n, const float* __restrict__ C,
                                                        const float* __restrict__ cnorm, int c, int d,
                                                        uint64_t* __restrict__ keys) {
    __shared__ float As[64 * T * LDS_STRIDE];
    __shared__ float Bs[64 * T * LDS_STRIDE];
    const int64_t row0 = (int64_t)blockIdx.x * (64 * T);
    const int64_t col0 = (int64_t)blockIdx.y * (64 * T);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm = wave >> 1, wn = wave & 1;
    floatx16 acc[T][T];
#pragma unroll
    for (int a = 0; a < T; ++a)
#pragma unroll
        for (int b = 0; b < T; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    for (int k0 = 0; k0 < d; k0 += KT) {
        __syncthreads();
        stage_rows<T>(X, n, d, row0, k0, As);
        stage_rows<T>(C, c, d, col0, k0, Bs);
        __syncthreads();
        mma_tiles<T>(As, Bs, wm, wn, acc);
    }
#pragma unroll
    for (int ta = 0; ta < T; ++ta)
#pragma unroll
        for (int tb = 0; tb < T; ++tb) {
            int64_t col = col0 + 32 * T * wn + 32 * tb + (lane & 31);
            float cn = (col < c) ? cnorm[col] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int64_t row = row0 + 32 * T * wm + 32 * ta + acc_row(v, lane);
                if (row < n && col < c) {
                    float dist = fmaxf(0.f, fmaf(-2.f, acc[ta][tb][v], xnorm[row] + cn));
                    keys[row * c + col] = ((uint64_t)__float_as_uint(dist) << 32) | (uint32_t)col;
                }
            }
        }
}

int ivfr_launch_dist_keys(const float* X, const float* xnorm, int64_t n, const float* C, const float* cnorm,
                          int c, int d, uint64_t* keys, hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    // 128 x 128 tiles unless they would leave most compute units without a workgroup
    const int64_t big = ((n + TM - 1) / TM) * ((c + TN - 1) / TN);
    if (big >= 256) {
        dim3 grid((unsigned)((n + TM - 1) / TM), (unsigned)((c + TN - 1) / TN));
        hipLaunchKernelGGL(dist_keys_kernel<2>, grid, dim3(256), 0, st, X, xnorm, n, C, cnorm, c, d, keys);
    } else {
        dim3 grid((unsigned)((n + 63) / 64), (unsigned)((c + 63) / 64));
        hipLaunchKernelGGL(dist_keys_kernel<1>, grid, dim3(256), 0, st, X, xnorm, n, C, cnorm, c, d, keys);
    }
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}

// Nearest centroid of each row: one workgroup per 128 rows walks all column tiles and keeps,
// per accumulator slot, the best (value, col) seen; columns are visited in increasing order
// so a strict '<' keeps the lowest index among equal values.  ||x||^2 is the same for every
// column of a row and is left out.
__global__ __launch_bounds__(256) void assign_kernel(const float* __restrict__ X, int64_t n,
                                                     const float* __restrict__ C, const float* __restrict__ cnorm,
                                                     int c, int d, int32_t* __restrict__ assign) {
    __shared__ float As[TM * LDS_STRIDE];
    __shared__ float Bs[TN * LDS_STRIDE];
    __shared__ float red_v[2][TM];
    __shared__ int red_i[2][TM];
    const int64_t row0 = (int64_t)blockIdx.x * TM;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm = wave >> 1, wn = wave & 1;
    float best_v[2][16];
    int best_i[2][16];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) { best_v[a][v] = INFINITY; best_i[a][v] = 0x7fffffff; }

    for (int64_t col0 = 0; col0 < c; col0 += TN) {
        floatx16 acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
        for (int k0 = 0; k0 < d; k0 += KT) {
            __syncthreads();
            stage_slab(X, n, d, row0, k0, As);
            stage_slab(C, c, d, col0, k0, Bs);
            __syncthreads();
            mma_slab(As, Bs, wm, wn, acc);
        }
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            int col = (int)col0 + 64 * wn + 32 * tb + (lane & 31);
            bool ok = col < c;
            float cn = ok ? cnorm[col] : 0.f;
#pragma unroll
            for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float val = fmaf(-2.f, acc[ta][tb][v], cn);
                    if (ok && val < best_v[ta][v]) { best_v[ta][v] = val; best_i[ta][v] = col; }
                }
        }
    }
    // reduce over the 32 lanes that share a row (same lane/32), then over the two column waves
#pragma unroll
    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float bv = best_v[ta][v];
            int bi = best_i[ta][v];
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1) {
                float ov = __shfl_xor(bv, off, 64);
                int oi = __shfl_xor(bi, off, 64);
                if (ov < bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if ((lane & 31) == 0) {
                int r = 64 * wm + 32 * ta + acc_row(v, lane);
                red_v[wn][r] = bv;
                red_i[wn][r] = bi;
            }
        }
    __syncthreads();
    if (threadIdx.x < TM) {
        int r = threadIdx.x;
        int64_t row = row0 + r;
        if (row < n) {
            float v0 = red_v[0][r], v1 = red_v[1][r];
            int i0 = red_i[0][r], i1 = red_i[1][r];
            assign[row] = (v1 < v0 || (v1 == v0 && i1 < i0)) ? i1 : i0;
        }
    }
}

// The same assignment with the 128 rows of X resident in LDS for the whole walk over the columns
// (d <= 128): a 512-thread workgroup (8 wavefronts, 2x4) takes 128 rows x 256 columns per step, only
// the centroid slabs are staged, double-buffered, and the global loads of the next slab are issued
// before the matrix instructions of the current one, so one barrier per slab remains.  Same slab
// order and accumulation as assign_kernel: the results are identical.
#define RN 256
__device__ __forceinline__ void mma_slab_rs(const float* As, int a_stride, const float* Bs, int wm, int wn,
                                            floatx16 acc[2][2]) {
    const int lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < KT / 8; ++kk) {
        float4 a[2], b[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            a[t] = *reinterpret_cast<const float4*>(As + (64 * wm + 32 * t + r) * a_stride + kk * 8 + 4 * h);
            b[t] = *reinterpret_cast<const float4*>(Bs + (64 * wn + 32 * t + r) * LDS_STRIDE + kk * 8 + 4 * h);
        }
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].x, b[tb].x, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].y, b[tb].y, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].z, b[tb].z, acc[ta][tb], 0, 0, 0);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta].w, b[tb].w, acc[ta][tb], 0, 0, 0);
            }
    }
}

__global__ __launch_bounds__(512) void assign_resident_kernel(const float* __restrict__ X, int64_t n,
                                                              const float* __restrict__ C,
                                                              const float* __restrict__ cnorm, int c, int d, int dpad,
                                                              int32_t* __restrict__ assign) {
    extern __shared__ float smem[];
    __shared__ float red_v[4][TM];
    __shared__ int red_i[4][TM];
    const int DP = dpad + 4;
    float* As = smem;             // [TM][DP]
    float* Bs = As + TM * DP;     // 2 x [RN][LDS_STRIDE]
    const int64_t row0 = (int64_t)blockIdx.x * TM;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 2, wn = wave & 3;
    const int kc = (tid & 7) * 4, sr = tid >> 3;   // staging: 64 rows x 8 float4 per pass
    for (int k0 = 0; k0 < dpad; k0 += KT)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = sr + 64 * i;
            const int64_t gr = row0 + r;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gr < n && k0 + kc < d) v = *reinterpret_cast<const float4*>(X + gr * d + k0 + kc);
            *reinterpret_cast<float4*>(As + r * DP + k0 + kc) = v;
        }
    const int ks = dpad / KT, ntile = (c + RN - 1) / RN, S = ntile * ks;
    float4 pre[4];
    auto load_b = [&](int s) {
        const int col0 = (s / ks) * RN, k0 = (s % ks) * KT;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int gc = col0 + sr + 64 * i;
            pre[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gc < c && k0 + kc < d) pre[i] = *reinterpret_cast<const float4*>(C + (int64_t)gc * d + k0 + kc);
        }
    };
    auto store_b = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<float4*>(Bs + buf * RN * LDS_STRIDE + (sr + 64 * i) * LDS_STRIDE + kc) = pre[i];
    };
    float best_v[2][16];
    int best_i[2][16];
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            best_v[a][v] = INFINITY; best_i[a][v] = 0x7fffffff;
            acc[a][0][v] = 0.f; acc[a][1][v] = 0.f;
        }
    load_b(0);
    store_b(0);
    __syncthreads();
    for (int s = 0; s < S; ++s) {
        if (s + 1 < S) load_b(s + 1);
        mma_slab_rs(As + (s % ks) * KT, DP, Bs + (s & 1) * RN * LDS_STRIDE, wm, wn, acc);
        if (s % ks == ks - 1) {
            const int col0 = (s / ks) * RN;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int col = col0 + 64 * wn + 32 * tb + (lane & 31);
                const bool ok = col < c;
                const float cn = ok ? cnorm[col] : 0.f;
#pragma unroll
                for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float val = fmaf(-2.f, acc[ta][tb][v], cn);
                        if (ok && val < best_v[ta][v]) { best_v[ta][v] = val; best_i[ta][v] = col; }
                        acc[ta][tb][v] = 0.f;
                    }
            }
        }
        if (s + 1 < S) store_b((s + 1) & 1);
        __syncthreads();
    }
    // reduce over the 32 lanes that share a row, then over the four column wavefronts
#pragma unroll
    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float bv = best_v[ta][v];
            int bi = best_i[ta][v];
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1) {
                float ov = __shfl_xor(bv, off, 64);
                int oi = __shfl_xor(bi, off, 64);
                if (ov < bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if ((lane & 31) == 0) {
                int r = 64 * wm + 32 * ta + acc_row(v, lane);
                red_v[wn][r] = bv;
                red_i[wn][r] = bi;
            }
        }
    __syncthreads();
    if (tid < TM) {
        const int64_t row = row0 + tid;
        if (row < n) {
            float bv = red_v[0][tid];
            int bi = red_i[0][tid];
#pragma unroll
            for (int x = 1; x < 4; ++x) {
                const float ov = red_v[x][tid];
                const int oi = red_i[x][tid];
                if (ov < bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            assign[row] = bi;
        }
    }
}

int ivfr_launch_assign(const float* X, int64_t n, const float* C, const float* cnorm, int c, int d,
                       int32_t* assign, hipStream_t st) {
    if (n <= 0) return IVFR_OK;
    dim3 grid((unsigned)((n + TM - 1) / TM));
    const int dpad = (d + KT - 1) / KT * KT;
    if (dpad <= 128) {
        const size_t lds = ((size_t)TM * (dpad + 4) + 2 * (size_t)RN * LDS_STRIDE) * sizeof(float);
        static bool attr_done = false;
        if (!attr_done) {
            IVFR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(assign_resident_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024));
            attr_done = true;
        }
        hipLaunchKernelGGL(assign_resident_kernel, grid, dim3(512), lds, st, X, n, C, cnorm, c, d, dpad, assign);
        IVFR_HIP(hipGetLastError());
        return IVFR_OK;
    }
    hipLaunchKernelGGL(assign_kernel, grid, dim3(256), 0, st, X, n, C, cnorm, c, d, assign);
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}
