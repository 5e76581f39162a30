// Query step 2 of section 3.2 (gfx950): for each short-list entry, rebuild the refined
// approximation  y^ = coarse[l] + decode(q_c code) + decode(q_r code)  of Eq. (9) explicitly and
// compute the squared distance ||x - y^||^2 of Eq. (10).  No full database vector is read:
// an entry costs m + m' + 4 gathered bytes; the codebooks and the coarse centroids are small
// enough to be served from cache.
//
// Eight lanes share one entry and interleave its dimensions in 16-byte pieces (lane t takes
// dimensions 4t..4t+3 of every group of 32), so that one load instruction of the eight lanes
// covers 128 contiguous bytes of the query and the coarse centroid and whole codebook rows (few
// cache lines per instruction); the partial sums are combined with three xor-shuffles.
// Everything that is fetched per candidate - id, list, code and refinement code - sits in one
// record that never straddles a 128-byte line, so the random gather from HBM costs one line per
// candidate.  Output per entry: the 64-bit key (distance bits << 32 | id) consumed by the final
// top-k selection.
#include "ivfr_internal.h"
#include <algorithm>

template <int VEC>
__global__ __launch_bounds__(256) void rerank_kernel(const float* __restrict__ queries, int d, int c, int m, int mr,
                                                     int dsub, int dsub_r, const float* __restrict__ coarse,
                                                     const float* __restrict__ pq, const float* __restrict__ rq,
                                                     const uint8_t* __restrict__ rec, int rec_stride,
                                                     int kprime, int q_base,
                                                     const uint32_t* __restrict__ short_pos,
                                                     const int32_t* __restrict__ short_n, uint64_t* __restrict__ keys,
                                                     float* __restrict__ refined_out, int32_t* __restrict__ ids_out) {
    const int q = q_base + blockIdx.y;
    const int n = short_n[q];
    const int slot = blockIdx.x * 32 + (threadIdx.x >> 3);
    const int t = threadIdx.x & 7;
    const bool live = slot < n;   // uniform over the 8 lanes of an entry
    float acc = 0.f;
    int32_t id = -1;
    if (live) {
        const uint32_t pos = short_pos[(int64_t)q * kprime + slot];
        const uint8_t* r = rec + (uint64_t)pos * rec_stride;
        id = *reinterpret_cast<const int32_t*>(r);
        const uint32_t l = *reinterpret_cast<const uint32_t*>(r + 4);
        const uint8_t* code = r + 8;
        const uint8_t* rcode = r + 8 + m;
        const float* x = queries + (int64_t)q * d;
        const float* cl = coarse + (int64_t)l * d;
        if (VEC == 4) {
            for (int e = 4 * t; e < d; e += 32) {
                const int j = e / dsub;
                float4 y = *reinterpret_cast<const float4*>(cl + e);
                float4 pv = *reinterpret_cast<const float4*>(pq + ((int64_t)j * IVFR_KS + code[j]) * dsub + (e - j * dsub));
                y.x += pv.x; y.y += pv.y; y.z += pv.z; y.w += pv.w;
                if (mr > 0) {
                    const int jr = e / dsub_r;
                    float4 rv = *reinterpret_cast<const float4*>(rq + ((int64_t)jr * IVFR_KS + rcode[jr]) * dsub_r +
                                                                 (e - jr * dsub_r));
                    y.x += rv.x; y.y += rv.y; y.z += rv.z; y.w += rv.w;
                }
                float4 xv = *reinterpret_cast<const float4*>(x + e);
                float a = xv.x - y.x, b = xv.y - y.y, cc = xv.z - y.z, dd = xv.w - y.w;
                acc = fmaf(a, a, acc); acc = fmaf(b, b, acc); acc = fmaf(cc, cc, acc); acc = fmaf(dd, dd, acc);
            }
        } else {
            for (int e = t; e < d; e += 8) {
                const int j = e / dsub;
                float y = cl[e] + pq[((int64_t)j * IVFR_KS + code[j]) * dsub + (e - j * dsub)];
                if (mr > 0) {
                    const int jr = e / dsub_r;
                    y += rq[((int64_t)jr * IVFR_KS + rcode[jr]) * dsub_r + (e - jr * dsub_r)];
                }
                float a = x[e] - y;
                acc = fmaf(a, a, acc);
            }
        }
    }
    acc += __shfl_xor(acc, 4, 64);
    acc += __shfl_xor(acc, 2, 64);
    acc += __shfl_xor(acc, 1, 64);
    if (t == 0 && slot < kprime) {
        const int64_t o = (int64_t)q * kprime + slot;
        if (live) {
            keys[o] = ((uint64_t)__float_as_uint(acc) << 32) | (uint32_t)id;
            if (refined_out) refined_out[o] = acc;
            if (ids_out) ids_out[o] = id;
        } else {
            keys[o] = ~0ull;
            if (refined_out) refined_out[o] = INFINITY;
            if (ids_out) ids_out[o] = -1;
        }
    }
}

// Variant for many short-list entries: the refinement codebook (256 d floats, 128 KB at d = 128) is
// copied into LDS once per workgroup and the workgroups (one per compute unit, 1024 threads) walk over
// blocks of 128 entries, each workgroup over one contiguous range of blocks, so that consecutive blocks belong to
// the same query and its vector stays in registers.  The codebook rows are short (d/m' floats), so gathering them through the
// vector cache fetches whole 128-byte lines for 32 or 64 useful bytes, and that fill traffic from L2 is
// what bounds the plain kernel when k' is large.  Arithmetic and summation order are the same.
// FM = m' (8, 16 or 32) for the common shape d = 128, m = 8: the record is then read with two or three 16-byte loads
// (id, list and the eight code bytes in the first) and this lane's code bytes are shifted out of registers, instead
// of ten narrow loads of the same line.  FM = 0: any shape.
template <int FM>
__global__ __launch_bounds__(1024) void rerank_lds_kernel(const float* __restrict__ queries, int d, int c, int m, int mr,
                                                          int dsub, int dsub_r, const float* __restrict__ coarse,
                                                          const float* __restrict__ pq, const float* __restrict__ rq,
                                                          const uint8_t* __restrict__ rec, int rec_stride,
                                                          int kprime, int q_base,
                                                          int nq, const uint32_t* __restrict__ short_pos,
                                                          const int32_t* __restrict__ short_n,
                                                          uint64_t* __restrict__ keys, float* __restrict__ refined_out,
                                                          int32_t* __restrict__ ids_out) {
    extern __shared__ float s_rq[];   // [m'][256][d/m'] = 256 d floats
    for (int i = threadIdx.x; i < 64 * d; i += 1024)
        reinterpret_cast<float4*>(s_rq)[i] = reinterpret_cast<const float4*>(rq)[i];
    __syncthreads();
    const int t = threadIdx.x & 7, g = threadIdx.x >> 3;
    // C entries per group of eight lanes and block (slots g, g + 128, ... of a block of 128 C slots): their decode
    // chains are independent, so C of each load are in flight per lane
    constexpr int C = FM > 0 ? 2 : 1;
    const int per_q = (kprime + 128 * C - 1) / (128 * C);
    const int64_t n_items = (int64_t)nq * per_q;
    // 16-byte pieces of a vector per lane (d is a multiple of 32 here, at most 128).  A run-time value on purpose: as a
    // compile-time constant the compiler issues all loads of an entry's decode up front, which measured slower
    // (0.88 -> 0.99 ms for 10^7 entries).
    const int nit = d / 32;
    // Three items are in flight per workgroup: the position of item i + 2 is being read, the record of item
    // i + 1 (id, list, code bytes: one random line from HBM per entry, the latency that bounds this kernel) is
    // being gathered, item i is decoded.  Loads return in issue order, so waiting for the oldest leaves the
    // younger ones in flight.
    struct Pos { int q, slot, n; uint32_t pos[C]; };   // slot: the first of the group's C slots
    struct Gather { int32_t id[C]; uint32_t list[C]; uint32_t cb[C][4], rb[C][4]; };
    const int64_t item_end = n_items * (int64_t)(blockIdx.x + 1) / (int64_t)gridDim.x;
    auto read_pos = [&](int64_t item) -> Pos {
        Pos r;
        r.q = 0; r.slot = 0; r.n = 0;
#pragma unroll
        for (int cc = 0; cc < C; ++cc) r.pos[cc] = 0;
        if (item < item_end) {
            r.q = q_base + (int)(item / per_q);
            r.slot = (int)(item % per_q) * (128 * C) + g;
            r.n = short_n[r.q];
#pragma unroll
            for (int cc = 0; cc < C; ++cc)
                if (r.slot + 128 * cc < kprime) r.pos[cc] = short_pos[(int64_t)r.q * kprime + r.slot + 128 * cc];
        }
        return r;
    };
    auto gather = [&](const Pos& p) -> Gather {
        Gather r;
#pragma unroll
        for (int cc = 0; cc < C; ++cc) {
            r.id[cc] = -1;
            r.list[cc] = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) { r.cb[cc][k] = 0; r.rb[cc][k] = 0; }
            const bool live = p.slot + 128 * cc < p.n;   // uniform over the 8 lanes of an entry
            if (FM > 0 && live) {
                // d = 128, m = 8: piece k of lane t lies in sub-quantizer 2k + t/4 of the first stage (16 dimensions each)
                const uint8_t* e = rec + (uint64_t)p.pos[cc] * rec_stride;
                const uint4 h = *reinterpret_cast<const uint4*>(e);
                r.id[cc] = (int32_t)h.x;
                r.list[cc] = h.y;
                const uint32_t cw[2] = {h.z, h.w};
                const uint32_t hi4 = (uint32_t)t >> 2;
#pragma unroll
                for (int k = 0; k < 4; ++k) r.cb[cc][k] = (cw[k >> 1] >> (8u * (2u * (k & 1) + hi4))) & 0xffu;
                if (FM == 8) {          // 16 dimensions per refinement sub-quantizer: the same byte pattern
                    const uint2 rw2 = *reinterpret_cast<const uint2*>(e + 16);
                    const uint32_t rw[2] = {rw2.x, rw2.y};
#pragma unroll
                    for (int k = 0; k < 4; ++k) r.rb[cc][k] = (rw[k >> 1] >> (8u * (2u * (k & 1) + hi4))) & 0xffu;
                } else if (FM == 16) {  // 8 dimensions each: byte 4k + t/2
                    const uint4 rw4 = *reinterpret_cast<const uint4*>(e + 16);
                    const uint32_t rw[4] = {rw4.x, rw4.y, rw4.z, rw4.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) r.rb[cc][k] = (rw[k] >> (8u * ((uint32_t)t >> 1))) & 0xffu;
                } else {                // 4 dimensions each: byte 8k + t
                    const uint4 ra = *reinterpret_cast<const uint4*>(e + 16), rb4 = *reinterpret_cast<const uint4*>(e + 32);
                    const uint32_t rw[8] = {ra.x, ra.y, ra.z, ra.w, rb4.x, rb4.y, rb4.z, rb4.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        r.rb[cc][k] = ((hi4 ? rw[2 * k + 1] : rw[2 * k]) >> (8u * ((uint32_t)t & 3u))) & 0xffu;
                }
            } else if (live) {
                const uint8_t* e = rec + (uint64_t)p.pos[cc] * rec_stride;
                r.id[cc] = *reinterpret_cast<const int32_t*>(e);
                r.list[cc] = *reinterpret_cast<const uint32_t*>(e + 4);
                const uint8_t* code = e + 8;
                const uint8_t* rcode = e + 8 + m;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int e2 = 4 * t + 32 * k;
                    if (k < nit) { r.cb[cc][k] = code[e2 / dsub]; r.rb[cc][k] = rcode[e2 / dsub_r]; }
                }
            }
        }
        return r;
    };
    int64_t item = n_items * (int64_t)blockIdx.x / (int64_t)gridDim.x;
    Pos p0 = read_pos(item), p1 = read_pos(item + 1);
    Gather g0 = gather(p0);
    float4 xr[4];   // this lane's pieces of the current query
    int xq = -1;
#pragma unroll
    for (int k = 0; k < 4; ++k) xr[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    // sub-vector widths: compile-time for the common shape (shifts instead of multiplications)
    const int ds = FM > 0 ? 16 : dsub, dr = FM > 0 ? 128 / (FM > 0 ? FM : 1) : dsub_r;
    for (; item < item_end; ++item) {
        const Pos p2 = read_pos(item + 2);
        const Gather g1 = gather(p1);
        if (p0.q != xq) {   // uniform over the workgroup
            xq = p0.q;
            const float* x = queries + (int64_t)xq * d;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (k < nit) xr[k] = *reinterpret_cast<const float4*>(x + 4 * t + 32 * k);
        }
        float acc[C];
        bool live[C];
        const float* cl[C];
#pragma unroll
        for (int cc = 0; cc < C; ++cc) {
            acc[cc] = 0.f;
            live[cc] = p0.slot + 128 * cc < p0.n;
            cl[cc] = coarse + (int64_t)g0.list[cc] * d;   // list 0 for an entry that is not there: a valid row, unused
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (k < nit) {
                const int e = 4 * t + 32 * k;
                const int j = e / ds, jr = e / dr;
                float4 y[C], pv[C], rv[C];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    y[cc] = *reinterpret_cast<const float4*>(cl[cc] + e);
                    pv[cc] = *reinterpret_cast<const float4*>(pq + (j * IVFR_KS + (int)g0.cb[cc][k]) * ds + (e - j * ds));
                    rv[cc] = *reinterpret_cast<const float4*>(s_rq + (jr * IVFR_KS + (int)g0.rb[cc][k]) * dr + (e - jr * dr));
                }
                const float4 xv = xr[k];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    float4 yy = y[cc];
                    yy.x += pv[cc].x; yy.y += pv[cc].y; yy.z += pv[cc].z; yy.w += pv[cc].w;
                    yy.x += rv[cc].x; yy.y += rv[cc].y; yy.z += rv[cc].z; yy.w += rv[cc].w;
                    const float a = xv.x - yy.x, b = xv.y - yy.y, c2 = xv.z - yy.z, dd = xv.w - yy.w;
                    acc[cc] = fmaf(a, a, acc[cc]); acc[cc] = fmaf(b, b, acc[cc]);
                    acc[cc] = fmaf(c2, c2, acc[cc]); acc[cc] = fmaf(dd, dd, acc[cc]);
                }
            }
        }
#pragma unroll
        for (int cc = 0; cc < C; ++cc) {
            float a = acc[cc];
            a += __shfl_xor(a, 4, 64);
            a += __shfl_xor(a, 2, 64);
            a += __shfl_xor(a, 1, 64);
            const int slot = p0.slot + 128 * cc;
            if (t == 0 && slot < kprime) {
                const int64_t o = (int64_t)p0.q * kprime + slot;
                if (live[cc]) {
                    keys[o] = ((uint64_t)__float_as_uint(a) << 32) | (uint32_t)g0.id[cc];
                    if (refined_out) refined_out[o] = a;
                    if (ids_out) ids_out[o] = g0.id[cc];
                } else {
                    keys[o] = ~0ull;
                    if (refined_out) refined_out[o] = INFINITY;
                    if (ids_out) ids_out[o] = -1;
                }
            }
        }
        p0 = p1; p1 = p2; g0 = g1;
    }
}

int ivfr_rerank_init() {
    IVFR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rerank_lds_kernel<0>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    IVFR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rerank_lds_kernel<8>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    IVFR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rerank_lds_kernel<16>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    IVFR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rerank_lds_kernel<32>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    return IVFR_OK;
}

int ivfr_launch_rerank(const ivfr_index* ix, const float* queries, int q_base, int nq, int kprime,
                       const uint32_t* short_pos, const int32_t* short_n, uint64_t* keys, float* refined_out,
                       int32_t* ids_out, hipStream_t st) {
    if (nq <= 0) return IVFR_OK;
    dim3 grid((kprime + 31) / 32, nq);
    const bool vec0 = (ix->dsub % 4 == 0) && (ix->p.m_refine == 0 || ix->dsub_r % 4 == 0) && ((ix->p.d / 8) % 4 == 0);
    const size_t rq_bytes = (size_t)IVFR_KS * ix->p.d * sizeof(float);
    if (vec0 && ix->p.m_refine > 0 && rq_bytes <= 128 * 1024 && (int64_t)nq * kprime >= (int64_t)ix->n_cu * 1024) {
        const int64_t n_items = (int64_t)nq * ((kprime + 127) / 128);   // an upper bound of the kernel's own count
        const int groups = (int)std::min<int64_t>(n_items, ix->n_cu);
#define IVFR_RERANK_LDS(FM)                                                                                       \
    hipLaunchKernelGGL(rerank_lds_kernel<FM>, dim3(groups), dim3(1024), rq_bytes, st, queries, ix->p.d, ix->p.c,      \
                       ix->p.m, ix->p.m_refine, ix->dsub, ix->dsub_r, ix->coarse, ix->pq, ix->rq, ix->rec,            \
                       ix->rec_stride, kprime, q_base, nq, short_pos, short_n, keys, refined_out, ids_out)
        const int mr = ix->p.m_refine;
        const bool common = ix->p.d == 128 && ix->p.m == 8 && ix->rec_stride % 16 == 0;
        if (common && mr == 8) IVFR_RERANK_LDS(8);
        else if (common && mr == 16) IVFR_RERANK_LDS(16);
        else if (common && mr == 32) IVFR_RERANK_LDS(32);
        else IVFR_RERANK_LDS(0);
#undef IVFR_RERANK_LDS
        IVFR_HIP(hipGetLastError());
        return IVFR_OK;
    }
    const bool vec = (ix->dsub % 4 == 0) && (ix->p.m_refine == 0 || ix->dsub_r % 4 == 0) && ((ix->p.d / 8) % 4 == 0);
#define IVFR_RERANK_ARGS                                                                                       \
    queries, ix->p.d, ix->p.c, ix->p.m, ix->p.m_refine, ix->dsub, ix->dsub_r, ix->coarse, ix->pq, ix->rq,      \
        ix->rec, ix->rec_stride, kprime, q_base, short_pos, short_n, keys, refined_out, ids_out
    if (vec) hipLaunchKernelGGL(rerank_kernel<4>, grid, dim3(256), 0, st, IVFR_RERANK_ARGS);
    else hipLaunchKernelGGL(rerank_kernel<1>, grid, dim3(256), 0, st, IVFR_RERANK_ARGS);
#undef IVFR_RERANK_ARGS
    IVFR_HIP(hipGetLastError());
    return IVFR_OK;
}
