// HIP implementation of the seeded synthetic vector generator (same integer recipe as gen.py;
// the two must produce identical bytes).  Holds none of the search method's arithmetic.
//
//   h(t)  = mix64(key + (t + 1) * GOLDEN)                       (splitmix64 output function)
//   comp  = #{g : cum[g] <= (h(64 i) >> 32)}, clipped to G-1
//   dims 4(r-1)..4(r-1)+3 of vector i take the four 16-bit fields of h(64 i + r), low first
//   value = clip(rint(centre[comp][e] + gauss[u16]), 0, 255)    one fp32 add, round-half-even
#include <hip/hip_runtime.h>
#include <stdint.h>

#define GOLDEN 0x9E3779B97F4A7C15ull

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void synth_kernel(const float* __restrict__ centres,
                                                    const uint32_t* __restrict__ cum,
                                                    const float* __restrict__ gauss, int G, int d, uint64_t key,
                                                    int64_t start, int64_t n, uint8_t* __restrict__ out) {
    const int per = d / 4;
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n * per) return;
    const int64_t row = t / per;
    const int r = (int)(t % per);
    const uint64_t i = (uint64_t)(start + row);
    const uint32_t u = (uint32_t)(mix64(key + (i * 64ull + 1ull) * GOLDEN) >> 32);
    int lo = 0, hi = G;   // first g with cum[g] > u
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (cum[mid] <= u) lo = mid + 1; else hi = mid;
    }
    const int comp = lo < G - 1 ? lo : G - 1;
    const uint64_t h = mix64(key + (i * 64ull + (uint64_t)(r + 1) + 1ull) * GOLDEN);
    uint32_t packed = 0;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint32_t u16 = (uint32_t)(h >> (16 * s)) & 0xFFFFu;
        float v = __fadd_rn(centres[(int64_t)comp * d + 4 * r + s], gauss[u16]);
        v = rintf(v);
        v = fminf(fmaxf(v, 0.f), 255.f);
        packed |= ((uint32_t)v) << (8 * s);
    }
    reinterpret_cast<uint32_t*>(out)[row * per + r] = packed;
}

// All pointers are device memory.  Returns 0 or the hipError_t of the launch.
extern "C" int synth_generate(const float* centres, const uint32_t* cum, const float* gauss, int G, int d,
                              uint64_t key, int64_t start, int64_t n, uint8_t* out, void* stream) {
    if (n <= 0) return 0;
    if (d % 4 != 0 || d / 4 >= 64 || G < 1) return -1;
    const int64_t total = n * (d / 4);
    hipLaunchKernelGGL(synth_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), centres, cum, gauss, G, d, key, start, n, out);
    return (int)hipGetLastError();
}
