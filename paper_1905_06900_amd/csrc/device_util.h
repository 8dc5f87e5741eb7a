// Device-side helpers shared by several kernels of libdcpq (HIP translation units only).
#pragma once

#include "common.h"

namespace dcpq {

// Minimum or maximum of v over a workgroup of 256 threads (4 wavefronts): cross-lane shuffles inside
// a wave, then through `red` (4 floats of LDS).  The barriers inside also order the caller's earlier
// LDS writes before its later reads.  Every thread returns the result.
__device__ inline float block_reduce(float v, bool want_max, float *red)
{
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(v, off, kWave);
        v = want_max ? fmaxf(v, o) : fminf(v, o);
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float out = red[0];
    for (int w = 1; w < 4; ++w) out = want_max ? fmaxf(out, red[w]) : fminf(out, red[w]);
    return out;
}

// The 8-bit quantizer of the Tables step (Alg. 3, Sec. 3.3): floor(255 (v - qmin) / (qmax - qmin))
// clamped to 255; everything maps to 0 when qmax <= qmin.  fp32, one rounding per operation in this
// order (subtract, divide, multiply): the result feeds an integer decision.
__device__ inline uint8_t quantize_entry(float v, float qmin, float qmax)
{
    const float den = __fsub_rn(qmax, qmin);
    if (!(den > 0.0f)) return 0;
    const float u = __fmul_rn(__fdiv_rn(__fsub_rn(v, qmin), den), 255.0f);
    return (u >= 255.0f) ? static_cast<uint8_t>(255) : static_cast<uint8_t>(floorf(u));
}

// In-place bitonic sort of n_pow2 64-bit keys by one workgroup (array in LDS or global memory).
__device__ inline void bitonic_sort(uint64_t *a, uint32_t n_pow2)
{
    for (uint32_t size = 2; size <= n_pow2; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (uint32_t t = threadIdx.x; t < (n_pow2 >> 1); t += blockDim.x) {
                const uint32_t lo = 2 * t - (t & (stride - 1));
                const uint32_t hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint64_t x = a[lo], y = a[hi];
                if ((x > y) == up) { a[lo] = y; a[hi] = x; }
            }
        }
    }
    __syncthreads();
}

}  // namespace dcpq
