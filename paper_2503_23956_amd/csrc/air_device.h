// Device-side helpers: storage-dtype loads / stores and workgroup reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace air {

typedef uint16_t bf16_t;  // bf16 bit pattern

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even fp32 -> bf16 (NaN stays NaN)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float ldf(const float *p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t *p) { return bf16_bits_to_float(*p); }
__device__ __forceinline__ void stf(float *p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t *p, float v) { *p = float_to_bf16_bits(v); }

// Load one row of D elements (16-byte aligned) into fp32 registers.
template <int D>
__device__ __forceinline__ void load_row(const float *p, float (&r)[D]) {
    const float4 *p4 = reinterpret_cast<const float4 *>(p);
#pragma unroll
    for (int i = 0; i < D / 4; ++i) {
        float4 x = p4[i];
        r[4 * i + 0] = x.x;
        r[4 * i + 1] = x.y;
        r[4 * i + 2] = x.z;
        r[4 * i + 3] = x.w;
    }
}
template <int D>
__device__ __forceinline__ void load_row(const bf16_t *p, float (&r)[D]) {
    const uint4 *p4 = reinterpret_cast<const uint4 *>(p);
#pragma unroll
    for (int i = 0; i < D / 8; ++i) {
        uint4 x = p4[i];
        r[8 * i + 0] = __uint_as_float(x.x << 16);
        r[8 * i + 1] = __uint_as_float(x.x & 0xffff0000u);
        r[8 * i + 2] = __uint_as_float(x.y << 16);
        r[8 * i + 3] = __uint_as_float(x.y & 0xffff0000u);
        r[8 * i + 4] = __uint_as_float(x.z << 16);
        r[8 * i + 5] = __uint_as_float(x.z & 0xffff0000u);
        r[8 * i + 6] = __uint_as_float(x.w << 16);
        r[8 * i + 7] = __uint_as_float(x.w & 0xffff0000u);
    }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum over a workgroup of NW waves in a fixed order; every thread gets the result.
// `scratch` holds NW doubles; the call contains two barriers.
template <int NW>
__device__ __forceinline__ double block_sum(double v, double *scratch) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) r += scratch[w];
    return r;
}

// Exclusive prefix sum of one int per thread over a workgroup of NW waves (thread order).
// `scratch` holds NW + 1 ints; *total receives the sum.  Contains two barriers.
template <int NW>
__device__ __forceinline__ int block_excl_scan(int v, int *scratch, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o, 64);
        if (lane >= o) incl += y;
    }
    __syncthreads();
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        if (w < wave) base += scratch[w];
        tot += scratch[w];
    }
    *total = tot;
    return base + incl - v;
}

}  // namespace air
