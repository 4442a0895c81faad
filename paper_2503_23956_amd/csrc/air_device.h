// Device-side helpers: storage-dtype loads / stores and workgroup reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace air {

typedef uint16_t bf16_t;  // bf16 bit pattern
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
// Buffer cache policy sc0 | sc1 of the raw buffer loads / stores that exchange data between workgroups of one launch
// (they may run on XCDs whose L2s are not kept coherent): written through to memory / read past the L2 of this XCD.
constexpr int kSysScope = 17;

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

// All-reduce over each group of 16 consecutive lanes with DPP modifiers (no LDS traffic):
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.
#define AIR_DPP_STEP(OP, v, ctrl) OP((v), __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (v)), (ctrl), 0xf, 0xf, false)))
__device__ __forceinline__ float max16(float v) {
    v = AIR_DPP_STEP(fmaxf, v, 0xB1);
    v = AIR_DPP_STEP(fmaxf, v, 0x4E);
    v = AIR_DPP_STEP(fmaxf, v, 0x141);
    v = AIR_DPP_STEP(fmaxf, v, 0x140);
    return v;
}
__device__ __forceinline__ float add_f(float a, float b) { return a + b; }
__device__ __forceinline__ float sum16(float v) {
    v = AIR_DPP_STEP(add_f, v, 0xB1);
    v = AIR_DPP_STEP(add_f, v, 0x4E);
    v = AIR_DPP_STEP(add_f, v, 0x141);
    v = AIR_DPP_STEP(add_f, v, 0x140);
    return v;
}

// The same for doubles: the DPP move is applied to the two halves.
#define AIR_DPP_STEP64(OP, v, ctrl)                                                                             \
    {                                                                                                           \
        const unsigned long long u_ = __builtin_bit_cast(unsigned long long, (v));                              \
        const int lo_ = __builtin_amdgcn_update_dpp(0, (int)(unsigned)u_, (ctrl), 0xf, 0xf, false);              \
        const int hi_ = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(u_ >> 32), (ctrl), 0xf, 0xf, false);      \
        (v) = OP((v), __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi_ << 32) | (unsigned)lo_));    \
    }
__device__ __forceinline__ double add_d(double a, double b) { return a + b; }
__device__ __forceinline__ double max_d(double a, double b) { return fmax(a, b); }

// All-reduce over the 64 lanes of a wave: four DPP steps inside each row of 16 lanes, then the two
// cross-row steps through the permute unit (a third of the latency of six permutes).
__device__ __forceinline__ float wave_max(float v) {
    v = max16(v);
    v = fmaxf(v, __shfl_xor(v, 16, 64));
    return fmaxf(v, __shfl_xor(v, 32, 64));
}
__device__ __forceinline__ float wave_sum(float v) {
    v = sum16(v);
    v += __shfl_xor(v, 16, 64);
    return v + __shfl_xor(v, 32, 64);
}
__device__ __forceinline__ double sum16(double v) {  // over each row of 16 lanes
    AIR_DPP_STEP64(add_d, v, 0xB1)
    AIR_DPP_STEP64(add_d, v, 0x4E)
    AIR_DPP_STEP64(add_d, v, 0x141)
    AIR_DPP_STEP64(add_d, v, 0x140)
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
    v = sum16(v);
    v += __shfl_xor(v, 16, 64);
    return v + __shfl_xor(v, 32, 64);
}
__device__ __forceinline__ double wave_max(double v) {
    AIR_DPP_STEP64(max_d, v, 0xB1)
    AIR_DPP_STEP64(max_d, v, 0x4E)
    AIR_DPP_STEP64(max_d, v, 0x141)
    AIR_DPP_STEP64(max_d, v, 0x140)
    v = fmax(v, __shfl_xor(v, 16, 64));
    return fmax(v, __shfl_xor(v, 32, 64));
}

// Sequence b and layer li of a workgroup whose grid index is z = b + B * li (z < 2^16, B <= 64): the quotient
// is the high word of z * (floor(2^32 / B) + 1), exact in that range, instead of an integer division in
// front of the kernel's first loads.
template <typename DimsT>
__device__ __forceinline__ void seq_layer_of(const DimsT &dm, int z, int &b, int &li) {
    li = dm.B == 1 ? z : (int)__umulhi((unsigned)z, dm.inv_B);
    b = z - li * dm.B;
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

// exp(d * c / log2(e)) = 2^(d * c) for d <= 0 and a constant c given as a hi/lo pair (c_hi + c_lo = c to
// ~48 bits): the product is split exactly, its integer part goes through ldexp and only the
// fraction through the hardware exp2, so that the result is good to about 2 ulp for any d.
__device__ __forceinline__ float exp2_scaled(float d, float c_hi, float c_lo) {
    const float t = d * c_hi;
    const float lo = fmaf(d, c_hi, -t) + d * c_lo;
    const float nf = rintf(t);
    const float f = (t - nf) + lo;
    return ldexpf(__builtin_amdgcn_exp2f(f), (int)nf);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load and store of the wave (its fence covers global memory), which drains
// prefetches; use this one where only LDS data crosses the barrier.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Exclusive prefix sum of one int per thread over a workgroup of NW waves (thread order).
// `scratch` holds NW + 1 ints; *total receives the sum.  Contains two barriers.
template <int NW>
__device__ __forceinline__ int block_excl_scan(int v, int *scratch, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // inclusive scan over the wave: shifts inside each row of 16 lanes on DPP (lanes shifted in from outside the
    // row read 0), then the totals of the rows in front are added from lanes 15, 31 and 47
    int incl = v;
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x111, 0xf, 0xf, true);  // row_shr:1
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x112, 0xf, 0xf, true);  // row_shr:2
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x114, 0xf, 0xf, true);  // row_shr:4
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x118, 0xf, 0xf, true);  // row_shr:8
    const int t0 = __builtin_amdgcn_readlane(incl, 15), t1 = __builtin_amdgcn_readlane(incl, 31),
              t2 = __builtin_amdgcn_readlane(incl, 47);
    incl += (lane >= 16 ? t0 : 0) + (lane >= 32 ? t1 : 0) + (lane >= 48 ? t2 : 0);
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
