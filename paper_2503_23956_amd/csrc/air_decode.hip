// air_decode_attn: Eq.2 append, then softmax(q K'^T / sqrt(d)) V' over the compacted cache.
//
//   append_kernel   writes k_new / v_new behind the last row of each (layer, sequence, KV head).
//   decode_kernel   split-K: workgroup (split, unit) streams its share of K' and V' once and
//                   leaves an online-softmax partial (max, sum, unnormalised output) for the
//                   G query heads that share the KV head.
//   combine_kernel  merges the kDecodeSplits partials and stores the output in the storage dtype.
#include "air_device.h"
#include "air_internal.h"

namespace air {

constexpr int kMaxGroup = 16;

template <typename T, int D>
__global__ __launch_bounds__(64) void append_kernel(Dims dm, DevTables t, int l0, int lbase, LaunchLayers ll,
                                                    const T *k_new, const T *v_new) {
    const int u = blockIdx.x;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const int row = t.base_len[(int64_t)b * dm.L + l] + ll.appended[li];
    const int64_t dst_row = ((int64_t)b * dm.Hkv + kvh) * dm.pool_rows + t.layer_off[(int64_t)b * dm.L + l] + row;
    const int64_t src = (((int64_t)(lbase + li) * dm.B + b) * dm.Hkv + kvh) * D;
    constexpr int kVec = D * (int)sizeof(T) / 16;
    if (threadIdx.x < kVec) {
        const int c = threadIdx.x * (16 / (int)sizeof(T));
        *reinterpret_cast<uint4 *>((T *)t.kcache + dst_row * D + c) = *reinterpret_cast<const uint4 *>(k_new + src + c);
        *reinterpret_cast<uint4 *>((T *)t.vcache + dst_row * D + c) = *reinterpret_cast<const uint4 *>(v_new + src + c);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_kernel(Dims dm, DevTables t, int l0, int lbase, LaunchLayers ll,
                                                     const T *q_new) {
    constexpr int NP = 256 / D;  // key-parallel parts in the P*V phase
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int split = blockIdx.x;
    const int u = blockIdx.y;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const int G = dm.G;
    const int len = t.base_len[(int64_t)b * dm.L + l] + ll.appended[li] + 1;
    const int cs = (len + kDecodeSplits - 1) / kDecodeSplits;
    const int k0 = split * cs, k1 = min(len, k0 + cs);
    const int64_t row0 = ((int64_t)b * dm.Hkv + kvh) * dm.pool_rows + t.layer_off[(int64_t)b * dm.L + l];
    const T *kc = (const T *)t.kcache + row0 * D;
    const T *vc = (const T *)t.vcache + row0 * D;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;

    __shared__ float s_q[kMaxGroup][D];
    __shared__ float s_p[kMaxGroup][256];
    __shared__ float s_m[kMaxGroup], s_l[kMaxGroup], s_corr[kMaxGroup];
    __shared__ float s_o[NP][kMaxGroup][D];

    const T *q = q_new + (((int64_t)(lbase + li) * dm.B + b) * dm.Hq + (int64_t)kvh * G) * D;
    for (int idx = tid; idx < G * D; idx += 256) s_q[idx / D][idx % D] = ldf(q + idx);
    if (tid < kMaxGroup) {
        s_m[tid] = -INFINITY;
        s_l[tid] = 0.f;
    }
    const float scale = 1.0f / sqrtf((float)D);
    const int dcol = tid % D, part = tid / D;
    float acc[kMaxGroup];
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g) acc[g] = 0.f;
    __syncthreads();

    for (int kb = k0; kb < k1; kb += 256) {
        const int nk = min(256, k1 - kb);
        {
            float kreg[D];
            if (tid < nk) load_row<D>(kc + (int64_t)(kb + tid) * D, kreg);
            for (int g = 0; g < G; ++g) {
                float a = 0.f;
                if (tid < nk) {
#pragma unroll
                    for (int c = 0; c < D; ++c) a = fmaf(s_q[g][c], kreg[c], a);
                }
                s_p[g][tid] = tid < nk ? a * scale : -INFINITY;
            }
        }
        __syncthreads();
        for (int g = wave; g < G; g += 4) {
            float v0 = s_p[g][lane], v1 = s_p[g][lane + 64], v2 = s_p[g][lane + 128], v3 = s_p[g][lane + 192];
            const float mb = wave_max(fmaxf(fmaxf(v0, v1), fmaxf(v2, v3)));
            const float mo = s_m[g];
            const float mn = fmaxf(mo, mb);
            v0 = expf(v0 - mn);
            v1 = expf(v1 - mn);
            v2 = expf(v2 - mn);
            v3 = expf(v3 - mn);
            s_p[g][lane] = v0;
            s_p[g][lane + 64] = v1;
            s_p[g][lane + 128] = v2;
            s_p[g][lane + 192] = v3;
            const float lb = wave_sum((v0 + v1) + (v2 + v3));
            if (lane == 0) {
                const float corr = expf(mo - mn);  // 0 on the first block (mo = -inf)
                s_corr[g] = corr;
                s_l[g] = s_l[g] * corr + lb;
                s_m[g] = mn;
            }
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g)
            if (g < G) acc[g] *= s_corr[g];
        for (int tk = part; tk < nk; tk += NP) {
            const float vv = ldf(vc + (int64_t)(kb + tk) * D + dcol);
#pragma unroll
            for (int g = 0; g < kMaxGroup; ++g)
                if (g < G) acc[g] = fmaf(s_p[g][tk], vv, acc[g]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g)
        if (g < G) s_o[part][g][dcol] = acc[g];
    __syncthreads();
    float *po = t.dec_o + (unit * kDecodeSplits + split) * (int64_t)G * D;
    for (int idx = tid; idx < G * D; idx += 256) {
        const int g = idx / D, c = idx % D;
        float o = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) o += s_o[p][g][c];
        po[idx] = o;
    }
    if (tid < G) t.dec_ml[(unit * kDecodeSplits + split) * G + tid] = make_float2(s_m[tid], s_l[tid]);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void combine_kernel(Dims dm, DevTables t, int l0, int lbase, T *out) {
    const int u = blockIdx.x;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const int G = dm.G;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
    const float2 *ml = t.dec_ml + unit * kDecodeSplits * G;
    const float *po = t.dec_o + unit * kDecodeSplits * (int64_t)G * D;
    T *o = out + (((int64_t)(lbase + li) * dm.B + b) * dm.Hq + (int64_t)kvh * G) * D;
    for (int idx = threadIdx.x; idx < G * D; idx += 256) {
        const int g = idx / D;
        float M = -INFINITY;
#pragma unroll
        for (int s = 0; s < kDecodeSplits; ++s) M = fmaxf(M, ml[s * G + g].x);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int s = 0; s < kDecodeSplits; ++s) {
            const float2 x = ml[s * G + g];
            const float wgt = x.y > 0.f ? expf(x.x - M) : 0.f;
            num = fmaf(wgt, po[(int64_t)s * G * D + idx], num);
            den = fmaf(wgt, x.y, den);
        }
        stf(o + idx, num / den);
    }
}

template <typename T, int D>
static hipError_t append_launch(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, int lbase,
                                const LaunchLayers &ll, const void *k_new, const void *v_new) {
    hipLaunchKernelGGL((append_kernel<T, D>), dim3(nl * dm.B * dm.Hkv), dim3(64), 0, s, dm, t, l0, lbase, ll,
                       (const T *)k_new, (const T *)v_new);
    return hipGetLastError();
}

hipError_t launch_append(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl, int lbase,
                         const LaunchLayers &ll, const void *k_new, const void *v_new) {
    if (dtype == AIR_BF16)
        return dm.D == 128 ? append_launch<bf16_t, 128>(s, dm, t, l0, nl, lbase, ll, k_new, v_new)
                           : append_launch<bf16_t, 64>(s, dm, t, l0, nl, lbase, ll, k_new, v_new);
    return dm.D == 128 ? append_launch<float, 128>(s, dm, t, l0, nl, lbase, ll, k_new, v_new)
                       : append_launch<float, 64>(s, dm, t, l0, nl, lbase, ll, k_new, v_new);
}

template <typename T, int D>
static hipError_t decode_launch(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, int lbase,
                                const LaunchLayers &ll, const void *q_new, void *out) {
    hipLaunchKernelGGL((decode_kernel<T, D>), dim3(kDecodeSplits, nl * dm.B * dm.Hkv), dim3(256), 0, s, dm, t, l0,
                       lbase, ll, (const T *)q_new);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((combine_kernel<T, D>), dim3(nl * dm.B * dm.Hkv), dim3(256), 0, s, dm, t, l0, lbase, (T *)out);
    return hipGetLastError();
}

hipError_t launch_decode(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl, int lbase,
                         const LaunchLayers &ll, const void *q_new, void *out) {
    if (dtype == AIR_BF16)
        return dm.D == 128 ? decode_launch<bf16_t, 128>(s, dm, t, l0, nl, lbase, ll, q_new, out)
                           : decode_launch<bf16_t, 64>(s, dm, t, l0, nl, lbase, ll, q_new, out);
    return dm.D == 128 ? decode_launch<float, 128>(s, dm, t, l0, nl, lbase, ll, q_new, out)
                       : decode_launch<float, 64>(s, dm, t, l0, nl, lbase, ll, q_new, out);
}

}  // namespace air
