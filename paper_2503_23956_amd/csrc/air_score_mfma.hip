// air_score, bf16 / head_dim 128: the window-query x visual-key product (Eq.6-7) on MFMA.
//
// A workgroup of 4 waves owns one 256-key chunk of one unit (layer, sequence, KV head); each
// wave keeps its 64 keys (4 tiles of 16) in registers as MFMA B operands, loaded straight from
// global memory: lane (n = lane % 16, c = lane / 16) holds elements 8c..8c+7 of every 32-element
// slice of key n of the tile.  The elite rows of the G query heads of the group are the A
// operand, 16 rows per block, so that S[row][key] comes out with lane (key n, c) holding rows
// 4c..4c+3 of the tile: the sum over window rows that Eq.8 needs is then in-lane plus two
// cross-lane steps.
//
//   PASS 1  per (row, chunk): max and sum-exp over the chunk's keys.
//   PASS 2  prologue: row maxima M_r and weights w_r = 1 / (R_h G Z_r) from the chunk partials
//           and the elite-text columns; main: I[key] = sum_rows w_r exp(s - M_r) (Eq.8 and the
//           mean over the group's heads); epilogue: fp64 power sums of I over the chunk, from
//           which the budget kernel forms Eq.9-10.
// K_v is read once per pass; the launcher runs the two passes over groups of layers small
// enough that the second pass finds its keys in the 256 MB memory-side cache.
#include "air_device.h"
#include "air_internal.h"

namespace air {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kRowsLds = 1024;  // rows whose (M, w) are staged in LDS at a time

template <int PASS>
__global__ __launch_bounds__(256) void score_mfma_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll,
                                                         air_strides st) {
    constexpr int D = 128;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 15, c = lane >> 4;
    const int chunk = blockIdx.x;
    const int u = blockIdx.y;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const air_seq sq = t.seq_tab[b];
    if (chunk * kChunkKeys >= sq.vis_len) return;
    const int t0 = sq.vis_start + sq.vis_len;
    const int G = dm.G, W = dm.max_window;
    const bf16_t *q = (const bf16_t *)ll.p[li].q + (int64_t)b * st.q_b;
    const bf16_t *k = (const bf16_t *)ll.p[li].k + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const int64_t hrow0 = ((int64_t)l * dm.B + b) * dm.Hq + (int64_t)kvh * G;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;

    __shared__ int s_pref[17];  // row-list offset of each of the (at most 16) heads of the group
    __shared__ float s_M[kRowsLds], s_w[kRowsLds];
    __shared__ float s_pm[4][16], s_pz[4][16];
    __shared__ double s_mom[4][3];

    // keys of this wave: 4 tiles of 16
    const int key0 = chunk * kChunkKeys + wave * 64;
    uint4 kreg[4][4];
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) {
        const int key = key0 + 16 * tile + n;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {
            kreg[tile][sl] = make_uint4(0, 0, 0, 0);
            if (key < sq.vis_len)
                kreg[tile][sl] = *reinterpret_cast<const uint4 *>(k + (int64_t)(sq.vis_start + key) * st.kv_t + 32 * sl + 8 * c);
        }
    }
    if (tid == 0) {
        int run = 0;
        for (int g = 0; g < G; ++g) {
            s_pref[g] = run;
            run += t.elite_cnt[hrow0 + g];
        }
        s_pref[G] = run;
    }
    __syncthreads();
    const int R_total = s_pref[G];
    const float scale = 0.08838834764831845f;  // 1/sqrt(128)
    bool valid[4];
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) valid[tile] = key0 + 16 * tile + n < sq.vis_len;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};

    for (int rs = 0; rs < R_total; rs += kRowsLds) {
        const int rows_here = min(kRowsLds, R_total - rs);
        if (PASS == 2) {
            // row maxima and weights of this block of rows: one wave per row, lanes over the chunk partials
            __syncthreads();
            const int nch = (sq.vis_len + kChunkKeys - 1) / kChunkKeys;
            for (int rr = wave; rr < rows_here; rr += 4) {
                const int rho = rs + rr;
                int g = 0;
                while (g + 1 < G && s_pref[g + 1] <= rho) ++g;
                const int64_t slot = (hrow0 + g) * W + (rho - s_pref[g]);
                const float2 *p = t.part + slot * dm.n_chunks;
                const float mt = t.row_mtext[slot];
                float M = mt;
                for (int cc = lane; cc < nch; cc += 64) M = fmaxf(M, p[cc].x);
                M = wave_max(M);
                double Z = 0.0;
                for (int cc = lane; cc < nch; cc += 64) {
                    const float2 x = p[cc];
                    Z += (double)(x.y * expf(x.x - M));
                }
                Z = wave_sum(Z);
                Z += (double)(t.row_ztext[slot] * expf(mt - M));
                if (lane == 0) {
                    s_M[rr] = M;
                    s_w[rr] = (float)(1.0 / ((double)(s_pref[g + 1] - s_pref[g]) * (double)G * Z));
                }
            }
            __syncthreads();
        }
        for (int rb = 0; rb < rows_here; rb += 16) {
            // A operand.  MFMA row m = 4c'+i' carries list row rb + 4i' + c' (c' = m / 4, i' = m % 4), so that
            // output lane group c holds rows rb + c, rb + 4 + c, ...: with fewer than 16 rows in the
            // block every lane group has the same number of live rows and the i loop stops early.
            const int rho = rs + rb + 4 * (n & 3) + (n >> 2);
            uint4 qa[4];
            {
                int g = 0;
                while (g + 1 < G && s_pref[g + 1] <= rho) ++g;
                const bool have = rho < R_total;
                int tok = t0;
                if (have) tok = t.elite_idx[(hrow0 + g) * W + (rho - s_pref[g])];
                const bf16_t *qr = q + (int64_t)(kvh * G + g) * st.q_h + (int64_t)(tok - t0) * st.q_t;
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) {
                    qa[sl] = make_uint4(0, 0, 0, 0);
                    if (have) qa[sl] = *reinterpret_cast<const uint4 *>(qr + 32 * sl + 8 * c);
                }
            }
            f32x4 s[4];
#pragma unroll
            for (int tile = 0; tile < 4; ++tile) {
                s[tile] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int sl = 0; sl < 4; ++sl)
                    s[tile] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qa[sl]),
                                                                      __builtin_bit_cast(bf16x8, kreg[tile][sl]), s[tile], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i) s[tile][i] *= scale;
            }
            const int n_i = min(4, (rows_here - rb + 3) >> 2);  // live values of i (uniform over the workgroup)
            if (PASS == 1) {
                float m[4], z[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    m[i] = -INFINITY;
                    z[i] = 0.f;
                    if (i >= n_i) continue;
                    float mx = -INFINITY;
#pragma unroll
                    for (int tile = 0; tile < 4; ++tile) mx = fmaxf(mx, valid[tile] ? s[tile][i] : -INFINITY);
#pragma unroll
                    for (int o = 1; o < 16; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
                    float zz = 0.f;
#pragma unroll
                    for (int tile = 0; tile < 4; ++tile) zz += valid[tile] ? expf(s[tile][i] - mx) : 0.f;
#pragma unroll
                    for (int o = 1; o < 16; o <<= 1) zz += __shfl_xor(zz, o, 64);
                    m[i] = mx;
                    z[i] = zz;
                }
                __syncthreads();
                if (n == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        s_pm[wave][4 * i + c] = m[i];  // indexed by list row within the block
                        s_pz[wave][4 * i + c] = z[i];
                    }
                }
                __syncthreads();
                if (tid < 16 && rs + rb + tid < R_total) {
                    const int rho2 = rs + rb + tid;
                    float M = fmaxf(fmaxf(s_pm[0][tid], s_pm[1][tid]), fmaxf(s_pm[2][tid], s_pm[3][tid]));
                    float Z = 0.f;
#pragma unroll
                    for (int w = 0; w < 4; ++w) Z += s_pz[w][tid] > 0.f ? s_pz[w][tid] * expf(s_pm[w][tid] - M) : 0.f;
                    int g = 0;
                    while (g + 1 < G && s_pref[g + 1] <= rho2) ++g;
                    const int64_t slot = (hrow0 + g) * W + (rho2 - s_pref[g]);
                    t.part[slot * dm.n_chunks + chunk] = make_float2(M, Z);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (i >= n_i) continue;
                    const int rr = rb + 4 * i + c;
                    const bool have = rr < rows_here;
                    const float M = have ? s_M[rr] : 0.f;
                    const float w = have ? s_w[rr] : 0.f;
#pragma unroll
                    for (int tile = 0; tile < 4; ++tile) acc[tile] = fmaf(w, expf(s[tile][i] - M), acc[tile]);
                }
            }
        }
    }
    if (PASS == 2) {
        double m1 = 0.0, m2 = 0.0, m3 = 0.0;
#pragma unroll
        for (int tile = 0; tile < 4; ++tile) {
            float v = acc[tile];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (c == 0 && valid[tile]) {
                t.scores[unit * dm.max_vis + key0 + 16 * tile + n] = v;
                const double x = (double)v;
                m1 += x;
                m2 += x * x;
                m3 += x * x * x;
            }
        }
        m1 = wave_sum(m1);
        m2 = wave_sum(m2);
        m3 = wave_sum(m3);
        if (lane == 0) {
            s_mom[wave][0] = m1;
            s_mom[wave][1] = m2;
            s_mom[wave][2] = m3;
        }
        __syncthreads();
        if (tid < 3) {
            double *mo = t.moments + (unit * dm.n_chunks + chunk) * 3;
            mo[tid] = ((s_mom[0][tid] + s_mom[1][tid]) + s_mom[2][tid]) + s_mom[3][tid];
        }
    }
}

hipError_t launch_score_mfma(hipStream_t s, const Dims &dm, const DevTables &t, int pass, int l0, int nl,
                             const LaunchLayers &ll, const air_strides &st) {
    const dim3 grid(dm.n_chunks, nl * dm.B * dm.Hkv);
    if (pass == 1)
        hipLaunchKernelGGL(score_mfma_kernel<1>, grid, dim3(256), 0, s, dm, t, l0, ll, st);
    else
        hipLaunchKernelGGL(score_mfma_kernel<2>, grid, dim3(256), 0, s, dm, t, l0, ll, st);
    return hipGetLastError();
}

}  // namespace air
