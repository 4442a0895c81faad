// air_score: Alg.1 first loop (Eq.4-10).
//
// Kernels, in stream order, for a range of layers:
//   elite_kernel       Eq.4 (last row) + Eq.5: elite index set of every query head, and the
//                      contribution of the elite text keys to each elite row's softmax.
//   score_pass1_kernel Eq.6-7: per 256-key chunk of K_v, the running (max, sum-exp) of every
//                      elite row.
//   score_rows_kernel  combines the chunk partials into each row's maximum M_r and weight
//                      w_r = 1 / (R_h * G * Z_r).
//   score_pass2_kernel Eq.7-8 + GQA mean: I[i] = sum_rows w_r * exp(s_ri - M_r).
//   stats_kernel       Eq.9-10 per (layer, sequence, KV head) in fp64, two passes.
#include "air_device.h"
#include "air_internal.h"

namespace air {

constexpr int kRowBlock = 8;  // elite rows scored together per pass over the registers holding a key

// ---------------------------------------------------------------------------------------
// Eq.4-5.  One workgroup per (query head, sequence, layer).  The decision of Eq.5 is taken
// in fp64: exp(s_j - max_j s) >= alpha, the form in which the softmax normaliser of Eq.4 has
// cancelled.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void elite_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll, air_strides st,
                                                    SeqArgs seqs, double alpha) {
    const int tid = threadIdx.x;
    const int h = blockIdx.x, b = blockIdx.y, li = blockIdx.z;
    const int l = l0 + li;
    const air_seq sq = seqs.s[b];
    if (li == 0 && h == 0 && tid == 0) t.seq_tab[b] = sq;
    const int t0 = sq.vis_start + sq.vis_len;
    const int kvh = h / dm.G;
    const T *q = (const T *)ll.p[li].q + (int64_t)b * st.q_b + (int64_t)h * st.q_h;
    const T *k = (const T *)ll.p[li].k + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const int64_t hrow = ((int64_t)l * dm.B + b) * dm.Hq + h;
    const int W = dm.max_window;
    const int wl = sq.win_len;

    extern __shared__ double s_dyn[];  // max_window doubles (last-row logits), then max_window ints (elite list)
    double *s_logit = s_dyn;
    int *s_elite = reinterpret_cast<int *>(s_dyn + W);
    __shared__ double s_red[4];
    __shared__ int s_cnt[5];

    const int ref = sq.win_start + wl - 1;
    // last-row logits in fp64: 16 lanes per candidate key (coalesced row reads), D/16 elements per
    // lane, 16 candidates per round of the workgroup, 8 rounds of loads in flight
    constexpr int E = D / 16, UN = 8;
    const int sub = tid & 15, grp = tid >> 4;
    double qd[E];
    {
        T tmp[E];
        __builtin_memcpy(tmp, __builtin_assume_aligned(q + (int64_t)(ref - t0) * st.q_t + sub * E, sizeof(T) * E), sizeof(tmp));
#pragma unroll
        for (int e = 0; e < E; ++e) qd[e] = (double)ldf(&tmp[e]);
    }
    const double sqrt_d = sqrt((double)D);
    for (int j0 = 0; j0 < wl; j0 += 16 * UN) {
        T kv[UN][E];
#pragma unroll
        for (int un = 0; un < UN; ++un) {
            const int j = j0 + un * 16 + grp;
            if (j < wl)
                __builtin_memcpy(kv[un], __builtin_assume_aligned(k + (int64_t)(sq.win_start + j) * st.kv_t + sub * E, sizeof(T) * E),
                                 sizeof(kv[un]));
        }
#pragma unroll
        for (int un = 0; un < UN; ++un) {
            const int j = j0 + un * 16 + grp;
            double acc = 0.0;
            if (j < wl) {
#pragma unroll
                for (int e = 0; e < E; ++e) acc += qd[e] * (double)ldf(&kv[un][e]);
            }
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) acc += __shfl_xor(acc, o, 64);
            if (sub == 0 && j < wl) s_logit[j] = acc / sqrt_d;
        }
    }
    __syncthreads();
    double lmax = -INFINITY;
    for (int j = tid; j < wl; j += 256) lmax = fmax(lmax, s_logit[j]);
    lmax = wave_max(lmax);
    if ((tid & 63) == 0) s_red[tid >> 6] = lmax;
    __syncthreads();
    const double smax = fmax(fmax(s_red[0], s_red[1]), fmax(s_red[2], s_red[3]));

    // ordered compaction of the flagged candidates: thread t owns a contiguous slice (at most 16
    // candidates, AIR_MAX_TEXT / 256), whose flags it keeps as a bit mask
    const int per = (wl + 255) / 256;
    const int j0 = min(wl, tid * per), j1 = min(wl, j0 + per);
    unsigned flags = 0;
    for (int j = j0; j < j1; ++j)
        if (exp(s_logit[j] - smax) >= alpha) flags |= 1u << (j - j0);
    int R;
    int pos = block_excl_scan<4>(__popc(flags), s_cnt, &R);
    for (int j = j0; j < j1; ++j) {
        if (flags & (1u << (j - j0))) {
            s_elite[pos] = sq.win_start + j;
            t.elite_idx[hrow * W + pos] = sq.win_start + j;
            ++pos;
        }
    }
    if (tid == 0) t.elite_cnt[hrow] = R;
    __syncthreads();

    // elite-text columns of Eq.7: (max, sum-exp) of every elite row over the elite text keys.
    // One wave per row; each (row, key) logit is a 64-lane dot product.  Up to 8 keys are
    // scored in one batch of loads; longer rows are scored twice (maximum, then sum).
    // The maximum is kept as the RAW dot product (before the 1/sqrt(d) scale), the sum is of
    // exp((a - max) / sqrt(d)).
    const float scale = 1.0f / sqrtf((float)D);
    const int wave = tid >> 6, lane = tid & 63;
    constexpr int kPer = D / 64;  // elements per lane
    for (int r = wave; r < R; r += 4) {
        const T *qr = q + (int64_t)(s_elite[r] - t0) * st.q_t;
        float qv[kPer];
#pragma unroll
        for (int e = 0; e < kPer; ++e) qv[e] = ldf(qr + lane * kPer + e);
        float m = -INFINITY, z = 0.f;
        if (R <= 8) {
            float a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                a[j] = 0.f;
                if (j < R) {
                    const T *kj = k + (int64_t)s_elite[j] * st.kv_t;
#pragma unroll
                    for (int e = 0; e < kPer; ++e) a[j] = fmaf(qv[e], ldf(kj + lane * kPer + e), a[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < R) {
                    a[j] = wave_sum(a[j]);
                    m = fmaxf(m, a[j]);
                }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < R) z += expf((a[j] - m) * scale);
        } else {
            for (int j = 0; j < R; ++j) {
                const T *kj = k + (int64_t)s_elite[j] * st.kv_t;
                float a = 0.f;
#pragma unroll
                for (int e = 0; e < kPer; ++e) a = fmaf(qv[e], ldf(kj + lane * kPer + e), a);
                m = fmaxf(m, wave_sum(a));
            }
            for (int j = 0; j < R; ++j) {
                const T *kj = k + (int64_t)s_elite[j] * st.kv_t;
                float a = 0.f;
#pragma unroll
                for (int e = 0; e < kPer; ++e) a = fmaf(qv[e], ldf(kj + lane * kPer + e), a);
                z += expf((wave_sum(a) - m) * scale);
            }
        }
        if (lane == 0) {
            t.row_mtext[hrow * W + r] = m;
            t.row_ztext[hrow * W + r] = z;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Eq.6-7 over the visual keys.  One workgroup per (256-key chunk, unit); a unit is one
// (layer, sequence, KV head).  Thread i keeps key i of the chunk in registers and scores it
// against the elite rows of the G query heads of the group, kRowBlock rows at a time.
// PASS 1 writes per-row (max, sum-exp) of the chunk; PASS 2 accumulates Eq.8.
// ---------------------------------------------------------------------------------------
template <typename T, int D, int PASS>
__global__ __launch_bounds__(256) void score_pass_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll,
                                                         air_strides st) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int chunk = blockIdx.x;
    const int u = blockIdx.y;  // unit inside this launch
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const air_seq sq = t.seq_tab[b];
    if (chunk * kChunkKeys >= sq.vis_len) return;
    const int t0 = sq.vis_start + sq.vis_len;
    const int i = chunk * kChunkKeys + tid;
    const bool valid = i < sq.vis_len;
    const T *q = (const T *)ll.p[li].q + (int64_t)b * st.q_b;
    const T *k = (const T *)ll.p[li].k + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const int W = dm.max_window;

    float kreg[D];
    if (valid) {
        load_row<D>(k + (int64_t)(sq.vis_start + i) * st.kv_t, kreg);
    } else {
#pragma unroll
        for (int c = 0; c < D; ++c) kreg[c] = 0.f;
    }

    __shared__ float s_q[kRowBlock][D];
    __shared__ float s_red[kRowBlock][4];
    __shared__ float s_M[kRowBlock], s_w[kRowBlock];
    const float scale = 1.0f / sqrtf((float)D);
    float imp = 0.f;

    for (int g = 0; g < dm.G; ++g) {
        const int h = kvh * dm.G + g;
        const int64_t hrow = ((int64_t)l * dm.B + b) * dm.Hq + h;
        const int R = t.elite_cnt[hrow];
        const T *qh = q + (int64_t)h * st.q_h;
        for (int r0 = 0; r0 < R; r0 += kRowBlock) {
            const int nb = min(kRowBlock, R - r0);
            __syncthreads();
            for (int idx = tid; idx < nb * D; idx += 256) {
                const int rr = idx / D, c = idx % D;
                const int tok = t.elite_idx[hrow * W + r0 + rr];
                s_q[rr][c] = ldf(qh + (int64_t)(tok - t0) * st.q_t + c);
            }
            if (PASS == 2 && tid < nb) {
                s_M[tid] = t.row_M[hrow * W + r0 + tid];
                s_w[tid] = t.row_w[hrow * W + r0 + tid];
            }
            __syncthreads();
            float s[kRowBlock];
#pragma unroll
            for (int rr = 0; rr < kRowBlock; ++rr) {
                float acc = 0.f;
                if (rr < nb) {
#pragma unroll
                    for (int c = 0; c < D; ++c) acc = fmaf(s_q[rr][c], kreg[c], acc);
                }
                s[rr] = acc * scale;
            }
            if (PASS == 1) {
#pragma unroll
                for (int rr = 0; rr < kRowBlock; ++rr) {
                    float m = wave_max(valid ? s[rr] : -INFINITY);
                    if (lane == 0) s_red[rr][wave] = m;
                }
                __syncthreads();
                float mrow[kRowBlock];
#pragma unroll
                for (int rr = 0; rr < kRowBlock; ++rr)
                    mrow[rr] = fmaxf(fmaxf(s_red[rr][0], s_red[rr][1]), fmaxf(s_red[rr][2], s_red[rr][3]));
                __syncthreads();
#pragma unroll
                for (int rr = 0; rr < kRowBlock; ++rr) {
                    float e = (valid && rr < nb) ? expf(s[rr] - mrow[rr]) : 0.f;
                    e = wave_sum(e);
                    if (lane == 0) s_red[rr][wave] = e;
                }
                __syncthreads();
                if (tid < nb) {
                    const float z = (s_red[tid][0] + s_red[tid][1]) + (s_red[tid][2] + s_red[tid][3]);
                    t.part[(hrow * W + r0 + tid) * dm.n_chunks + chunk] = make_float2(mrow[tid], z);
                }
            } else {
#pragma unroll
                for (int rr = 0; rr < kRowBlock; ++rr)
                    if (rr < nb) imp = fmaf(s_w[rr], expf(s[rr] - s_M[rr]), imp);
            }
        }
    }
    if (PASS == 2 && valid) {
        const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
        t.scores[unit * dm.max_vis + i] = imp;
    }
}

// One workgroup per (layer, sequence, query head): row maximum over all chunks and the
// elite text keys, normaliser in fp64, weight 1 / (R_h * G * Z_r).
__global__ __launch_bounds__(64) void score_rows_kernel(Dims dm, DevTables t, int l0) {
    const int64_t hrow = (int64_t)l0 * dm.B * dm.Hq + blockIdx.x;
    const int b = (blockIdx.x / dm.Hq) % dm.B;
    const air_seq sq = t.seq_tab[b];
    const int nch = (sq.vis_len + kChunkKeys - 1) / kChunkKeys;
    const int R = t.elite_cnt[hrow];
    const int W = dm.max_window;
    for (int r = threadIdx.x; r < R; r += 64) {
        const int64_t slot = hrow * W + r;
        const float2 *p = t.part + slot * dm.n_chunks;
        const float mt = t.row_mtext[slot] * (1.0f / sqrtf((float)dm.D));  // stored unscaled
        float M = mt;
        for (int c = 0; c < nch; ++c) M = fmaxf(M, p[c].x);
        double Z = (double)t.row_ztext[slot] * exp((double)mt - (double)M);
        for (int c = 0; c < nch; ++c) Z += (double)p[c].y * exp((double)p[c].x - (double)M);
        t.row_M[slot] = M;
        t.row_w[slot] = (float)(1.0 / ((double)R * (double)dm.G * Z));
    }
}

// Eq.9-10 for one unit: fp64, mean first, then central moments.
__global__ __launch_bounds__(256) void stats_kernel(Dims dm, DevTables t, int l0) {
    const int64_t unit = (int64_t)l0 * dm.B * dm.Hkv + blockIdx.x;
    const int b = (blockIdx.x / dm.Hkv) % dm.B;
    const int n = t.seq_tab[b].vis_len;
    const float *imp = t.scores + unit * dm.max_vis;
    __shared__ double scratch[4];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += (double)imp[i];
    const double s_t = block_sum<4>(s, scratch);
    const double mu = s_t / (double)n;
    double s2 = 0.0, s3 = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) {
        const double c = (double)imp[i] - mu;
        s2 += c * c;
        s3 += c * c * c;
    }
    s2 = block_sum<4>(s2, scratch);
    s3 = block_sum<4>(s3, scratch);
    if (threadIdx.x == 0) {
        double sk = 0.0;
        if (n >= 3) {
            const double var = s2 / (double)(n - 1);
            if (var > 0.0) {
                const double sigma = sqrt(var);
                sk = (double)n / (((double)n - 1.0) * ((double)n - 2.0)) * (s3 / (sigma * sigma * sigma));
            }
        }
        t.unit_st[unit] = s_t;
        t.unit_sk[unit] = sk;
    }
}

// ---------------------------------------------------------------------------------------
template <typename T, int D>
static hipError_t elite_launch(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl,
                               const LaunchLayers &ll, const air_strides &st, const SeqArgs &seqs, double alpha) {
    const size_t lds = (size_t)dm.max_window * (sizeof(double) + sizeof(int));
    hipLaunchKernelGGL((elite_kernel<T, D>), dim3(dm.Hq, dm.B, nl), dim3(256), lds, s, dm, t, l0, ll, st, seqs, alpha);
    return hipGetLastError();
}

hipError_t launch_elite(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                        const LaunchLayers &ll, const air_strides &st, const SeqArgs &seqs, double alpha) {
    if (dtype == AIR_BF16)
        return dm.D == 128 ? elite_launch<bf16_t, 128>(s, dm, t, l0, nl, ll, st, seqs, alpha)
                           : elite_launch<bf16_t, 64>(s, dm, t, l0, nl, ll, st, seqs, alpha);
    return dm.D == 128 ? elite_launch<float, 128>(s, dm, t, l0, nl, ll, st, seqs, alpha)
                       : elite_launch<float, 64>(s, dm, t, l0, nl, ll, st, seqs, alpha);
}

template <typename T, int D, int PASS>
static hipError_t pass_launch(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl,
                              const LaunchLayers &ll, const air_strides &st) {
    hipLaunchKernelGGL((score_pass_kernel<T, D, PASS>), dim3(dm.n_chunks, nl * dm.B * dm.Hkv), dim3(256), 0, s, dm, t,
                       l0, ll, st);
    return hipGetLastError();
}

template <int PASS>
static hipError_t pass_dispatch(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                                const LaunchLayers &ll, const air_strides &st) {
    if (dtype == AIR_BF16)
        return dm.D == 128 ? pass_launch<bf16_t, 128, PASS>(s, dm, t, l0, nl, ll, st)
                           : pass_launch<bf16_t, 64, PASS>(s, dm, t, l0, nl, ll, st);
    return dm.D == 128 ? pass_launch<float, 128, PASS>(s, dm, t, l0, nl, ll, st)
                       : pass_launch<float, 64, PASS>(s, dm, t, l0, nl, ll, st);
}

hipError_t launch_score_pass1(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                              const LaunchLayers &ll, const air_strides &st) {
    return pass_dispatch<1>(s, dm, t, dtype, l0, nl, ll, st);
}
hipError_t launch_score_pass2(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                              const LaunchLayers &ll, const air_strides &st) {
    return pass_dispatch<2>(s, dm, t, dtype, l0, nl, ll, st);
}

hipError_t launch_score_rows(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl) {
    hipLaunchKernelGGL(score_rows_kernel, dim3(nl * dm.B * dm.Hq), dim3(64), 0, s, dm, t, l0);
    return hipGetLastError();
}

hipError_t launch_stats(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl) {
    hipLaunchKernelGGL(stats_kernel, dim3(nl * dm.B * dm.Hkv), dim3(256), 0, s, dm, t, l0);
    return hipGetLastError();
}

}  // namespace air
