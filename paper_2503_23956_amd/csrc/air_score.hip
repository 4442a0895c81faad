// air_score: Alg.1 first loop (Eq.4-10).
//
// Kernels, in stream order, for a range of layers:
//   elite_kernel       Eq.4 (last row) + Eq.5: elite index set of every query head (one workgroup per KV group), and the
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
// Eq.4-5.  One workgroup per (KV head, sequence, layer): the candidate text keys are read once
// for all G query heads of the group.  The decision of Eq.5 is taken in fp64:
// exp(s_j - max_j s) >= alpha, the form in which the softmax normaliser of Eq.4 has cancelled.
//   phase 1 (all threads): last-row logits of every head of the batch against every candidate,
//           16 lanes per candidate key (coalesced row reads), D/16 elements per lane, fp64.
//   phase 2 (one wave per head): maximum, threshold, ordered compaction of the elite positions,
//           then the elite-text columns of Eq.7 for that head's elite rows.
// Heads are processed in batches of `gb` so that gb * max_window logits fit the LDS.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double sum16_f64(double v) {
    // all-reduce over 16 consecutive lanes, DPP on the two halves of the double
#define AIR_DPP_F64(ctrl)                                                                                  \
    {                                                                                                      \
        const unsigned long long u = __builtin_bit_cast(unsigned long long, v);                            \
        const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)u, (ctrl), 0xf, 0xf, false);           \
        const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(u >> 32), (ctrl), 0xf, 0xf, false);   \
        v += __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);           \
    }
    AIR_DPP_F64(0xB1)
    AIR_DPP_F64(0x4E)
    AIR_DPP_F64(0x141)
    AIR_DPP_F64(0x140)
#undef AIR_DPP_F64
    return v;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void elite_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll, air_strides st,
                                                    SeqArgs seqs, double alpha, int gb) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int kvh = blockIdx.x, b = blockIdx.y, li = blockIdx.z;
    const int l = l0 + li;
    const air_seq sq = seqs.s[b];
    if (li == 0 && kvh == 0 && tid == 0) t.seq_tab[b] = sq;
    const int t0 = sq.vis_start + sq.vis_len;
    const int G = dm.G, W = dm.max_window, wl = sq.win_len;
    const T *qb = (const T *)ll.p[li].q + (int64_t)b * st.q_b;
    const T *k = (const T *)ll.p[li].k + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const int ref = sq.win_start + wl - 1;

    extern __shared__ double s_dyn[];  // gb * max_window doubles (last-row logits), then as many ints (elite lists)
    double *s_logit = s_dyn;
    int *s_elite = reinterpret_cast<int *>(s_dyn + (size_t)gb * W);

    constexpr int E = D / 16, UN = 4, HB = 8;  // elements per lane, candidate rounds in flight, heads per register batch
    const int sub = tid & 15, grp = tid >> 4;
    const double sqrt_d = sqrt((double)D);
    const float scale = 1.0f / sqrtf((float)D);

    for (int g0 = 0; g0 < G; g0 += gb) {
        const int ng = min(gb, G - g0);
        // ---- phase 1
        for (int hb = 0; hb < ng; hb += HB) {
            const int nh = min(HB, ng - hb);
            double qd[HB][E];
#pragma unroll
            for (int hh = 0; hh < HB; ++hh) {
                T tmp[E];
                const int h = kvh * G + g0 + hb + (hh < nh ? hh : 0);
                __builtin_memcpy(tmp, __builtin_assume_aligned(qb + (int64_t)h * st.q_h + (int64_t)(ref - t0) * st.q_t + sub * E,
                                                               sizeof(T) * E), sizeof(tmp));
#pragma unroll
                for (int e = 0; e < E; ++e) qd[hh][e] = (double)ldf(&tmp[e]);
            }
            for (int j0 = 0; j0 < wl; j0 += 16 * UN) {
                T kv[UN][E];
#pragma unroll
                for (int un = 0; un < UN; ++un) {
                    const int j = j0 + un * 16 + grp;
                    if (j < wl)
                        __builtin_memcpy(kv[un], __builtin_assume_aligned(k + (int64_t)(sq.win_start + j) * st.kv_t + sub * E,
                                                                          sizeof(T) * E), sizeof(kv[un]));
                }
#pragma unroll
                for (int un = 0; un < UN; ++un) {
                    const int j = j0 + un * 16 + grp;
                    double kd[E];
#pragma unroll
                    for (int e = 0; e < E; ++e) kd[e] = j < wl ? (double)ldf(&kv[un][e]) : 0.0;
#pragma unroll
                    for (int hh = 0; hh < HB; ++hh) {
                        if (hh >= nh) break;
                        double acc = 0.0;
#pragma unroll
                        for (int e = 0; e < E; ++e) acc += qd[hh][e] * kd[e];
                        acc = sum16_f64(acc);
                        if (sub == 0 && j < wl) s_logit[(size_t)(hb + hh) * W + j] = acc / sqrt_d;
                    }
                }
            }
        }
        __syncthreads();
        // ---- phase 2
        for (int hh = wave; hh < ng; hh += 4) {
            const int h = kvh * G + g0 + hh;
            const int64_t hrow = ((int64_t)l * dm.B + b) * dm.Hq + h;
            const double *logit = s_logit + (size_t)hh * W;
            int *elite = s_elite + (size_t)hh * W;
            double lmax = -INFINITY;
            for (int j = lane; j < wl; j += 64) lmax = fmax(lmax, logit[j]);
            const double smax = wave_max(lmax);
            int R = 0;
            for (int j0 = 0; j0 < wl; j0 += 64) {
                const int j = j0 + lane;
                const bool flag = j < wl && exp(logit[j] - smax) >= alpha;
                const unsigned long long bal = __ballot(flag);
                if (flag) {
                    const int pos = R + __popcll(bal & ((1ull << lane) - 1ull));
                    elite[pos] = sq.win_start + j;
                    t.elite_idx[hrow * W + pos] = sq.win_start + j;
                }
                R += __popcll(bal);
            }
            if (lane == 0) t.elite_cnt[hrow] = R;
            // elite-text columns of Eq.7: (max, sum-exp) of every elite row over the elite text keys; each
            // (row, key) logit is a 64-lane dot product.  Up to 8 keys are scored in one batch of loads,
            // longer rows are scored twice (maximum, then sum).  The maximum is kept as the RAW dot
            // product (before the 1/sqrt(d) scale), the sum is of exp((a - max) / sqrt(d)).
            constexpr int kPer = D / 64;  // elements per lane
            const T *q = qb + (int64_t)h * st.q_h;
            for (int r = 0; r < R; ++r) {
                const T *qr = q + (int64_t)(elite[r] - t0) * st.q_t;
                float qv[kPer];
#pragma unroll
                for (int e = 0; e < kPer; ++e) qv[e] = ldf(qr + lane * kPer + e);
                float m = -INFINITY, z = 0.f;
                const int Rr = dm.causal_text ? r + 1 : R;  // keys this row sees: the list is in position order
                if (R <= 8) {
                    float a[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        a[j] = 0.f;
                        if (j < Rr) {
                            const T *kj = k + (int64_t)elite[j] * st.kv_t;
#pragma unroll
                            for (int e = 0; e < kPer; ++e) a[j] = fmaf(qv[e], ldf(kj + lane * kPer + e), a[j]);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (j < Rr) {
                            a[j] = wave_sum(a[j]);
                            m = fmaxf(m, a[j]);
                        }
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (j < Rr) z += expf((a[j] - m) * scale);
                } else {
                    for (int j = 0; j < Rr; ++j) {
                        const T *kj = k + (int64_t)elite[j] * st.kv_t;
                        float a = 0.f;
#pragma unroll
                        for (int e = 0; e < kPer; ++e) a = fmaf(qv[e], ldf(kj + lane * kPer + e), a);
                        m = fmaxf(m, wave_sum(a));
                    }
                    for (int j = 0; j < Rr; ++j) {
                        const T *kj = k + (int64_t)elite[j] * st.kv_t;
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
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------
// Visual observation window (the "visual window" of the ablation table, Tab.5): every token of the span
// is a row of every query head and no text key takes part, so the row lists are written out
// directly and the elite-text columns are empty (maximum -inf, sum 0).  One workgroup per
// (layer, sequence, query head).
__global__ __launch_bounds__(64) void window_rows_kernel(Dims dm, DevTables t, int l0, SeqArgs seqs) {
    const int h = blockIdx.x, b = blockIdx.y, li = blockIdx.z;
    const air_seq sq = seqs.s[b];
    if (li == 0 && h == 0 && threadIdx.x == 0) t.seq_tab[b] = sq;
    const int64_t hrow = ((int64_t)(l0 + li) * dm.B + b) * dm.Hq + h;
    const int W = dm.max_window;
    for (int j = threadIdx.x; j < sq.win_len; j += 64) {
        t.elite_idx[hrow * W + j] = sq.win_start + j;
        t.row_mtext[hrow * W + j] = -INFINITY;
        t.row_ztext[hrow * W + j] = 0.f;
    }
    if (threadIdx.x == 0) t.elite_cnt[hrow] = sq.win_len;
}

hipError_t launch_window_rows(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, const SeqArgs &seqs) {
    hipLaunchKernelGGL(window_rows_kernel, dim3(dm.Hq, dm.B, nl), dim3(64), 0, s, dm, t, l0, seqs);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Eq.6-7 over the visual keys.  One workgroup per (256-key chunk, unit); a unit is one
// (layer, sequence, KV head).  Thread i keeps key i of the chunk in registers and scores it
// against the elite rows of the G query heads of the group, kRowBlock rows at a time.
// PASS 1 writes per-row (max, sum-exp) of the chunk; PASS 2 accumulates Eq.8.
// With a visual window a row at visual index p sees the keys i <= p only; a chunk that lies wholly
// behind a row leaves (max -inf, sum 0) for it.
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
    const int qbase = dm.vis_window ? sq.win_start : sq.vis_start + sq.vis_len;  // token of row 0 of the query tensor
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
    __shared__ int s_lim[kRowBlock];  // last visual index a row sees
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
                s_q[rr][c] = ldf(qh + (int64_t)(tok - qbase) * st.q_t + c);
            }
            if (tid < nb) s_lim[tid] = dm.vis_window ? t.elite_idx[hrow * W + r0 + tid] - sq.vis_start : 0x7fffffff;
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
            bool ok[kRowBlock];
#pragma unroll
            for (int rr = 0; rr < kRowBlock; ++rr) ok[rr] = valid && rr < nb && i <= s_lim[rr];
            if (PASS == 1) {
#pragma unroll
                for (int rr = 0; rr < kRowBlock; ++rr) {
                    float m = wave_max(ok[rr] ? s[rr] : -INFINITY);
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
                    float e = ok[rr] ? expf(s[rr] - mrow[rr]) : 0.f;
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
                    if (ok[rr]) imp = fmaf(s_w[rr], expf(s[rr] - s_M[rr]), imp);
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
            const double sigma = sqrt(s2 / (double)(n - 1));
            // zero spread (Eq.10 undefined; taken as 0): a standard deviation at most 1e-6 of the mean
            if (sigma > 1e-6 * fabs(mu))
                sk = (double)n / (((double)n - 1.0) * ((double)n - 2.0)) * (s3 / (sigma * sigma * sigma));
        }
        t.unit_st[unit] = s_t;
        t.unit_sk[unit] = sk;
    }
}

// ---------------------------------------------------------------------------------------
template <typename T, int D>
static hipError_t elite_launch(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl,
                               const LaunchLayers &ll, const air_strides &st, const SeqArgs &seqs, double alpha) {
    const size_t per_head = (size_t)dm.max_window * (sizeof(double) + sizeof(int));
    int gb = (int)(49152 / per_head);  // heads whose logits share the LDS
    gb = gb < 1 ? 1 : (gb > dm.G ? dm.G : gb);
    hipLaunchKernelGGL((elite_kernel<T, D>), dim3(dm.Hkv, dm.B, nl), dim3(256), gb * per_head, s, dm, t, l0, ll, st, seqs,
                       alpha, gb);
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
