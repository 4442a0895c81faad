// air_budget: Eq.9-11 across layers and the cache-layout tables that follow from the budgets.
//
// One workgroup per sequence.  Everything that decides an integer runs in fp64 with every
// operation rounded once, in a fixed order (this file is compiled with floating-point
// contraction off): per-layer strength / skewness as the left-to-right mean over KV heads,
// layer shares by left-to-right sums, proportional allocation clamped to [min_keep, N_v] by
// repeatedly pinning the side with the larger total violation, floor + largest remainder
// (ties to the lower layer).  Independent per-layer work is spread over the threads; the
// order-dependent sums stay serial in thread 0.  Threads exchange data through LDS only, so the
// barriers order LDS traffic and do not wait for the global stores of the statistics and budgets.
#include "air_device.h"
#include "air_internal.h"

namespace air {

constexpr int kBT = 256;  // threads; also the largest layer count (AIR_MAX_LAYERS)

__global__ __launch_bounds__(kBT) void budget_kernel(Dims dm, DevTables t, double retention, int mode, int min_keep,
                                                     int skip_allocation, int use_moments, SeqArgs seqs) {
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int L = dm.L;
    const air_seq sq = seqs.s[b];  // from the kernel arguments: no table read in front of the power sums
    const int n_vis = sq.vis_len;
    __shared__ double w[kBT], x[kBT], frac[kBT], sh_t[kBT], sh_k[kBT];
    __shared__ int kk[kBT];
    __shared__ unsigned char is_free[kBT];
    __shared__ double s_sum_t, s_sum_k;
    __shared__ long long s_ktot;
    __shared__ int s_tot, s_elig, s_nfree, s_pin, s_npin;
    __shared__ double s_wfree, s_kfree, v_over[kBT], v_under[kBT];
    __shared__ double u_st[AIR_MAX_LAYERS * 16], u_sk[AIR_MAX_LAYERS * 16];  // per (layer, KV head), H_kv <= 16 staged

    double *s_t = t.s_t + (int64_t)b * L;
    double *s_k = t.s_k + (int64_t)b * L;
    int32_t *budgets = t.budgets + (int64_t)b * L;

    const bool stage = L * dm.Hkv <= AIR_MAX_LAYERS * 16;  // unit statistics fit the LDS staging arrays
    if (!skip_allocation) {
        if (use_moments) {
            // Eq.9-10 of every (layer, KV head) from the power sums of the importance row (one entry per
            // kFinishChunks chunks)
            const int nch = ((n_vis + kChunkKeys - 1) / kChunkKeys + kFinishChunks - 1) / kFinishChunks;  // entries per unit
            for (int p = tid; p < L * dm.Hkv; p += kBT) {
                const int l = p / dm.Hkv, h = p % dm.Hkv;
                const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + h;
                const double *mo = t.moments + unit * dm.n_chunks * 3;
                double S1 = 0.0, S2 = 0.0, S3 = 0.0;
#pragma unroll 8
                for (int c = 0; c < nch; ++c) {  // ordered sums; unrolled so that the loads of 8 chunks are in flight together
                    S1 += mo[3 * c + 0];
                    S2 += mo[3 * c + 1];
                    S3 += mo[3 * c + 2];
                }
                double sk = 0.0;
                if (n_vis >= 3) {
                    const double n = (double)n_vis;
                    const double mu = S1 / n;
                    const double c2 = S2 - S1 * mu;                           // sum (x - mu)^2
                    const double c3 = S3 - 3.0 * mu * S2 + 2.0 * mu * mu * S1;  // sum (x - mu)^3
                    const double var = c2 / (n - 1.0);
                    if (var > 0.0) {
                        const double sigma = sqrt(var);
                        sk = n / ((n - 1.0) * (n - 2.0)) * (c3 / (sigma * sigma * sigma));
                    }
                }
                t.unit_st[unit] = S1;
                t.unit_sk[unit] = sk;
                if (stage) {
                    u_st[p] = S1;
                    u_sk[p] = sk;
                }
            }
            if (stage) lds_barrier();  // the statistics cross in LDS: no wait for the global stores above
            else __syncthreads();
        }
        if (tid < L) {  // mean over the KV heads, left to right
            double a = 0.0, c = 0.0;
            for (int h = 0; h < dm.Hkv; ++h) {
                const int64_t unit = ((int64_t)tid * dm.B + b) * dm.Hkv + h;
                const bool lds = use_moments && stage;
                a += lds ? u_st[tid * dm.Hkv + h] : t.unit_st[unit];
                c += lds ? u_sk[tid * dm.Hkv + h] : t.unit_sk[unit];
            }
            sh_t[tid] = a / (double)dm.Hkv;
            sh_k[tid] = c / (double)dm.Hkv;
            s_t[tid] = sh_t[tid];
            s_k[tid] = sh_k[tid];
        }
        lds_barrier();
        const int lo_i = min(min_keep, n_vis);
        const double lo = (double)lo_i, hi = (double)n_vis;
        if (tid == 0) {
            double sum_t = 0.0, sum_k = 0.0;
            for (int l = 0; l < L; ++l) {
                sum_t += sh_t[l];
                sum_k += fmax(sh_k[l], 0.0);
            }
            s_sum_t = sum_t;
            s_sum_k = sum_k;
            long long k_tot = (long long)floor(retention * (double)n_vis * (double)L + 0.5);
            const long long k_lo = (long long)L * lo_i, k_hi = (long long)L * n_vis;
            s_ktot = k_tot < k_lo ? k_lo : (k_tot > k_hi ? k_hi : k_tot);
            s_tot = 0;
            s_elig = 0;
            s_npin = 0;
        }
        lds_barrier();
        if (tid < L) {
            const double a = s_sum_t > 0.0 ? sh_t[tid] / s_sum_t : 1.0 / (double)L;
            const double c = s_sum_k > 0.0 ? fmax(sh_k[tid], 0.0) / s_sum_k : 1.0 / (double)L;
            double wl;
            if (mode == AIR_BUDGET_UNIFORM) wl = 1.0 / (double)L;
            else if (mode == AIR_BUDGET_STRENGTH) wl = a;
            else if (mode == AIR_BUDGET_SKEW) wl = c;
            else wl = 0.5 * (a + c);
            w[tid] = wl;
            x[tid] = 0.0;
            is_free[tid] = 1;
        }
        lds_barrier();
        // proportional allocation with clamping.  Per round: thread 0 sums the free weights in layer
        // order, every layer forms its own x_l (the divisions run in parallel), thread 0 sums the
        // violations in layer order and picks the side to pin.
        if (tid == 0) s_kfree = (double)s_ktot;
        for (int it = 0; it < L + 1; ++it) {
            lds_barrier();
            if (tid == 0) {
                double w_free = 0.0;
                int n_free = 0;
#pragma unroll 8
                for (int l = 0; l < L; ++l) {  // branch-free: a pinned layer adds an exact zero
                    w_free += is_free[l] ? w[l] : 0.0;
                    n_free += is_free[l];
                }
                s_wfree = w_free;
                s_nfree = n_free;
            }
            lds_barrier();
            if (s_nfree == 0) break;
            if (tid < L) {
                double vo = 0.0, vu = 0.0;
                if (is_free[tid]) {
                    const double xl = s_wfree > 0.0 ? (w[tid] / s_wfree) * s_kfree : s_kfree / (double)s_nfree;
                    x[tid] = xl;
                    if (xl > hi) vo = xl - hi;
                    else if (xl < lo) vu = lo - xl;
                }
                v_over[tid] = vo;
                v_under[tid] = vu;
            }
            lds_barrier();
            if (tid == 0) {
                double over = 0.0, under = 0.0;
#pragma unroll 4
                for (int l = 0; l < L; ++l) {  // pinned layers contribute exact zeros
                    over += v_over[l];
                    under += v_under[l];
                }
                s_pin = (over == 0.0 && under == 0.0) ? 0 : (over >= under ? 1 : 2);
            }
            lds_barrier();
            const int pin = s_pin;
            if (pin == 0) break;
            int pinned = 0;
            if (tid < L && is_free[tid]) {
                if (pin == 1 && x[tid] > hi) {
                    x[tid] = hi;
                    is_free[tid] = 0;
                    pinned = 1;
                } else if (pin == 2 && x[tid] < lo) {
                    x[tid] = lo;
                    is_free[tid] = 0;
                    pinned = 1;
                }
            }
            // k_free stays an integer-valued double: subtracting the bound once per pinned layer is exact in any order
            const unsigned long long any = __ballot(pinned);
            if (any && (tid & 63) == 0) atomicAdd(&s_npin, __popcll(any));
            lds_barrier();
            if (tid == 0) {
                const double bound = pin == 1 ? hi : lo;
                for (int q = 0; q < s_npin; ++q) s_kfree -= bound;
                s_npin = 0;
            }
        }
        lds_barrier();
        if (tid < L) {
            int fl = (int)floor(x[tid]);
            fl = max(lo_i, min(fl, n_vis));
            kk[tid] = fl;
            frac[tid] = x[tid] - (double)fl;
            atomicAdd(&s_tot, fl);
            if (fl < n_vis) atomicAdd(&s_elig, 1);
        }
        lds_barrier();
        const long long left = s_ktot - (long long)s_tot;
        if (left > 0 && left <= (long long)s_elig) {
            // largest remainder: the `left` eligible layers that come first by (fraction descending, layer ascending)
            int add = 0;
            if (tid < L && kk[tid] < n_vis) {
                int rank = 0;
                const double mine = frac[tid];
#pragma unroll 8
                for (int j = 0; j < L; ++j) {  // branch-free, so that the LDS reads of several layers are in flight together
                    const double fj = frac[j];
                    rank += (int)(kk[j] < n_vis) & ((int)(fj > mine) | ((int)(fj == mine) & (int)(j < tid)));
                }
                add = rank < (int)left ? 1 : 0;
            }
            lds_barrier();
            if (tid < L) kk[tid] += add;
        } else if (left > 0) {
            if (tid == 0) {  // more leftovers than eligible layers: hand them out one by one
                long long rem = left;
                while (rem > 0) {
                    int best = -1;
                    for (int l = 0; l < L; ++l)
                        if (kk[l] < n_vis && (best < 0 || frac[l] > frac[best])) best = l;
                    if (best < 0) break;
                    kk[best] += 1;
                    frac[best] = -1.0;
                    --rem;
                }
            }
        }
        lds_barrier();
        if (tid < L) budgets[tid] = kk[tid];
        lds_barrier();
    }

    // cache layout: each layer's region holds system + kept + text rows and room for the
    // decode appends, and starts on a multiple of kCacheRowAlign rows
    if (skip_allocation && tid < L) kk[tid] = budgets[tid];  // otherwise kk still holds what was just written
    lds_barrier();
    const int nonvis = sq.seq_len - sq.vis_len;
    if (tid < L) {
        int off = 0;
#pragma unroll 8
        for (int l = 0; l < tid; ++l) {
            const int cap = nonvis + kk[l] + dm.max_steps;
            off += (cap + kCacheRowAlign - 1) / kCacheRowAlign * kCacheRowAlign;
        }
        t.base_len[(int64_t)b * L + tid] = nonvis + kk[tid];
        t.layer_off[(int64_t)b * L + tid] = off;
        t.len_off[(int64_t)b * L + tid] = make_int2(nonvis + kk[tid], off);
    }
}

hipError_t launch_budget(hipStream_t s, const Dims &dm, const DevTables &t, double retention, int mode,
                         int min_keep, int skip_allocation, int use_moments, const SeqArgs &seqs) {
    hipLaunchKernelGGL(budget_kernel, dim3(dm.B), dim3(kBT), 0, s, dm, t, retention, mode, min_keep, skip_allocation,
                       use_moments, seqs);
    return hipGetLastError();
}

}  // namespace air
