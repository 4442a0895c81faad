// air_budget: Eq.9-11 across layers and the cache-layout tables that follow from the budgets.
//
// One workgroup per sequence.  Everything that decides an integer runs in fp64 with every
// operation rounded once, in a fixed order (this file is compiled with floating-point
// contraction off): per-layer strength / skewness as the left-to-right mean over KV heads,
// layer shares by left-to-right sums, proportional allocation clamped to [min_keep, N_v] by
// repeatedly pinning the side with the larger total violation, floor + largest remainder
// (ties to the lower layer).  Up to 64 layers are done by one wave, a layer per lane, whose lanes
// read each other's registers: no LDS, no barriers.  Beyond that the per-layer work is spread over
// the threads of the workgroup and the order-dependent sums stay serial in thread 0; the threads
// exchange data through LDS only, so the barriers order LDS traffic and do not wait for the
// global stores of the statistics and budgets.
#include "air_device.h"
#include "air_internal.h"

namespace air {

constexpr int kBT = 256;  // threads; also the largest layer count (AIR_MAX_LAYERS)

// Value that lane `l` (the same for every lane of the wave) holds, handed to all lanes through a scalar register.
__device__ __forceinline__ double lane_value(double v, int l) {
    const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)u, l);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u >> 32), l);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// Eq.11 and the cache layout for up to 64 layers by ONE wave, a layer per lane.  The order-dependent
// sums run left to right over the lanes (every lane forms the same sum from scalar reads of the other
// lanes' registers), so the wave needs neither LDS nor barriers; the arithmetic and its order are
// those of the many-layer path below.
__device__ __forceinline__ void allocate_one_wave(const Dims &dm, const DevTables &t, double retention, int mode, int min_keep,
                                                  int skip_allocation, bool stats_in_lds, const air_seq &sq, int b,
                                                  const double *u_st, const double *u_sk) {
    const int lane = threadIdx.x, L = dm.L, n_vis = sq.vis_len;
    const bool mine = lane < L;
    int32_t *budgets = t.budgets + (int64_t)b * L;
    int kk = 0;
    if (skip_allocation) {
        if (mine) kk = budgets[lane];
    } else {
        double st = 0.0, sk = 0.0;
        if (mine) {  // mean over the KV heads, left to right
            double a = 0.0, c = 0.0;
            for (int h = 0; h < dm.Hkv; ++h) {
                const int64_t unit = ((int64_t)lane * dm.B + b) * dm.Hkv + h;
                a += stats_in_lds ? u_st[lane * dm.Hkv + h] : t.unit_st[unit];
                c += stats_in_lds ? u_sk[lane * dm.Hkv + h] : t.unit_sk[unit];
            }
            st = a / (double)dm.Hkv;
            sk = c / (double)dm.Hkv;
            t.s_t[(int64_t)b * L + lane] = st;
            t.s_k[(int64_t)b * L + lane] = sk;
        }
        const int lo_i = min(min_keep, n_vis);
        const double lo = (double)lo_i, hi = (double)n_vis;
        const double skp = fmax(sk, 0.0);
        double sum_t = 0.0, sum_k = 0.0;
        for (int l = 0; l < L; ++l) {
            sum_t += lane_value(st, l);
            sum_k += lane_value(skp, l);
        }
        long long k_tot = (long long)floor(retention * (double)n_vis * (double)L + 0.5);
        const long long k_lo = (long long)L * lo_i, k_hi = (long long)L * n_vis;
        k_tot = k_tot < k_lo ? k_lo : (k_tot > k_hi ? k_hi : k_tot);
        const double a = sum_t > 0.0 ? st / sum_t : 1.0 / (double)L;
        const double c = sum_k > 0.0 ? skp / sum_k : 1.0 / (double)L;
        double wl;
        if (mode == AIR_BUDGET_UNIFORM) wl = 1.0 / (double)L;
        else if (mode == AIR_BUDGET_STRENGTH) wl = a;
        else if (mode == AIR_BUDGET_SKEW) wl = c;
        else wl = 0.5 * (a + c);
        // proportional allocation with clamping: pin the side with the larger total violation, repeat
        bool is_free = mine;
        double x = 0.0, k_free = (double)k_tot;
        for (int it = 0; it < L + 1; ++it) {
            const int n_free = __popcll(__ballot(is_free));
            if (n_free == 0) break;
            const double w_mine = is_free ? wl : 0.0;  // a pinned layer adds an exact zero
            double w_free = 0.0;
            for (int l = 0; l < L; ++l) w_free += lane_value(w_mine, l);
            double vo = 0.0, vu = 0.0;
            if (is_free) {
                x = w_free > 0.0 ? (wl / w_free) * k_free : k_free / (double)n_free;
                if (x > hi) vo = x - hi;
                else if (x < lo) vu = lo - x;
            }
            double over = 0.0, under = 0.0;
            for (int l = 0; l < L; ++l) {
                over += lane_value(vo, l);
                under += lane_value(vu, l);
            }
            const int pin = (over == 0.0 && under == 0.0) ? 0 : (over >= under ? 1 : 2);
            if (pin == 0) break;
            bool pinned = false;
            if (is_free && pin == 1 && x > hi) {
                x = hi;
                pinned = true;
            } else if (is_free && pin == 2 && x < lo) {
                x = lo;
                pinned = true;
            }
            is_free = is_free && !pinned;
            // k_free stays an integer-valued double: the bound is subtracted once per pinned layer
            const int n_pin = __popcll(__ballot(pinned));
            const double bound = pin == 1 ? hi : lo;
            for (int q = 0; q < n_pin; ++q) k_free -= bound;
        }
        double frac = -1.0;
        if (mine) {
            kk = max(lo_i, min((int)floor(x), n_vis));
            frac = x - (double)kk;
        }
        int tot = 0;
        for (int l = 0; l < L; ++l) tot += __builtin_amdgcn_readlane(kk, l);
        unsigned long long elig = __ballot(mine && kk < n_vis);
        const long long left = k_tot - (long long)tot;
        if (left > 0 && left <= (long long)__popcll(elig)) {
            // largest remainder: the `left` eligible layers that come first by (fraction descending, layer ascending)
            int rank = 0;
            for (int j = 0; j < L; ++j) {
                const double fj = lane_value(frac, j);
                rank += (int)((elig >> j) & 1ull) & ((int)(fj > frac) | ((int)(fj == frac) & (int)(j < lane)));
            }
            if (((elig >> lane) & 1ull) && rank < (int)left) kk += 1;
        } else if (left > 0) {
            // more leftovers than eligible layers: hand them out one by one, each to the eligible layer
            // with the largest fraction (the lowest such layer), which then counts as served
            for (long long rem = left; rem > 0 && elig != 0ull; --rem) {
                int best = -1;
                double fbest = 0.0;
                for (int l = 0; l < L; ++l) {
                    const double fl = lane_value(frac, l);
                    if (((elig >> l) & 1ull) && (best < 0 || fl > fbest)) {
                        best = l;
                        fbest = fl;
                    }
                }
                if (lane == best) {
                    kk += 1;
                    frac = -1.0;
                }
                elig = __ballot(mine && kk < n_vis);
            }
        }
        if (mine) budgets[lane] = kk;
    }
    // cache layout: each layer's region holds system + kept + text rows and room for the decode
    // appends, and starts on a multiple of kCacheRowAlign rows
    const int nonvis = sq.seq_len - sq.vis_len;
    const int cap = (nonvis + kk + dm.max_steps + kCacheRowAlign - 1) / kCacheRowAlign * kCacheRowAlign;
    int off = 0;
    for (int l = 0; l < L; ++l) {
        const int cl = __builtin_amdgcn_readlane(cap, l);
        off += l < lane ? cl : 0;
    }
    if (mine) {
        t.base_len[(int64_t)b * L + lane] = nonvis + kk;
        t.layer_off[(int64_t)b * L + lane] = off;
        t.len_off[(int64_t)b * L + lane] = make_int2(nonvis + kk, off);
    }
}

__global__ __launch_bounds__(kBT) void budget_kernel(Dims dm, DevTables t, double retention, int mode, int min_keep,
                                                     int skip_allocation, int use_moments, SeqArgs seqs) {
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int L = dm.L;
    const air_seq sq = seqs.s[b];  // from the kernel arguments: no table read in front of the moment entries
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
            // Eq.9-10 of every (layer, KV head) from the moment entries of its importance row: entry c holds
            // the sum S1_c, the mean m_c and the moments M2_c, M3_c about m_c of the n_c scores of kFinishChunks
            // chunks.  With d_c = m_c - mu the central moments of the row are
            //   sum (x - mu)^2 = sum_c M2_c + n_c d_c^2,   sum (x - mu)^3 = sum_c M3_c + 3 d_c M2_c + n_c d_c^3,
            // sums of terms no larger than their result (raw power sums would cancel on rows of little spread).
            constexpr int kEntryKeys = kFinishChunks * kChunkKeys;
            const int nch = (n_vis + kEntryKeys - 1) / kEntryKeys;  // entries per unit
            for (int p = tid; p < L * dm.Hkv; p += kBT) {
                const int l = p / dm.Hkv, h = p % dm.Hkv;
                const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + h;
                const double *mo = t.moments + unit * dm.n_entries * 4;
                double S1 = 0.0;
#pragma unroll 4
                for (int c = 0; c < nch; ++c) S1 += mo[4 * c];  // ordered sum; unrolled so that the loads of 4 entries are in flight together
                double sk = 0.0;
                if (n_vis >= 3) {
                    const double n = (double)n_vis;
                    const double mu = S1 / n;
                    double c2 = 0.0, c3 = 0.0;
#pragma unroll 4
                    for (int c = 0; c < nch; ++c) {
                        const double nc = (double)min(kEntryKeys, n_vis - c * kEntryKeys);
                        const double dl = mo[4 * c + 1] - mu, M2 = mo[4 * c + 2], M3 = mo[4 * c + 3];
                        c2 += M2 + nc * (dl * dl);
                        c3 += (M3 + 3.0 * dl * M2) + nc * (dl * dl * dl);
                    }
                    const double sigma = sqrt(c2 / (n - 1.0));
                    // zero spread (Eq.10 undefined; taken as 0): a standard deviation at most 1e-6 of the mean
                    if (sigma > 1e-6 * fabs(mu)) sk = n / ((n - 1.0) * (n - 2.0)) * (c3 / (sigma * sigma * sigma));
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
        if (L <= 64) {  // the usual depth: one wave takes it from here
            if (tid < 64) allocate_one_wave(dm, t, retention, mode, min_keep, 0, use_moments && stage, sq, b, u_st, u_sk);
            return;
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

    if (L <= 64) {  // only the layout is left (the budgets were set by the caller)
        if (tid < 64) allocate_one_wave(dm, t, retention, mode, min_keep, 1, false, sq, b, u_st, u_sk);
        return;
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
