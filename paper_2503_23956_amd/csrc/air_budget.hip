// air_budget: Eq.11 and the cache-layout tables that follow from the budgets.
//
// One workgroup per sequence; thread 0 runs the allocation serially in fp64 (L is at most a
// few hundred).  This file is compiled with floating-point contraction off so that every
// operation rounds once, in the order written: layer shares by left-to-right sums,
// proportional allocation clamped to [min_keep, N_v] by repeatedly pinning the side with
// the larger total violation, floor + largest remainder (ties to the lower layer).
#include "air_device.h"
#include "air_internal.h"

namespace air {

__global__ __launch_bounds__(64) void budget_kernel(Dims dm, DevTables t, double retention, int mode, int min_keep,
                                                    int skip_allocation) {
    if (threadIdx.x != 0) return;
    const int b = blockIdx.x;
    const int L = dm.L;
    const air_seq sq = t.seq_tab[b];
    const int n_vis = sq.vis_len;
    __shared__ double w[AIR_MAX_LAYERS], x[AIR_MAX_LAYERS], frac[AIR_MAX_LAYERS];
    __shared__ int kk[AIR_MAX_LAYERS];
    __shared__ unsigned char is_free[AIR_MAX_LAYERS];

    double *s_t = t.s_t + (int64_t)b * L;
    double *s_k = t.s_k + (int64_t)b * L;
    int32_t *budgets = t.budgets + (int64_t)b * L;

    if (!skip_allocation) {
        // per-layer strength / skewness: mean over the KV heads, left to right
        for (int l = 0; l < L; ++l) {
            double a = 0.0, c = 0.0;
            for (int h = 0; h < dm.Hkv; ++h) {
                const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + h;
                a += t.unit_st[unit];
                c += t.unit_sk[unit];
            }
            s_t[l] = a / (double)dm.Hkv;
            s_k[l] = c / (double)dm.Hkv;
        }
        double sum_t = 0.0, sum_k = 0.0;
        for (int l = 0; l < L; ++l) {
            sum_t += s_t[l];
            sum_k += fmax(s_k[l], 0.0);
        }
        for (int l = 0; l < L; ++l) {
            const double a = sum_t > 0.0 ? s_t[l] / sum_t : 1.0 / (double)L;
            const double c = sum_k > 0.0 ? fmax(s_k[l], 0.0) / sum_k : 1.0 / (double)L;
            double wl;
            if (mode == AIR_BUDGET_UNIFORM) wl = 1.0 / (double)L;
            else if (mode == AIR_BUDGET_STRENGTH) wl = a;
            else if (mode == AIR_BUDGET_SKEW) wl = c;
            else wl = 0.5 * (a + c);
            w[l] = wl;
        }
        const int lo_i = min(min_keep, n_vis);
        const double lo = (double)lo_i, hi = (double)n_vis;
        long long k_tot = (long long)floor(retention * (double)n_vis * (double)L + 0.5);
        const long long k_lo = (long long)L * lo_i, k_hi = (long long)L * n_vis;
        k_tot = k_tot < k_lo ? k_lo : (k_tot > k_hi ? k_hi : k_tot);

        for (int l = 0; l < L; ++l) {
            x[l] = 0.0;
            is_free[l] = 1;
        }
        double k_free = (double)k_tot;
        for (int it = 0; it < L + 1; ++it) {
            double w_free = 0.0;
            int n_free = 0;
            for (int l = 0; l < L; ++l)
                if (is_free[l]) {
                    w_free += w[l];
                    ++n_free;
                }
            if (n_free == 0) break;
            double over = 0.0, under = 0.0;
            for (int l = 0; l < L; ++l)
                if (is_free[l]) {
                    x[l] = w_free > 0.0 ? (w[l] / w_free) * k_free : k_free / (double)n_free;
                    if (x[l] > hi) over += x[l] - hi;
                    else if (x[l] < lo) under += lo - x[l];
                }
            if (over == 0.0 && under == 0.0) break;
            const bool pin_hi = over >= under;
            for (int l = 0; l < L; ++l)
                if (is_free[l]) {
                    if (pin_hi && x[l] > hi) {
                        x[l] = hi;
                        is_free[l] = 0;
                        k_free -= hi;
                    } else if (!pin_hi && x[l] < lo) {
                        x[l] = lo;
                        is_free[l] = 0;
                        k_free -= lo;
                    }
                }
        }
        long long tot = 0;
        for (int l = 0; l < L; ++l) {
            int fl = (int)floor(x[l]);
            fl = max(lo_i, min(fl, n_vis));
            kk[l] = fl;
            frac[l] = x[l] - (double)fl;
            tot += fl;
        }
        long long left = k_tot - tot;
        while (left > 0) {
            int best = -1;
            for (int l = 0; l < L; ++l)
                if (kk[l] < n_vis && (best < 0 || frac[l] > frac[best])) best = l;
            if (best < 0) break;
            kk[best] += 1;
            frac[best] = -1.0;
            --left;
        }
        for (int l = 0; l < L; ++l) budgets[l] = kk[l];
    }

    // cache layout: each layer's region holds system + kept + text rows and room for the
    // decode appends, and starts on a multiple of kCacheRowAlign rows
    const int nonvis = sq.seq_len - sq.vis_len;
    int off = 0;
    for (int l = 0; l < L; ++l) {
        const int len = nonvis + budgets[l];
        t.base_len[(int64_t)b * L + l] = len;
        t.layer_off[(int64_t)b * L + l] = off;
        const int cap = len + dm.max_steps;
        off += (cap + kCacheRowAlign - 1) / kCacheRowAlign * kCacheRowAlign;
    }
}

hipError_t launch_budget(hipStream_t s, const Dims &dm, const DevTables &t, double retention, int mode,
                         int min_keep, int skip_allocation) {
    hipLaunchKernelGGL(budget_kernel, dim3(dm.B), dim3(64), 0, s, dm, t, retention, mode, min_keep, skip_allocation);
    return hipGetLastError();
}

}  // namespace air
