// Eq.11 across the layers of one sequence and the cache-layout tables that follow from the budgets: device code shared
// by the budget kernel and by the tail of air_score's last kernel (whose last workgroup of a sequence does the
// allocation itself when the layers fit one wave).
//
// Everything that decides an integer runs in fp64 with every operation rounded once, in a fixed order (contraction is
// switched off inside these functions): per-layer strength / skewness as the left-to-right mean over KV heads, layer
// shares by left-to-right sums, proportional allocation clamped to [min_keep, N_v] by repeatedly pinning the side with
// the larger total violation, floor + largest remainder (ties to the lower layer).  Thread l owns layer l.  The
// order-dependent sums over the layers are formed by EVERY thread for itself, left to right, from a copy of the addends
// in LDS: all lanes read the same address (a broadcast), the reads of several addends are in flight together, and no
// thread waits for another one's serial loop (a wave that handed values from lane to lane through scalar registers
// spent 35-40 ns per addend; here an addend costs one dependent fp64 add).  The threads exchange data through LDS
// only, so the barriers order LDS traffic and do not wait for the global stores of the statistics and budgets.
#pragma once

#include "air_device.h"
#include "air_internal.h"

namespace air {

// left-to-right sum of a[0 .. n), the same in every thread that calls it.  The entries from n up to the next
// multiple of 8 hold exact zeros (every thread writes its slot, threads past the last layer write zero), so the
// sum runs over whole groups of 8 whose reads are in flight together: adding +0.0 changes nothing.
__device__ __forceinline__ double ordered_sum(const double *a, int n) {
    double sum = 0.0;
    for (int l = 0; l < n; l += 8) {
        double v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = a[l + j];
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += v[j];
    }
    return sum;
}
__device__ __forceinline__ int int_sum(const int *a, int n) {  // n a multiple of 8, zeros past the last layer
    int sum = 0;
    for (int l = 0; l < n; l += 8) {
        int v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = a[l + j];
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += v[j];
    }
    return sum;
}

// Called by the threads 0 .. max(64, L rounded up) of a workgroup (ONE_WAVE: by one wave, for up to 64 layers; the
// exchanges through LDS then need no workgroup barrier, a wave's LDS accesses complete in program order, only the
// compiler is kept from moving them).  a0, a1, frac, i0, i1: LDS arrays of one slot per calling thread.
// head_sums(l, a, c): the left-to-right sums over the KV heads of layer l's unit strengths and skewnesses.
template <bool ONE_WAVE, class HeadSums>
__device__ __forceinline__ void allocate_and_lay_out(const Dims &dm, const DevTables &t, int b, const air_seq &sq,
                                                     double retention, int mode, int min_keep, bool skip_allocation,
                                                     int tid, double *a0, double *a1, double *frac, int *i0, int *i1,
                                                     HeadSums head_sums) {
#pragma clang fp contract(off)
    const int L = dm.L;
    const int n_vis = sq.vis_len;
    const bool mine = tid < L;
    const int L8 = (L + 7) & ~7;  // the sums over the layers run over whole groups of 8 (zeros past the last layer)
    auto sync = [&]() __attribute__((always_inline)) {
        if (ONE_WAVE) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            lds_barrier();
        }
    };
    int32_t *budgets = t.budgets + (int64_t)b * L;
    int kk = 0;
    if (skip_allocation) {
        if (mine) kk = budgets[tid];  // the budgets were set by the caller: only the layout is left
    } else {
        double st = 0.0, sk = 0.0;
        if (mine) {  // mean over the KV heads, left to right
            double a = 0.0, c = 0.0;
            head_sums(tid, a, c);
            st = a / (double)dm.Hkv;
            sk = c / (double)dm.Hkv;
            t.s_t[(int64_t)b * L + tid] = st;
            t.s_k[(int64_t)b * L + tid] = sk;
        }
        const int lo_i = min(min_keep, n_vis);
        const double lo = (double)lo_i, hi = (double)n_vis;
        const double skp = fmax(sk, 0.0);
        a0[tid] = st;   // threads past the last layer hold exact zeros
        a1[tid] = skp;
        sync();
        const double sum_t = ordered_sum(a0, L8), sum_k = ordered_sum(a1, L8);
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
        // proportional allocation with clamping: pin the side with the larger total violation, repeat.  Every
        // thread carries the same k_free, n_free and pin decision, formed from the same LDS copies.
        bool is_free = mine;
        double x = 0.0, k_free = (double)k_tot;
        for (int it = 0; it < L + 1; ++it) {
            sync();  // the sums of the round before (or of the shares) have been read
            a0[tid] = is_free ? wl : 0.0;  // a pinned layer adds an exact zero
            i0[tid] = is_free ? 1 : 0;
            sync();
            const int n_free = int_sum(i0, L8);
            if (n_free == 0) break;
            const double w_free = ordered_sum(a0, L8);
            double vo = 0.0, vu = 0.0;
            if (is_free) {
                x = w_free > 0.0 ? (wl / w_free) * k_free : k_free / (double)n_free;
                if (x > hi) vo = x - hi;
                else if (x < lo) vu = lo - x;
            }
            sync();
            a0[tid] = vo;
            a1[tid] = vu;
            sync();
            const double over = ordered_sum(a0, L8), under = ordered_sum(a1, L8);
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
            i1[tid] = pinned ? 1 : 0;
            sync();
            // k_free stays an integer-valued double: the bound is subtracted once per pinned layer
            const int n_pin = int_sum(i1, L8);
            const double bound = pin == 1 ? hi : lo;
            for (int q = 0; q < n_pin; ++q) k_free -= bound;
        }
        sync();
        double fr = -1.0;
        if (mine) {
            kk = max(lo_i, min((int)floor(x), n_vis));
            fr = x - (double)kk;
        }
        frac[tid] = fr;
        i0[tid] = mine ? kk : 0;
        i1[tid] = (mine && kk < n_vis) ? 1 : 0;  // eligible for a leftover token
        sync();
        const long long left = k_tot - (long long)int_sum(i0, L8);
        const int n_elig = int_sum(i1, L8);
        if (left > 0 && left <= (long long)n_elig) {
            // largest remainder: the `left` eligible layers that come first by (fraction descending, layer ascending)
            if (mine && kk < n_vis) {
                int rank = 0;
                for (int j0 = 0; j0 < L8; j0 += 8) {  // branch-free groups of 8: their LDS reads are in flight together
#pragma unroll
                    for (int j = j0; j < j0 + 8; ++j) {
                        const double fj = frac[j];
                        rank += i1[j] & ((int)(fj > fr) | ((int)(fj == fr) & (int)(j < tid)));
                    }
                }
                if (rank < (int)left) kk += 1;
            }
        } else if (left > 0) {
            // more leftovers than eligible layers: hand them out one by one, each to the eligible layer with the
            // largest fraction (the lowest such layer), which then counts as served
            sync();
            if (tid == 0) {
                for (long long rem = left; rem > 0; --rem) {
                    int best = -1;
                    for (int l = 0; l < L; ++l)
                        if (i0[l] < n_vis && (best < 0 || frac[l] > frac[best])) best = l;
                    if (best < 0) break;
                    i0[best] += 1;
                    frac[best] = -1.0;
                }
            }
            sync();
            if (mine) kk = i0[tid];
        }
        if (mine) budgets[tid] = kk;
        sync();  // i0 is reused below
    }
    // cache layout: each layer's region holds system + kept + text rows and room for the decode
    // appends, and starts on a multiple of kCacheRowAlign rows
    const int nonvis = sq.seq_len - sq.vis_len;
    i0[tid] = mine ? (nonvis + kk + dm.max_steps + kCacheRowAlign - 1) / kCacheRowAlign * kCacheRowAlign : 0;
    i1[tid] = mine ? kk : -1;
    sync();
    if (mine) {
        // one pass over the layers gives the layer's row offset and its rank by falling cache length (ties: the
        // lower layer first); the table by rank serves decode launches that take their longest units first
        int off = 0, rank = 0;
        for (int l0 = 0; l0 < L8; l0 += 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                off += l0 + j < tid ? i0[l0 + j] : 0;
                rank += (int)(i1[l0 + j] > kk) | ((int)(i1[l0 + j] == kk) & (int)(l0 + j < tid));
            }
        }
        t.base_len[(int64_t)b * L + tid] = nonvis + kk;
        t.layer_off[(int64_t)b * L + tid] = off;
        t.len_off[(int64_t)b * L + tid] = make_int2(nonvis + kk, off);
        t.by_length[(int64_t)b * L + rank] = make_int4(nonvis + kk, off, tid, 0);
    }
}


}  // namespace air
