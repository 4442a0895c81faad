// air_budget: Eq.9-11 across layers and the cache-layout tables that follow from the budgets.  One workgroup per
// sequence; the arithmetic is in air_budget_dev.h (this file is compiled with floating-point contraction off as well).
#include "air_budget_dev.h"

namespace air {

constexpr int kBT = 256;  // threads; also the largest layer count (AIR_MAX_LAYERS)

// ONE_WAVE (up to 64 layers, the usual depth): after the statistics are staged the first wave does the rest alone.
template <bool ONE_WAVE>
__global__ __launch_bounds__(kBT) void budget_kernel(Dims dm, DevTables t, double retention, int mode, int min_keep,
                                                     int skip_allocation, SeqArgs seqs) {
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int L = dm.L;
    const air_seq sq = seqs.s[b];  // from the kernel arguments: no table read in front of the statistics
    __shared__ double a0[kBT], a1[kBT];  // addends of the ordered sums (one per layer)
    __shared__ double frac[kBT];
    __shared__ int i0[kBT], i1[kBT];
    __shared__ double u_st[AIR_MAX_LAYERS * 16], u_sk[AIR_MAX_LAYERS * 16];  // per (layer, KV head), H_kv <= 16 staged
    // Eq.9-10 of every (layer, KV head) are there (air_score's last kernel leaves them per unit): staged through LDS
    // in one round of loads where they fit
    const int n_units = L * dm.Hkv;
    const bool stage = !skip_allocation && n_units <= AIR_MAX_LAYERS * 16;
    if (stage) {
        for (int p = tid; p < n_units; p += kBT) {
            const int l = p / dm.Hkv, h = p % dm.Hkv;
            const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + h;
            u_st[p] = t.unit_st[unit];
            u_sk[p] = t.unit_sk[unit];
        }
        __syncthreads();
    }
    if (ONE_WAVE && tid >= 64) return;  // one wave takes it from here
    allocate_and_lay_out<ONE_WAVE>(dm, t, b, sq, retention, mode, min_keep, skip_allocation != 0, tid, a0, a1, frac, i0, i1,
                                   [&](int l, double &a, double &c) __attribute__((always_inline)) {
                                       for (int h = 0; h < dm.Hkv; ++h) {
                                           const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + h;
                                           a += stage ? u_st[l * dm.Hkv + h] : t.unit_st[unit];
                                           c += stage ? u_sk[l * dm.Hkv + h] : t.unit_sk[unit];
                                       }
                                   });
}

hipError_t launch_budget(hipStream_t s, const Dims &dm, const DevTables &t, double retention, int mode,
                         int min_keep, int skip_allocation, const SeqArgs &seqs) {
    if (dm.L <= 64)
        hipLaunchKernelGGL(budget_kernel<true>, dim3(dm.B), dim3(kBT), 0, s, dm, t, retention, mode, min_keep,
                           skip_allocation, seqs);
    else
        hipLaunchKernelGGL(budget_kernel<false>, dim3(dm.B), dim3(kBT), 0, s, dm, t, retention, mode, min_keep,
                           skip_allocation, seqs);
    return hipGetLastError();
}

}  // namespace air
