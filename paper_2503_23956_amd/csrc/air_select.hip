// air_select_compact: Alg.1 second loop.
//
//   select_kernel  top-k_l of the importance row of one (layer, sequence, KV head): radix
//                  select on the fp32 bit patterns (importance is non-negative, so unsigned
//                  integer order is value order), then an ordered compaction that keeps
//                  everything above the k-th value and the lowest-index ties at it.
//   gather_kernel  K' = [K_sys ; K_v[idx] ; K_t], V' likewise, as 16-byte vector copies.
#include "air_device.h"
#include "air_internal.h"

namespace air {

constexpr int kSelThreads = 512;                     // threads of the selection kernel for long rows (256 for rows up to 8192 scores)
constexpr int kSelRegs = 32;                         // scores per thread kept in registers, at most (compiled for 8, 16 and 32)
constexpr int kSelCand = 1024;                       // scores of the deciding 12-bit bin that are ranked directly

// leading 12 bits of a score pattern; importance is non-negative, a set sign bit (never produced) falls into the top bin
__device__ __forceinline__ uint32_t digit12(uint32_t v) { return min(v >> 20, 2047u); }

template <int NT, int REGS>
__global__ __launch_bounds__(NT) void select_kernel(Dims dm, DevTables t, int l0, int cand_cap) {
    constexpr int kSpan = NT * REGS;  // scores per sweep
    constexpr int kBinsPer = 2048 / NT;   // bins of the 12-bit histogram per thread
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.y, l = l0 + (int)blockIdx.z;  // grid (KV head, sequence, layer)
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + blockIdx.x;
    const uint32_t *key = reinterpret_cast<const uint32_t *>(t.scores + unit * dm.max_vis);
    // A sweep of up to kSpan scores stays in registers for all passes: thread t owns the `per`
    // consecutive scores from base + t * per on.  `per` follows the row capacity (a kernel argument),
    // not the sequence's own length, so that a short row's loads go out before anything has been
    // read (entries past the sequence's span exist and are never counted).  Rows longer than
    // kSpan are re-read sweep by sweep.
    // the two table entries are requested in front of the scores, so that they are not waited for behind them
    const int n = t.seq_tab[b].vis_len;
    const int k = t.budgets[(int64_t)b * dm.L + l];
    const bool cached = dm.max_vis <= kSpan;
    const int per = cached ? (dm.max_vis + NT - 1) / NT : REGS;
    uint32_t v[REGS];
    if (cached) {
#pragma unroll
        for (int j = 0; j < REGS; ++j) {
            const int i = tid * per + j;
            v[j] = (j < per && i < dm.max_vis) ? key[i] : 0u;
        }
    }
    int32_t *out = t.indices + unit * dm.max_vis;
    if (k <= 0) return;
    if (k >= n) {
        for (int i = tid; i < n; i += NT) out[i] = i;
        return;
    }

    __shared__ uint32_t hist[NT / 64][256];  // one histogram per wave: scores share leading bits, so few bins are hot
    __shared__ uint32_t s_prefix, s_kk, s_m, s_ncand, s_tau, s_ktau;
    __shared__ uint32_t h12[2048], cand[kSelCand];
    __shared__ int s_scan[NT / 64 + 1];

    auto load_sweep = [&](int base) {
#pragma unroll
        for (int j = 0; j < REGS; ++j) {
            const int i = base + tid * per + j;
            v[j] = (j < per && i < n) ? key[i] : 0u;
        }
    };
    auto live = [&](int base, int j) { return j < per && base + tid * per + j < n; };

    uint32_t prefix = 0, mask = 0, kk = (uint32_t)k;
    // Short rows (all scores in registers): one histogram over the leading 12 bits (sign, exponent,
    // three mantissa bits: 2048 bins for non-negative values) finds the bin of the k-th largest;
    // when that bin holds at most kSelCand scores they are ranked against each other directly
    // and the four 8-bit passes below are skipped.
    bool found = false;
    if (cached) {
        for (int i = tid; i < 2048; i += NT) h12[i] = 0;
        if (tid == 0) s_ncand = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < REGS; ++j)
            if (live(0, j)) atomicAdd(&h12[digit12(v[j])], 1u);
        __syncthreads();
        // thread t takes the kBinsPer bins at positions kBinsPer t .. from the top
        uint32_t hb[kBinsPer];
        int s4 = 0;
#pragma unroll
        for (int q = 0; q < kBinsPer; ++q) {
            hb[q] = h12[2047 - (kBinsPer * tid + q)];
            s4 += (int)hb[q];
        }
        int total;
        int excl = block_excl_scan<NT / 64>(s4, s_scan, &total);
#pragma unroll
        for (int q = 0; q < kBinsPer; ++q) {
            if (hb[q] > 0 && (uint32_t)excl < kk && kk <= (uint32_t)excl + hb[q]) {
                s_prefix = (uint32_t)(2047 - (kBinsPer * tid + q));
                s_kk = kk - (uint32_t)excl;
                s_m = hb[q];
            }
            excl += (int)hb[q];
        }
        __syncthreads();
        const uint32_t bin = s_prefix, kk2 = s_kk, m = s_m;
        if ((int)m <= cand_cap) {  // uniform over the workgroup
            // the bin's scores are collected in any order (their ranks do not depend on it)
#pragma unroll
            for (int j = 0; j < REGS; ++j)
                if (live(0, j) && digit12(v[j]) == bin) cand[atomicAdd(&s_ncand, 1u)] = v[j];
            __syncthreads();
            // candidate i is the k-th largest iff (#greater) < kk2 <= (#greater) + (#equal)
            for (int i = tid; i < (int)m; i += NT) {
                const uint32_t x = cand[i];
                uint32_t gt = 0, eq = 0;
                for (int j = 0; j < (int)m; ++j) {
                    const uint32_t y = cand[j];
                    gt += y > x ? 1u : 0u;
                    eq += y == x ? 1u : 0u;
                }
                if (gt < kk2 && kk2 <= gt + eq) {  // every candidate with this value writes the same pair
                    s_tau = x;
                    s_ktau = kk2 - gt;
                }
            }
            __syncthreads();
            prefix = s_tau;
            kk = s_ktau;
            found = true;
        }
    }
    for (int pass = 0; pass < 4 && !found; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int i = tid; i < (NT / 64) * 256; i += NT) (&hist[0][0])[i] = 0;
        __syncthreads();
        for (int base = 0; base < n; base += kSpan) {
            if (!cached) load_sweep(base);
            // Scores share their leading bits, so in the first passes most of a thread's scores fall
            // into one bin and whole waves collide on it: each thread counts the scores that share
            // the digit of its first candidate itself and adds them once; the others add one by one.
            int d0 = -1, c0 = 0;
#pragma unroll
            for (int j = 0; j < REGS; ++j)
                if (live(base, j) && (v[j] & mask) == prefix) {
                    const int dgt = (int)((v[j] >> shift) & 255u);
                    if (d0 < 0) d0 = dgt;
                    if (dgt == d0) ++c0;
                    else atomicAdd(&hist[wave][dgt], 1u);
                }
            if (c0 > 0) atomicAdd(&hist[wave][d0], (uint32_t)c0);
        }
        __syncthreads();
        // position p = 255 - bin; the k-th largest lies in the bin whose prefix count first reaches kk
        int h = 0;
        if (tid < 256) {
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) h += (int)hist[w][255 - tid];
        }
        int total;
        const int excl = block_excl_scan<NT / 64>(h, s_scan, &total);
        if (tid < 256 && h > 0 && (uint32_t)excl < kk && kk <= (uint32_t)(excl + h)) {
            s_prefix = prefix | ((uint32_t)(255 - tid) << shift);
            s_kk = kk - (uint32_t)excl;
        }
        __syncthreads();
        prefix = s_prefix;
        kk = s_kk;
        mask |= 255u << shift;
    }
    const uint32_t tau = prefix;  // bit pattern of the k-th largest score; kk of the entries equal to it are kept

    // ordered compaction: count per thread, one scan per sweep, then each thread writes its slice in order
    int base_gt = 0, base_eq = 0;
    for (int base = 0; base < n; base += kSpan) {
        if (!cached) load_sweep(base);
        int c_gt = 0, c_eq = 0;
#pragma unroll
        for (int j = 0; j < REGS; ++j)
            if (live(base, j)) {
                c_gt += v[j] > tau ? 1 : 0;
                c_eq += v[j] == tau ? 1 : 0;
            }
        // both counts in one scan: a sweep has at most 2^14 scores, so each count fits 16 bits
        int tot;
        const int before = block_excl_scan<NT / 64>(c_gt | (c_eq << 16), s_scan, &tot);
        const int tot_gt = tot & 0xffff, tot_eq = tot >> 16;
        int gt_before = base_gt + (before & 0xffff);
        int eq_before = base_eq + (before >> 16);
#pragma unroll
        for (int j = 0; j < REGS; ++j)
            if (live(base, j)) {
                const bool gt = v[j] > tau, eq = v[j] == tau;
                if (gt || (eq && eq_before < (int)kk)) out[gt_before + min(eq_before, (int)kk)] = base + tid * per + j;
                gt_before += gt ? 1 : 0;
                eq_before += eq ? 1 : 0;
            }
        base_gt += tot_gt;
        base_eq += tot_eq;
    }
}

// One workgroup copies kGatherRows rows of K and of V; workgroups stride over the rows of a unit.
template <typename T, int D>
__global__ __launch_bounds__(256) void gather_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll, air_strides st) {
    const int u = blockIdx.y;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const air_seq sq = t.seq_tab[b];
    const int kl = t.budgets[(int64_t)b * dm.L + l];
    const int n_rows = sq.seq_len - sq.vis_len + kl;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
    const int32_t *idx = t.indices + unit * dm.max_vis;
    const T *ksrc = (const T *)ll.p[li].k + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const T *vsrc = (const T *)ll.p[li].v + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const int64_t dst_row0 = ((int64_t)b * dm.Hkv + kvh) * dm.pool_rows + t.layer_off[(int64_t)b * dm.L + l];
    T *kdst = (T *)t.kcache + dst_row0 * D;
    T *vdst = (T *)t.vcache + dst_row0 * D;
    constexpr int kVecPerRow = D * (int)sizeof(T) / 16;
    constexpr int kElemPerVec = 16 / (int)sizeof(T);
    for (int r0 = blockIdx.x * kGatherRows; r0 < n_rows; r0 += gridDim.x * kGatherRows) {
        for (int v = threadIdx.x; v < kGatherRows * kVecPerRow; v += 256) {
            const int j = r0 + v / kVecPerRow, c = (v % kVecPerRow) * kElemPerVec;
            if (j >= n_rows) break;
            int tok;
            if (j < sq.vis_start) tok = j;
            else if (j < sq.vis_start + kl) tok = sq.vis_start + idx[j - sq.vis_start];
            else tok = sq.vis_start + sq.vis_len + (j - sq.vis_start - kl);
            const uint4 kx = *reinterpret_cast<const uint4 *>(ksrc + (int64_t)tok * st.kv_t + c);
            const uint4 vx = *reinterpret_cast<const uint4 *>(vsrc + (int64_t)tok * st.kv_t + c);
            *reinterpret_cast<uint4 *>(kdst + (int64_t)j * D + c) = kx;
            *reinterpret_cast<uint4 *>(vdst + (int64_t)j * D + c) = vx;
        }
    }
}

// bf16 / head_dim 128: the cache is written in the layouts the decode kernel feeds to MFMA.  One
// workgroup stages the 32 gathered K and V rows of a block in LDS and writes K' as two 16-token
// tiles (see k_tiled) and V' block-transposed (see v_tiled).
// Slots of the last block that have no token yet are written as zeros.
__global__ __launch_bounds__(256) void gather_vt_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll, air_strides st) {
    constexpr int D = 128;
    typedef bf16_t T;
    const int kvh = blockIdx.y;  // grid (workgroup of the unit, KV head, sequence + B * layer)
    int b, li;
    seq_layer_of(dm, (int)blockIdx.z, b, li);
    const int l = l0 + li;
    const air_seq sq = t.seq_tab[b];
    const int kl = t.budgets[(int64_t)b * dm.L + l];
    const int n_rows = sq.seq_len - sq.vis_len + kl;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
    const int32_t *idx = t.indices + unit * dm.max_vis;
    const T *ksrc = (const T *)ll.p[li].k + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const T *vsrc = (const T *)ll.p[li].v + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const int64_t dst_row0 = ((int64_t)b * dm.Hkv + kvh) * dm.pool_rows + t.layer_off[(int64_t)b * dm.L + l];
    T *kdst = (T *)t.kcache + dst_row0 * D;
    T *vdst = (T *)t.vcache + dst_row0 * D;
    if (t.dec_steps && blockIdx.x == 0 && threadIdx.x == 0) {  // a fresh cache: nothing appended yet, cache-full flag down
        t.dec_steps[unit] = 0;
        if (blockIdx.y == 0 && blockIdx.z == 0) t.dec_steps[(int64_t)dm.L * dm.B * dm.Hkv] = 0;
    }
    __shared__ bf16_t tile[32][D + 8];   // V rows, indexed [slot][column]; +8 keeps the 16-byte row alignment and spreads banks
    __shared__ bf16_t ktile[32][D + 8];  // K rows, indexed [row][column]
    // Two 16-byte pieces of K and of V per thread and block of 32 rows.  The rows of the workgroup's next block are
    // requested before the current block is written out, so that its index and row reads (two dependent
    // round trips) run under the stores.
    uint4 kx[2], vx[2];
    auto fetch = [&](int r0) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int v = threadIdx.x + 256 * it;
            const int row = v >> 4, c = (v & 15) * 8;
            const int j = r0 + row;
            kx[it] = make_uint4(0, 0, 0, 0);
            vx[it] = kx[it];
            if (j < n_rows) {
                int tok;
                if (j < sq.vis_start) tok = j;
                else if (j < sq.vis_start + kl) tok = sq.vis_start + idx[j - sq.vis_start];
                else tok = sq.vis_start + sq.vis_len + (j - sq.vis_start - kl);
                kx[it] = *reinterpret_cast<const uint4 *>(ksrc + (int64_t)tok * st.kv_t + c);
                vx[it] = *reinterpret_cast<const uint4 *>(vsrc + (int64_t)tok * st.kv_t + c);
            }
        }
    };
    const int stride = gridDim.x * 32;
    if ((int)blockIdx.x * 32 < n_rows) fetch(blockIdx.x * 32);
    for (int r0 = blockIdx.x * 32; r0 < n_rows; r0 += stride) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int v = threadIdx.x + 256 * it;
            const int row = v >> 4, c = (v & 15) * 8;
            *reinterpret_cast<uint4 *>(&ktile[row][c]) = kx[it];
            *reinterpret_cast<uint4 *>(&tile[v_slot(row)][c]) = vx[it];
        }
        if (r0 + stride < n_rows) fetch(r0 + stride);
        lds_barrier();  // LDS traffic only: the requested rows of the next block stay in flight
        // K': the two 16-token tiles of the block in k_tiled order, 16 bytes per thread, consecutive in memory
        for (int v = threadIdx.x; v < 32 * 16; v += 256) {
            const int tl = v >> 8, sl = (v >> 6) & 3, n = (v >> 2) & 15, c = v & 3;
            *reinterpret_cast<uint4 *>(kdst + (int64_t)r0 * D + (int64_t)v * 8) =
                *reinterpret_cast<const uint4 *>(&ktile[16 * tl + n][32 * sl + 8 * c]);
        }
        // V': the block in v_tiled order, 8 slots of one column per thread, consecutive in memory
        for (int v = threadIdx.x; v < D * 4; v += 256) {
            const int j = v >> 6, c = (v >> 4) & 3, col = 16 * j + (v & 15);
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = (uint32_t)tile[8 * c + 2 * i][col] | ((uint32_t)tile[8 * c + 2 * i + 1][col] << 16);
            *reinterpret_cast<uint4 *>(vdst + (int64_t)r0 * D + (int64_t)v * 8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
        lds_barrier();  // LDS traffic only: the requested rows of the next block stay in flight
    }
}

// The same compaction INSIDE the prompt's own K / V tensors (token stride == head_dim, so a unit is a contiguous
// run of rows): block j of the compacted cache (rows 32 j .. 32 j + 31, K' tiled, V' block-transposed) lands on
// the 8 KB that source rows 32 j .. 32 j + 31 occupy.  A kept token never moves backwards (compact row <= source
// row), so the sources of block j lie at rows >= 32 j and the rows a block overwrites are needed by that block
// and earlier ones only: ONE workgroup per unit walks the blocks front to back and reads a block's sources
// (into registers, then LDS) before it stores the block.  Reading the NEXT block's sources ahead of the current
// block's stores is safe as well (they lie behind the rows being overwritten), which keeps the index and row
// reads of block j + 1 in flight under the stores of block j.
__global__ __launch_bounds__(256) void gather_in_place_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll, air_strides st) {
    constexpr int D = 128;
    typedef bf16_t T;
    const int kvh = blockIdx.x;  // grid (KV head, sequence + B * layer)
    int b, li;
    seq_layer_of(dm, (int)blockIdx.y, b, li);
    const int l = l0 + li;
    const air_seq sq = t.seq_tab[b];
    const int kl = t.budgets[(int64_t)b * dm.L + l];
    const int n_rows = sq.seq_len - sq.vis_len + kl;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
    const int32_t *idx = t.indices + unit * dm.max_vis;
    T *kbase = (T *)const_cast<void *>(ll.p[li].k) + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    T *vbase = (T *)const_cast<void *>(ll.p[li].v) + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    if (threadIdx.x == 0) {
        if (kvh == 0 && b == 0) {  // where the decode kernel finds this layer's cache from now on
            t.cache_ptrs[l].k = const_cast<void *>(ll.p[li].k);
            t.cache_ptrs[l].v = const_cast<void *>(ll.p[li].v);
        }
        if (t.dec_steps) {  // a fresh cache: nothing appended yet, cache-full flag down
            t.dec_steps[unit] = 0;
            if (blockIdx.x == 0 && blockIdx.y == 0) t.dec_steps[(int64_t)dm.L * dm.B * dm.Hkv] = 0;
        }
    }
    __shared__ bf16_t tile[32][D + 8];   // V rows, indexed [slot][column]
    __shared__ bf16_t ktile[32][D + 8];  // K rows, indexed [row][column]
    uint4 kx[2], vx[2];
    auto fetch = [&](int r0) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int v = threadIdx.x + 256 * it;
            const int row = v >> 4, c = (v & 15) * 8;
            const int j = r0 + row;
            kx[it] = make_uint4(0, 0, 0, 0);
            vx[it] = kx[it];
            if (j < n_rows) {
                int tok;
                if (j < sq.vis_start) tok = j;
                else if (j < sq.vis_start + kl) tok = sq.vis_start + idx[j - sq.vis_start];
                else tok = sq.vis_start + sq.vis_len + (j - sq.vis_start - kl);
                kx[it] = *reinterpret_cast<const uint4 *>(kbase + (int64_t)tok * D + c);
                vx[it] = *reinterpret_cast<const uint4 *>(vbase + (int64_t)tok * D + c);
            }
        }
    };
    if (n_rows > 0) fetch(0);
    for (int r0 = 0; r0 < n_rows; r0 += 32) {
        // the wait for this block's rows (a use of kx / vx) comes before any store of this block
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int v = threadIdx.x + 256 * it;
            const int row = v >> 4, c = (v & 15) * 8;
            *reinterpret_cast<uint4 *>(&ktile[row][c]) = kx[it];
            *reinterpret_cast<uint4 *>(&tile[v_slot(row)][c]) = vx[it];
        }
        if (r0 + 32 < n_rows) fetch(r0 + 32);  // rows >= r0 + 32: untouched by the stores below
        __syncthreads();  // every thread's rows of this block are in LDS (and therefore read) before the block is overwritten
        for (int v = threadIdx.x; v < 32 * 16; v += 256) {
            const int sl = (v >> 6) & 3, tl = v >> 8, n = (v >> 2) & 15, c = v & 3;
            *reinterpret_cast<uint4 *>(kbase + (int64_t)r0 * D + (int64_t)v * 8) =
                *reinterpret_cast<const uint4 *>(&ktile[16 * tl + n][32 * sl + 8 * c]);
        }
        for (int v = threadIdx.x; v < D * 4; v += 256) {
            const int j = v >> 6, c = (v >> 4) & 3, col = 16 * j + (v & 15);
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = (uint32_t)tile[8 * c + 2 * i][col] | ((uint32_t)tile[8 * c + 2 * i + 1][col] << 16);
            *reinterpret_cast<uint4 *>(vbase + (int64_t)r0 * D + (int64_t)v * 8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
        __syncthreads();  // LDS is free for the next block; the next block's rows were requested above, before these stores
    }
}

hipError_t launch_gather_in_place(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, const LaunchLayers &ll,
                                  const air_strides &st) {
    hipLaunchKernelGGL(gather_in_place_kernel, dim3(dm.Hkv, nl * dm.B), dim3(256), 0, s, dm, t, l0, ll, st);
    return hipGetLastError();
}

// threads: 256 | 512, 0 = chosen here; direct_max: largest deciding bin that is ranked directly (0 = always the radix
// passes), negative = kSelCand
hipError_t launch_select(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, int threads, int direct_max) {
    const int cap = direct_max < 0 || direct_max > kSelCand ? kSelCand : direct_max;
    // Many short rows take workgroups of 256 threads (cheaper barriers and scans, more workgroups per CU:
    // 1792 rows of ~2500 scores 23 us against 38 us); few long rows are faster with 512 (112 rows of 7290
    // scores 13.7 us against 16.3 us).
    int nt = (dm.max_vis <= 4096 && nl * dm.B * dm.Hkv >= 256) ? 256 : kSelThreads;
    if (threads == 256 || threads == 512) nt = threads;
    // registers per thread: the smallest compiled count that holds a whole row (every pass walks all of a
    // thread's slots, so unused ones cost instructions); longer rows are swept 32 per thread at a time
    const int per = (dm.max_vis + nt - 1) / nt;
    const int regs = per <= 8 ? 8 : (per <= 16 ? 16 : kSelRegs);
    const dim3 grid(dm.Hkv, dm.B, nl);
#define AIR_SELECT_LAUNCH(NT_, REGS_) hipLaunchKernelGGL((select_kernel<NT_, REGS_>), grid, dim3(NT_), 0, s, dm, t, l0, cap)
    if (nt == 256) {
        if (regs == 8) AIR_SELECT_LAUNCH(256, 8);
        else if (regs == 16) AIR_SELECT_LAUNCH(256, 16);
        else AIR_SELECT_LAUNCH(256, kSelRegs);
    } else {
        if (regs == 8) AIR_SELECT_LAUNCH(kSelThreads, 8);
        else if (regs == 16) AIR_SELECT_LAUNCH(kSelThreads, 16);
        else AIR_SELECT_LAUNCH(kSelThreads, kSelRegs);
    }
#undef AIR_SELECT_LAUNCH
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t gather_launch(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl,
                                const LaunchLayers &ll, const air_strides &st) {
    hipLaunchKernelGGL((gather_kernel<T, D>), dim3(32, nl * dm.B * dm.Hkv), dim3(256), 0, s, dm, t, l0, ll, st);
    return hipGetLastError();
}

hipError_t launch_gather(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                         const LaunchLayers &ll, const air_strides &st, int wgs_per_unit) {
    if (v_transposed(dtype, dm.D)) {
        // workgroups per unit: about 4096 in the launch, so that with many units each workgroup walks several
        // blocks of 32 rows (the next block's reads run under the current block's stores); wgs_per_unit > 0 overrides
        const int units = nl * dm.B * dm.Hkv;
        int gx = (4096 + units - 1) / units;
        gx = gx < 2 ? 2 : (gx > 32 ? 32 : gx);
        if (wgs_per_unit >= 1 && wgs_per_unit <= 64) gx = wgs_per_unit;
        hipLaunchKernelGGL(gather_vt_kernel, dim3(gx, dm.Hkv, nl * dm.B), dim3(256), 0, s, dm, t, l0, ll, st);
        return hipGetLastError();
    }
    if (dtype == AIR_BF16)
        return dm.D == 128 ? gather_launch<bf16_t, 128>(s, dm, t, l0, nl, ll, st)
                           : gather_launch<bf16_t, 64>(s, dm, t, l0, nl, ll, st);
    return dm.D == 128 ? gather_launch<float, 128>(s, dm, t, l0, nl, ll, st)
                       : gather_launch<float, 64>(s, dm, t, l0, nl, ll, st);
}

}  // namespace air
