// air_score, bf16 / head_dim 128: the window-query x visual-key product (Eq.6-7) on MFMA.
//
// A workgroup of 4 waves owns one 256-key chunk of one unit (layer, sequence, KV head); each
// wave keeps its 64 keys (4 tiles of 16) in registers as MFMA B operands, loaded straight from
// global memory: lane (n = lane % 16, c = lane / 16) holds elements 8c..8c+7 of every 32-element
// slice of key n of the tile.  The elite rows of the G query heads of the group are the A
// operand, 16 rows per block, so that S[row][key] comes out with lane (key n, c) holding four
// rows of key n: the sum over window rows that Eq.8 needs is then in-lane plus two cross-lane
// steps.
//
// Eq.8 needs every row's softmax normaliser before any column can be finished, and the
// normaliser needs all keys.  Three kernels:
//
//   score_stream_kernel  reads K_v ONCE.  Per (row, chunk) it leaves the chunk maximum m and
//       sum-exp z; when the unit has at most kStashRows window rows (the elite window: a few
//       rows per head) it also stashes e = exp(s - m) per (row, key) in fp32, 4 bytes per row
//       and key against the 256 bytes of the key itself.
//   score_rows_mfma_kernel  per row: M = max over chunks (and over the elite-text columns),
//       Z = sum z exp(m - M), weight w = 1 / (R_h G Z).  Launched for the windows that turn their
//       whole span into rows; the elite window's few rows are done inside the finish kernel.
//   score_finish_kernel  units with a stash never touch K again:
//       I[key] = sum_rows e[row][key] * (w exp(m_chunk - M)).  Units with more rows (continuous
//       or all-text windows) recompute their logits from K_v: I[key] = sum_rows w exp(s - M).
//       Epilogue: the workgroup's sum of I and its second and third moments about the workgroup's own
//       mean (fp64); the unit's last workgroup to finish shifts the entries to the row mean and adds them
//       up for Eq.9-10 (raw power sums would cancel on rows of little spread: S2 - S1 mu loses
//       (mu / sigma)^2 of its digits), and, where the layers fit one wave, the last unit of a sequence
//       goes on to Eq.11 and the cache layout (air_budget_dev.h).
#include "air_device.h"
#include "air_internal.h"
#include "air_budget_dev.h"
#include <type_traits>

namespace air {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kRowsLds = 512;  // rows whose (M, w) are staged in LDS at a time (recompute path)

struct UnitCtx {
    int kvh, b, li, l, chunk, t0, G, W, R_total;
    int qbase;  // token that row 0 of the query tensor belongs to (start of the text span, or of a visual window)
    air_seq sq;
    const bf16_t *q, *k;
    int64_t hrow0, unit;
};

// row-list offsets of the heads of the group: s_pref[g] .. s_pref[g+1] are the rows of head g
__device__ __forceinline__ void head_prefix(const DevTables &t, int64_t hrow0, int G, int *s_pref) {
    if (threadIdx.x == 0) {
        int run = 0;
        for (int g = 0; g < G; ++g) {
            s_pref[g] = run;
            run += t.elite_cnt[hrow0 + g];
        }
        s_pref[G] = run;
    }
    lds_barrier();
}

__device__ __forceinline__ int head_of_row(const int *s_pref, int G, int rho) {
    int g = 0;
    while (g + 1 < G && s_pref[g + 1] <= rho) ++g;
    return g;
}

// keys of one wave: 4 tiles of 16, as MFMA B operands.  Keys past the end of the visual span re-read
// the last one (no predication in front of the loads); `valid` masks their logits.
__device__ __forceinline__ void load_keys(const UnitCtx &u, const air_strides &st, int key0, int n, int c,
                                          uint4 (&kreg)[4][4], bool (&valid)[4]) {
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) {
        const int key = key0 + 16 * tile + n;
        valid[tile] = key < u.sq.vis_len;
        const bf16_t *src = u.k + (int64_t)(u.sq.vis_start + min(key, u.sq.vis_len - 1)) * st.kv_t + 8 * c;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) kreg[tile][sl] = *reinterpret_cast<const uint4 *>(src + 32 * sl);
    }
}

// A operand of one block of 16 window rows.  MFMA row m = 4c'+i' carries list row rbase + 4i' + c'
// (c' = m / 4, i' = m % 4), so that output lane group c holds rows rbase + c, rbase + 4 + c, ...:
// with fewer than 16 rows in the block every lane group has the same number of live rows and
// loops over i stop early.
__device__ __forceinline__ void load_rows(const DevTables &t, const UnitCtx &u, const air_strides &st,
                                          const int *s_pref, int rbase, int n, int c, uint4 (&qa)[4]) {
    const int rho = rbase + 4 * (n & 3) + (n >> 2);
    const int g = head_of_row(s_pref, u.G, rho);
    const bool have = rho < u.R_total;
    int tok = u.qbase;
    if (have) tok = t.elite_idx[(u.hrow0 + g) * u.W + (rho - s_pref[g])];
    const bf16_t *qr = u.q + (int64_t)(u.kvh * u.G + g) * st.q_h + (int64_t)(tok - u.qbase) * st.q_t;
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
        qa[sl] = make_uint4(0, 0, 0, 0);
        if (have) qa[sl] = *reinterpret_cast<const uint4 *>(qr + 32 * sl + 8 * c);
    }
}

// RAW logits (dot products, before the 1/sqrt(d) scale) of a block of 16 rows against the wave's 64
// keys: lane (key n, c) gets rows rbase + 4i + c.  Maxima are taken and exchanged in raw units and
// the scale is folded into the exponential, exp((s - M) / sqrt(d)) = 2^((s - M) * kC).
constexpr float kCHi = 0.127517431974411f, kCLo = -1.1498123564379625e-09f;  // log2(e) / sqrt(128), split
__device__ __forceinline__ float exp_raw(float d) { return exp2_scaled(d, kCHi, kCLo); }
// The per-key exponentials take the one-multiply form: its rounding of d * kCHi costs a relative
// 0.7 * 2^-24 * |log2 of the result|, below 6e-6 down to the smallest fp32 the result can be.
__device__ __forceinline__ float exp_key(float d) { return __builtin_amdgcn_exp2f(d * kCHi); }

__device__ __forceinline__ void logits_of(const uint4 (&qa)[4], const uint4 (&kreg)[4][4], f32x4 (&s)[4]) {
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) {
        s[tile] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
            s[tile] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qa[sl]),
                                                              __builtin_bit_cast(bf16x8, kreg[tile][sl]), s[tile], 0, 0, 0);
    }
}

__device__ __forceinline__ void block_logits(const DevTables &t, const UnitCtx &u, const air_strides &st,
                                             const int *s_pref, int rbase, int n, int c, const uint4 (&kreg)[4][4],
                                             f32x4 (&s)[4]) {
    uint4 qa[4];
    load_rows(t, u, st, s_pref, rbase, n, c, qa);
    logits_of(qa, kreg, s);
}

// Windows with many rows per unit (a continuous or all-text window: every span token of every head is a row) keep
// the query rows of up to kLdsRows rows in LDS, so that a block of 16 rows costs four LDS reads per lane instead
// of two dependent trips to memory (row token, then row).  Rows are padded to 272 bytes: the sixteen rows a
// load touches then fall into different banks.
constexpr int kLdsRows = 128;
constexpr int kLdsRowElems = 128 + 8;
typedef bf16_t QRows[kLdsRowElems];

// rows [r0, r0 + count) of the unit's row list into s_q[0 .. count); sixteen threads per row, 16 bytes each
__device__ __forceinline__ void stage_query_rows(const DevTables &t, const UnitCtx &u, const air_strides &st, const int *s_pref,
                                                 int r0, int count, QRows *s_q) {
    for (int p = threadIdx.x; p < count * 16; p += blockDim.x) {
        const int rr = p >> 4, piece = p & 15;
        const int rho = r0 + rr;
        const int g = head_of_row(s_pref, u.G, rho);
        const int tok = t.elite_idx[(u.hrow0 + g) * u.W + (rho - s_pref[g])];
        const bf16_t *qr = u.q + (int64_t)(u.kvh * u.G + g) * st.q_h + (int64_t)(tok - u.qbase) * st.q_t;
        *reinterpret_cast<uint4 *>(&s_q[rr][8 * piece]) = *reinterpret_cast<const uint4 *>(qr + 8 * piece);
    }
}
// A operand of the block of 16 rows that starts at staged row rb (see load_rows for the row order); rows past `count` are zero
__device__ __forceinline__ void load_rows_lds(const QRows *s_q, int rb, int count, int n, int c, uint4 (&qa)[4]) {
    const int rr = rb + 4 * (n & 3) + (n >> 2);
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
        qa[sl] = make_uint4(0, 0, 0, 0);
        if (rr < count) qa[sl] = *reinterpret_cast<const uint4 *>(&s_q[rr][32 * sl + 8 * c]);
    }
}

__device__ __forceinline__ bool unit_setup(const Dims &dm, const SeqArgs &seqs, int l0, const LaunchLayers &ll,
                                           const air_strides &st, UnitCtx &u, int chunks_per_wg) {
    u.chunk = blockIdx.x * chunks_per_wg;  // first chunk of this workgroup
    u.kvh = blockIdx.y;  // grid (chunk group, KV head, sequence + B * layer)
    seq_layer_of(dm, (int)blockIdx.z, u.b, u.li);
    u.l = l0 + u.li;
    u.sq = seqs.s[u.b];  // from the kernel arguments: no table read in front of the key loads
    if (u.chunk * kChunkKeys >= u.sq.vis_len) return false;
    u.t0 = u.sq.vis_start + u.sq.vis_len;
    u.qbase = dm.vis_window ? u.sq.win_start : u.t0;
    u.G = dm.G;
    u.W = dm.max_window;
    u.q = (const bf16_t *)ll.p[u.li].q + (int64_t)u.b * st.q_b;
    u.k = (const bf16_t *)ll.p[u.li].k + (int64_t)u.b * st.kv_b + (int64_t)u.kvh * st.kv_h;
    u.hrow0 = ((int64_t)u.l * dm.B + u.b) * dm.Hq + (int64_t)u.kvh * u.G;
    u.unit = ((int64_t)u.l * dm.B + u.b) * dm.Hkv + u.kvh;
    return true;
}

// ---------------------------------------------------------------------------------------
// One workgroup streams kStreamChunks consecutive chunks of a unit; the keys of the next chunk are
// requested before the current one is scored, so that the memory pipe never drains while the
// workgroup computes.  The window rows (A operands) of the first row block are loaded once.
// Stash layout of one (unit, chunk, row): 256 floats, key 64w + 16 tile + n at position 64w + 4n + tile,
// i.e. the four tiles of a lane are one 16-byte store.
constexpr int kStreamChunks = 1;

__device__ __forceinline__ int stash_pos(int key_in_chunk) {
    return (key_in_chunk & ~63) | ((key_in_chunk & 15) << 2) | ((key_in_chunk >> 4) & 3);
}

// VIS: the rows are the tokens of a visual window (all heads have the same win_len rows); row rho sits at
// visual index prow0 + rho % win_len and sees the keys up to itself.  A (row, chunk) pair that lies wholly
// behind the row leaves the partial (-inf, 0) and zeros in the stash.
// MANY: launches whose window turns its whole span into rows (dozens to hundreds of rows per unit): the query rows are
// staged in LDS, kLdsRows at a time.
template <bool VIS, bool MANY>
__global__ __launch_bounds__(256, 4) void score_stream_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll,
                                                              air_strides st, SeqArgs seqs) {
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 15, c = lane >> 4;
    UnitCtx u;
    if (!unit_setup(dm, seqs, l0, ll, st, u, kStreamChunks)) return;
    __shared__ int s_pref[17];
    __shared__ float s_pm[4][16], s_pz[4][16], s_mw[16];

    const int nch = (u.sq.vis_len + kChunkKeys - 1) / kChunkKeys;
    const int first = u.chunk, last = min(nch, first + kStreamChunks);
    uint4 kreg[4][4], knext[4][4];
    bool valid[4], vnext[4];
    load_keys(u, st, first * kChunkKeys + wave * 64, n, c, kreg, valid);
    head_prefix(t, u.hrow0, u.G, s_pref);
    u.R_total = s_pref[u.G];
    const bool stash = u.R_total <= kStashRows;
    uint4 qa0[4];
    if (!MANY) load_rows(t, u, st, s_pref, 0, n, c, qa0);

#pragma unroll
    for (int ci = 0; ci < kStreamChunks; ++ci) {
        const int chunk = first + ci;
        if (chunk >= last) break;
        if (chunk + 1 < last) load_keys(u, st, (chunk + 1) * kChunkKeys + wave * 64, n, c, knext, vnext);
        float *stash_base = t.stash + ((u.unit * dm.n_chunks + chunk) * (int64_t)kStashRows) * kChunkKeys;
        // per (row, chunk) maximum and sum-exp of the block of 16 rows that starts at list row rb, from its logits
        auto reduce_block = [&](int rb, f32x4 (&s)[4]) __attribute__((always_inline)) {
            const int n_i = min(4, (u.R_total - rb + 3) >> 2);  // live values of i (uniform over the workgroup)
            int lim[4];  // VIS: last key of the lane's tiles that row i sees, relative to the lane's key of tile 0
#pragma unroll
            for (int i = 0; i < 4; ++i)
                lim[i] = VIS ? (u.sq.win_start - u.sq.vis_start) + (rb + 4 * i + c) % u.sq.win_len -
                                   (chunk * kChunkKeys + wave * 64 + n)
                             : 0;
            auto live = [&](int tile, int i) __attribute__((always_inline)) {
                return VIS ? (valid[tile] && 16 * tile <= lim[i]) : valid[tile];
            };
            float m[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                m[i] = -INFINITY;
                if (i >= n_i) continue;
                float mx = -INFINITY;
#pragma unroll
                for (int tile = 0; tile < 4; ++tile) mx = fmaxf(mx, live(tile, i) ? s[tile][i] : -INFINITY);
                m[i] = max16(mx);
            }
            lds_barrier();
            if (n == 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) s_pm[wave][4 * i + c] = m[i];  // indexed by list row within the block
            }
            lds_barrier();
            // chunk maximum of every row: the reference of the stashed exponentials
            float z[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                z[i] = 0.f;
                if (i >= n_i) continue;
                const int r = 4 * i + c;
                const float M = fmaxf(fmaxf(s_pm[0][r], s_pm[1][r]), fmaxf(s_pm[2][r], s_pm[3][r]));
                f32x4 e;
#pragma unroll
                for (int tile = 0; tile < 4; ++tile) e[tile] = live(tile, i) ? exp_key(s[tile][i] - M) : 0.f;
                float zz = (e[0] + e[1]) + (e[2] + e[3]);
                if (stash && rb + r < u.R_total)
                    *reinterpret_cast<f32x4 *>(stash_base + (int64_t)(rb + r) * kChunkKeys + wave * 64 + 4 * n) = e;
                z[i] = sum16(zz);
                if (wave == 0 && n == 0) s_mw[r] = M;
            }
            if (n == 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) s_pz[wave][4 * i + c] = z[i];
            }
            lds_barrier();
            if (tid < 16 && rb + tid < u.R_total) {
                const int rho = rb + tid;
                const float Z = (s_pz[0][tid] + s_pz[1][tid]) + (s_pz[2][tid] + s_pz[3][tid]);
                const int g = head_of_row(s_pref, u.G, rho);
                const int64_t slot = (u.hrow0 + g) * u.W + (rho - s_pref[g]);
                t.part[slot * dm.n_chunks + chunk] = make_float2(s_mw[tid], Z);
            }
        };
        if constexpr (!MANY) {
            for (int rb = 0; rb < u.R_total; rb += 16) {
                f32x4 s[4];
                if (rb == 0) logits_of(qa0, kreg, s);
                else block_logits(t, u, st, s_pref, rb, n, c, kreg, s);
                reduce_block(rb, s);
            }
        } else {
            __shared__ QRows s_q[kLdsRows];
            for (int rs = 0; rs < u.R_total; rs += kLdsRows) {
                const int cnt = min(kLdsRows, u.R_total - rs);
                if (rs) lds_barrier();  // the blocks of the rows staged before have been read
                stage_query_rows(t, u, st, s_pref, rs, cnt, s_q);
                lds_barrier();
                for (int rb = 0; rb < cnt; rb += 16) {
                    uint4 qa[4];
                    load_rows_lds(s_q, rb, cnt, n, c, qa);
                    f32x4 s[4];
                    logits_of(qa, kreg, s);
                    reduce_block(rs + rb, s);
                }
            }
        }
#pragma unroll
        for (int tile = 0; tile < 4; ++tile) {
            valid[tile] = vnext[tile];
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) kreg[tile][sl] = knext[tile][sl];
        }
    }
}

// ---------------------------------------------------------------------------------------
// Parameters of one window row, by one wave (every lane gets the result): M = max over the chunk
// partials and the elite-text columns (raw units), Z = sum z exp(m - M) in fp64, w = 1 / (R_h G Z).
// p0 returns the lane's own partial of the first 64 chunks.  A partial with sum 0 (a chunk wholly
// behind a visual-window row; the empty text columns of such a window) has maximum -inf and takes no part.
__device__ __forceinline__ void row_params(const DevTables &t, int64_t slot, int nch, int n_chunks, int rows_of_head, int G,
                                           int lane, float &M, float &w, float2 &p0) {
    const float2 *p = t.part + slot * n_chunks;
    const float mt = t.row_mtext[slot], zt = t.row_ztext[slot];
    p0 = lane < nch ? p[lane] : make_float2(-INFINITY, 0.f);  // the first 64 chunks stay in registers
    M = fmaxf(mt, p0.x);
    for (int cc = lane + 64; cc < nch; cc += 64) M = fmaxf(M, p[cc].x);
    M = wave_max(M);
    double Z = lane < nch && p0.y > 0.f ? (double)(p0.y * exp_raw(p0.x - M)) : 0.0;
    for (int cc = lane + 64; cc < nch; cc += 64) {
        const float2 x = p[cc];
        if (x.y > 0.f) Z += (double)(x.y * exp_raw(x.x - M));
    }
    Z = wave_sum(Z);
    if (zt > 0.f) Z += (double)(zt * exp_raw(mt - M));
    w = (float)(1.0 / ((double)rows_of_head * (double)G * Z));
}
// the factor that turns a stashed exponential of a chunk into its share of Eq.8
__device__ __forceinline__ float chunk_factor(float2 part, float M, float w) {
    return part.y > 0.f ? w * exp_raw(part.x - M) : 0.f;
}

// ---------------------------------------------------------------------------------------
// Row parameters, once per unit: one wave per window row, lanes over the chunk partials.
// M = max over chunks and the elite-text columns, Z = sum z exp(m - M) in fp64,
// w = 1 / (R_h G Z).  Units with a stash also get f[row][chunk] = w exp(m_chunk - M), the factor
// that turns a stashed exponential into its share of Eq.8.
constexpr int kRowWaves = 16;  // up to one wave per row: a unit's usual dozen rows are then done in one round of loads
__global__ __launch_bounds__(64 * kRowWaves) void score_rows_mfma_kernel(Dims dm, DevTables t, int l0, SeqArgs seqs) {
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int kvh = blockIdx.x, b = blockIdx.y, l = l0 + (int)blockIdx.z;  // grid (KV head, sequence, layer)
    const int G = dm.G, W = dm.max_window;
    const int64_t hrow0 = ((int64_t)l * dm.B + b) * dm.Hq + (int64_t)kvh * G;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
    const int nch = (seqs.s[b].vis_len + kChunkKeys - 1) / kChunkKeys;
    __shared__ int s_pref[17];
    head_prefix(t, hrow0, G, s_pref);
    const int R_total = s_pref[G];
    const bool stash = R_total <= kStashRows;
    if (tid == 0) t.unit_R[unit] = R_total;
    for (int rho = wave; rho < R_total; rho += (int)(blockDim.x >> 6)) {
        const int g = head_of_row(s_pref, G, rho);
        const int64_t slot = (hrow0 + g) * W + (rho - s_pref[g]);
        const float2 *p = t.part + slot * dm.n_chunks;
        float M, w;
        float2 p0;
        row_params(t, slot, nch, dm.n_chunks, s_pref[g + 1] - s_pref[g], G, lane, M, w, p0);
        if (lane == 0) {
            t.row_M[slot] = M;  // raw units
            t.row_w[slot] = w;
        }
        if (stash) {
            float *f = t.row_f + (unit * kStashRows + rho) * dm.n_chunks;
            if (lane < nch) f[lane] = chunk_factor(p0, M, w);
            for (int cc = lane + 64; cc < nch; cc += 64) f[cc] = chunk_factor(p[cc], M, w);
        }
    }
}

// ---------------------------------------------------------------------------------------
// One workgroup finishes kFinishChunks consecutive chunks of a unit and leaves one moment entry.
// INLINE: no row-parameter kernel has run; every workgroup forms the parameters of the unit's rows
// itself from the chunk partials (the elite window's handful of rows: cheaper than a launch).

// Eq.9-10 of one (layer, sequence, KV head) from the moment entries of its importance row, by one wave.  Entry c holds
// the sum S1_c, the mean m_c and the moments M2_c, M3_c about m_c of the n_c scores of kFinishChunks chunks.  With
// d_c = m_c - mu the central moments of the row are
//   sum (x - mu)^2 = sum_c M2_c + n_c d_c^2,   sum (x - mu)^3 = sum_c M3_c + 3 d_c M2_c + n_c d_c^3,
// sums of terms no larger than their result (raw power sums would cancel on rows of little spread).  Lane g of each row
// of sixteen lanes takes the entries g, g + 16, ... (the first two stay in registers), the sums over the entries are
// butterflies over the sixteen lanes: a fixed order, the same on every run; every operation is rounded once (no
// contraction: the budgets that follow from these numbers must not depend on how the compiler fuses them).
__device__ __forceinline__ void unit_statistics(__amdgpu_buffer_rsrc_t ers, int n_ent, int n_vis, int lane, double &st_out,
                                                double &sk_out) {
#pragma clang fp contract(off)
    constexpr int kEntryKeys = kFinishChunks * kChunkKeys;
    const int gl = lane & 15;
    auto entry = [&](int c, double (&e)[4]) __attribute__((always_inline)) {
        const int cc = min(c, n_ent - 1);
        const u32x4 lo = __builtin_amdgcn_raw_buffer_load_b128(ers, cc * 32, 0, kSysScope);
        const u32x4 hi = __builtin_amdgcn_raw_buffer_load_b128(ers, cc * 32 + 16, 0, kSysScope);
        const bool have = c < n_ent;
        e[0] = have ? __builtin_bit_cast(double, (u32x2){lo[0], lo[1]}) : 0.0;
        e[1] = have ? __builtin_bit_cast(double, (u32x2){lo[2], lo[3]}) : 0.0;
        e[2] = have ? __builtin_bit_cast(double, (u32x2){hi[0], hi[1]}) : 0.0;
        e[3] = have ? __builtin_bit_cast(double, (u32x2){hi[2], hi[3]}) : 0.0;
    };
    double e0[4], e1[4];
    entry(gl, e0);
    entry(gl + 16, e1);
    const double n = (double)n_vis;
    double s1 = e0[0] + e1[0];
    for (int c = gl + 32; c < n_ent; c += 16) {  // beyond 32768 visual tokens
        double ex[4];
        entry(c, ex);
        s1 += ex[0];
    }
    const double S1 = sum16(s1);
    const double mu = S1 / n;
    double c2 = 0.0, c3 = 0.0;
    auto add = [&](int c, const double (&e)[4]) __attribute__((always_inline)) {
        if (c < n_ent) {
            const double nc = (double)min(kEntryKeys, n_vis - c * kEntryKeys);
            const double dl = e[1] - mu, M2 = e[2], M3 = e[3];
            c2 += M2 + nc * (dl * dl);
            c3 += (M3 + 3.0 * dl * M2) + nc * (dl * dl * dl);
        }
    };
    add(gl, e0);
    add(gl + 16, e1);
    for (int c = gl + 32; c < n_ent; c += 16) {
        double ex[4];
        entry(c, ex);
        add(c, ex);
    }
    c2 = sum16(c2);
    c3 = sum16(c3);
    double sk = 0.0;
    if (n_vis >= 3) {
        const double sigma = sqrt(c2 / (n - 1.0));
        // zero spread (Eq.10 undefined; taken as 0): a standard deviation at most 1e-6 of the mean
        if (sigma > 1e-6 * fabs(mu)) sk = n / ((n - 1.0) * (n - 2.0)) * (c3 / (sigma * sigma * sigma));
    }
    st_out = S1;
    sk_out = sk;
}

// MANY: as in the stream kernel, the query rows of the recompute path are staged in LDS.
template <bool VIS, bool INLINE, bool MANY>
__global__ __launch_bounds__(256, 4) void score_finish_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll,
                                                           air_strides st, SeqArgs seqs) {
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 15, c = lane >> 4;
    UnitCtx u;
    if (!unit_setup(dm, seqs, l0, ll, st, u, kFinishChunks)) return;
    __shared__ int s_pref[17];
    __shared__ float s_M[kRowsLds], s_w[kRowsLds];
    __shared__ float s_f[kFinishChunks][kStashRows];
    __shared__ double s_mom[4][3];

    const int nch = (u.sq.vis_len + kChunkKeys - 1) / kChunkKeys;
    const int first = u.chunk, last = min(nch, first + kFinishChunks);
    // factor table of the stash path goes out before anything else; rows past R_total are never used
    float f_mine = 0.f;
    if (!INLINE) {
        if (tid < kFinishChunks * kStashRows && first + tid / kStashRows < last)
            f_mine = t.row_f[(u.unit * kStashRows + (tid % kStashRows)) * dm.n_chunks + first + tid / kStashRows];
        u.R_total = t.unit_R[u.unit];
    } else {
        head_prefix(t, u.hrow0, u.G, s_pref);
        u.R_total = s_pref[u.G];
    }
    const bool stash = u.R_total <= kStashRows;
    if (!INLINE && !stash) head_prefix(t, u.hrow0, u.G, s_pref);

    // Moments of the workgroup's scores, every sum in a fixed order: S1 = sum x, the workgroup mean S1 / n, then
    // M2 = sum (x - mean)^2 and M3 = sum (x - mean)^3 in fp64.  One entry (S1, mean, M2, M3) per workgroup.
    const int n_wg = min(u.sq.vis_len, last * kChunkKeys) - first * kChunkKeys;  // scores of this workgroup
    auto wg_sum = [&](double v, int slot) {
        v = wave_sum(v);
        if (lane == 0) s_mom[wave][slot] = v;
        lds_barrier();
        return ((s_mom[0][slot] + s_mom[1][slot]) + s_mom[2][slot]) + s_mom[3][slot];
    };
    auto put_moments = [&](const auto &x, const auto &ok) __attribute__((always_inline)) {
        constexpr int NX = sizeof(x) / sizeof(x[0]);
        double s1 = 0.0;
#pragma unroll
        for (int i = 0; i < NX; ++i) s1 += ok[i] ? (double)x[i] : 0.0;
        const double S1 = wg_sum(s1, 0);
        const double mean = S1 / (double)n_wg;
        double m2 = 0.0, m3 = 0.0;
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const double dlt = ok[i] ? (double)x[i] - mean : 0.0;
            m2 += dlt * dlt;
            m3 += dlt * dlt * dlt;
        }
        m2 = wave_sum(m2);
        m3 = wave_sum(m3);
        if (lane == 0) {
            s_mom[wave][1] = m2;
            s_mom[wave][2] = m3;
        }
        lds_barrier();
        if (wave != 0) return;
        // The entry goes out written through to memory, and the workgroup then counts itself at the unit's arrival
        // counter; the one that counts last (every entry of the unit is in memory by then: each writer waited for its
        // stores before it counted) turns the entries into the unit's strength and skewness.  The ordering is that of
        // the decode kernel's exchange of partials: write-through stores, s_waitcnt, a relaxed device-scope
        // read-modify-write, loads that bypass the caches.
        double *mo_unit = t.moments + u.unit * dm.n_entries * 4;
        const __amdgpu_buffer_rsrc_t ers = __builtin_amdgcn_make_buffer_rsrc(mo_unit, 0, dm.n_entries * 32, 0x00020000);
        if (lane < 4) {
            const double r = lane == 0 ? S1 : (lane == 1 ? mean : ((s_mom[0][lane - 1] + s_mom[1][lane - 1]) + s_mom[2][lane - 1]) + s_mom[3][lane - 1]);
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, r), ers, (int)blockIdx.x * 32 + lane * 8, 0, kSysScope);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        int prev = 0;
        if (lane == 0) prev = __hip_atomic_fetch_add(&t.unit_cnt[u.unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        prev = __builtin_amdgcn_readfirstlane(prev);
        const int n_ent = (nch + kFinishChunks - 1) / kFinishChunks;  // workgroups of this unit
        if (prev != n_ent - 1) return;
        if (lane == 0) __hip_atomic_store(&t.unit_cnt[u.unit], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
        double unit_st, unit_sk;
        unit_statistics(ers, n_ent, u.sq.vis_len, lane, unit_st, unit_sk);
        if (!dm.fuse_budget) {
            if (lane == 0) {
                t.unit_st[u.unit] = unit_st;
                t.unit_sk[u.unit] = unit_sk;
            }
            return;
        }
        // The same once more, one level up: the unit's statistics go out written through, the wave counts the unit at
        // its sequence's arrival counter, and the wave that counts the last of the L * H_kv units does Eq.11 and the
        // cache layout of the sequence (the layers fit one wave): air_budget has nothing left to launch.
        const int64_t all_units = (int64_t)dm.L * dm.B * dm.Hkv;
        const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(t.unit_st, 0, (int)(all_units * 8), 0x00020000);
        const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(t.unit_sk, 0, (int)(all_units * 8), 0x00020000);
        if (lane == 0) {
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, unit_st), srs, (int)u.unit * 8, 0, kSysScope);
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, unit_sk), krs, (int)u.unit * 8, 0, kSysScope);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        prev = 0;
        if (lane == 0) prev = __hip_atomic_fetch_add(&t.seq_cnt[u.b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        prev = __builtin_amdgcn_readfirstlane(prev);
        if (prev != dm.L * dm.Hkv - 1) return;
        if (lane == 0) __hip_atomic_store(&t.seq_cnt[u.b], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next prompt
        __shared__ double s_a0[64], s_a1[64], s_frac[64];
        __shared__ int s_i0[64], s_i1[64];
        allocate_and_lay_out<true>(dm, t, u.b, u.sq, dm.retention, dm.budget_mode, dm.min_keep, false, lane, s_a0, s_a1, s_frac,
                                   s_i0, s_i1, [&](int l, double &a, double &c) __attribute__((always_inline)) {
                                       // all heads' loads go out together; the sums run left to right over the live ones
                                       u32x2 vs[16], vk[16];
#pragma unroll
                                       for (int h = 0; h < 16; ++h) {
                                           const int off = (int)((((int64_t)l * dm.B + u.b) * dm.Hkv + min(h, dm.Hkv - 1)) * 8);
                                           vs[h] = __builtin_amdgcn_raw_buffer_load_b64(srs, off, 0, kSysScope);
                                           vk[h] = __builtin_amdgcn_raw_buffer_load_b64(krs, off, 0, kSysScope);
                                       }
#pragma unroll
                                       for (int h = 0; h < 16; ++h) {
                                           if (h < dm.Hkv) {
                                               a += __builtin_bit_cast(double, vs[h]);
                                               c += __builtin_bit_cast(double, vk[h]);
                                           }
                                       }
                                   });
    };

    if (stash) {
        // factors f[chunk][row] into LDS: read from the table the row-parameter kernel left, or formed
        // here, a wave per row (rows past the list get zero)
        auto put_factors = [&]() __attribute__((always_inline)) {
            if (!INLINE) {
                if (tid < kFinishChunks * kStashRows) s_f[tid / kStashRows][tid % kStashRows] = (tid % kStashRows) < u.R_total ? f_mine : 0.f;
            } else {
                // a row of 16 lanes per window row (16 rows at a time), a lane takes every 16th chunk
                // partial: all loads of a round go out together and the reductions stay inside the row
                if (tid < kFinishChunks * kStashRows && (tid % kStashRows) >= u.R_total) s_f[tid / kStashRows][tid % kStashRows] = 0.f;
                const int grp = tid >> 4, gl = tid & 15;
                for (int r0 = 0; r0 < u.R_total; r0 += 16) {
                    const int rho = min(r0 + grp, u.R_total - 1);  // a row group past the list repeats the last row and stores nothing
                    const int g = head_of_row(s_pref, u.G, rho);
                    const int64_t slot = (u.hrow0 + g) * u.W + (rho - s_pref[g]);
                    const float2 *p = t.part + slot * dm.n_chunks;
                    const float mt = t.row_mtext[slot], zt = t.row_ztext[slot];
                    const float2 pf = p[min(first + gl, nch - 1)];  // the partial a factor is made of (lanes 0 .. 3)
                    float2 pc[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) pc[k] = gl + 16 * k < nch ? p[gl + 16 * k] : make_float2(-INFINITY, 0.f);
                    float M = mt;
#pragma unroll
                    for (int k = 0; k < 4; ++k) M = fmaxf(M, pc[k].x);
                    for (int cc = gl + 64; cc < nch; cc += 16) M = fmaxf(M, p[cc].x);
                    M = max16(M);
                    double Z = 0.0;
#pragma unroll
                    for (int k = 0; k < 4; ++k) Z += pc[k].y > 0.f ? (double)(pc[k].y * exp_raw(pc[k].x - M)) : 0.0;
                    for (int cc = gl + 64; cc < nch; cc += 16) {
                        const float2 x = p[cc];
                        if (x.y > 0.f) Z += (double)(x.y * exp_raw(x.x - M));
                    }
                    Z = sum16(Z);
                    if (zt > 0.f) Z += (double)(zt * exp_raw(mt - M));
                    const float w = (float)(1.0 / ((double)(s_pref[g + 1] - s_pref[g]) * (double)u.G * Z));
                    if (r0 + grp < u.R_total && gl < kFinishChunks) s_f[gl][rho] = first + gl < last ? chunk_factor(pf, M, w) : 0.f;
                }
            }
            lds_barrier();
        };
        // One wave per chunk; a lane takes 16 bytes of every stashed row (four keys, 16 apart: see
        // stash_pos) and all rows of a round are requested at once, in front of the factors.  Rows past
        // the list re-read its last row against a zero factor, a wave past the last chunk re-reads the
        // last chunk and stores nothing.
        const int ci = wave, chunk = first + ci;
        const float *sb = t.stash + ((u.unit * dm.n_chunks + min(chunk, last - 1)) * (int64_t)kStashRows) * kChunkKeys + 4 * lane;
        f32x4 imp = (f32x4){0.f, 0.f, 0.f, 0.f};
        auto get_rows = [&](auto &e, int r0) __attribute__((always_inline)) {
            constexpr int RB = sizeof(e) / sizeof(e[0]);
#pragma unroll
            for (int r = 0; r < RB; ++r)
                e[r] = *reinterpret_cast<const f32x4 *>(sb + (int64_t)min(r0 + r, max(u.R_total - 1, 0)) * kChunkKeys);
        };
        auto add_rows = [&](const auto &e, int r0) __attribute__((always_inline)) {
            constexpr int RB = sizeof(e) / sizeof(e[0]);
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const float f = s_f[ci][r0 + r];
#pragma unroll
                for (int i = 0; i < 4; ++i) imp[i] = fmaf(f, e[r][i], imp[i]);
            }
        };
        static_assert(kFinishChunks == 4, "one wave of the workgroup per chunk");
        static_assert(kStashRows == 32, "rows beyond 16 are taken in a second round of 16");
        bool ok[4] = {false, false, false, false};
        if (u.R_total == 0) {  // no window row: the importance is zero (and so are its moments)
            for (int key = first * kChunkKeys + tid; key < min(last * kChunkKeys, u.sq.vis_len); key += 256)
                t.scores[u.unit * dm.max_vis + key] = 0.f;
        } else {
            // 16 rows in flight at most: 32 at once would cost the kernel half of its occupancy
            if (u.R_total <= 8) {
                f32x4 e[8];
                get_rows(e, 0);
                put_factors();
                add_rows(e, 0);
            } else {
                f32x4 e[16];
                get_rows(e, 0);
                put_factors();
                add_rows(e, 0);
                if (u.R_total > 16) {
                    get_rows(e, 16);
                    add_rows(e, 16);
                }
            }
            if (chunk < last) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int key = chunk * kChunkKeys + 64 * (lane >> 4) + 16 * i + (lane & 15);
                    ok[i] = key < u.sq.vis_len;
                    if (ok[i]) t.scores[u.unit * dm.max_vis + key] = imp[i];
                }
            }
        }
        const float xs[4] = {imp[0], imp[1], imp[2], imp[3]};
        put_moments(xs, ok);
        return;
    }
    // recompute path: (M, w) of a block of rows staged from the row tables
    auto stage_rows = [&](int rs, int rows) {
        __syncthreads();
        if (!INLINE) {
            for (int rr = tid; rr < rows; rr += 256) {
                const int rho = rs + rr;
                const int g = head_of_row(s_pref, u.G, rho);
                const int64_t slot = (u.hrow0 + g) * u.W + (rho - s_pref[g]);
                s_M[rr] = t.row_M[slot];
                s_w[rr] = t.row_w[slot];
            }
        } else {
            for (int rr = wave; rr < rows; rr += 4) {
                const int rho = rs + rr;
                const int g = head_of_row(s_pref, u.G, rho);
                const int64_t slot = (u.hrow0 + g) * u.W + (rho - s_pref[g]);
                float M, w;
                float2 p0;
                row_params(t, slot, nch, dm.n_chunks, s_pref[g + 1] - s_pref[g], u.G, lane, M, w, p0);
                if (lane == 0) {
                    s_M[rr] = M;
                    s_w[rr] = w;
                }
            }
        }
        __syncthreads();
    };
    for (int chunk = first; chunk < last; ++chunk) {
        u.chunk = chunk;
        const int key0 = chunk * kChunkKeys + wave * 64;
        uint4 kreg[4][4];
        bool valid[4];
        load_keys(u, st, key0, n, c, kreg, valid);
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int rs = 0; rs < u.R_total; rs += kRowsLds) {
            const int rows_here = min(kRowsLds, u.R_total - rs);
            if (chunk == first || u.R_total > kRowsLds) stage_rows(rs, rows_here);
            for (int rb = 0; rb < rows_here; rb += 16) {
                f32x4 s[4];
                if constexpr (MANY) {
                    // the query rows of rows rs + [qs, qs + kLdsRows) are in LDS; they are staged once per workgroup when the
                    // unit has no more rows than that, else again for every chunk
                    __shared__ QRows s_q[kLdsRows];
                    const int qs = rb / kLdsRows * kLdsRows, cnt = min(kLdsRows, rows_here - qs);
                    if (rb == qs && (chunk == first || u.R_total > kLdsRows)) {
                        lds_barrier();  // the blocks of the rows staged before have been read
                        stage_query_rows(t, u, st, s_pref, rs + qs, cnt, s_q);
                        lds_barrier();
                    }
                    uint4 qa[4];
                    load_rows_lds(s_q, rb - qs, cnt, n, c, qa);
                    logits_of(qa, kreg, s);
                } else {
                    block_logits(t, u, st, s_pref, rs + rb, n, c, kreg, s);
                }
                const int n_i = min(4, (rows_here - rb + 3) >> 2);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (i >= n_i) continue;
                    const int rr = rb + 4 * i + c;
                    const bool have = rr < rows_here;
                    const float M = have ? s_M[rr] : 0.f;
                    const float w = have ? s_w[rr] : 0.f;
                    // visual window: the row sees the keys up to its own visual index
                    const int lim = VIS ? (u.sq.win_start - u.sq.vis_start) + (rs + rr) % u.sq.win_len - (key0 + n) : 0;
#pragma unroll
                    for (int tile = 0; tile < 4; ++tile) {
                        const float e = exp_key(s[tile][i] - M);
                        acc[tile] = fmaf(w, VIS && 16 * tile > lim ? 0.f : e, acc[tile]);
                    }
                }
            }
        }
#pragma unroll
        for (int tile = 0; tile < 4; ++tile) {
            float v = acc[tile];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (c == 0 && valid[tile]) t.scores[u.unit * dm.max_vis + key0 + 16 * tile + n] = v;
        }
    }
    // the moments need every score of the workgroup at once: each lane reads back the ones it stored itself
    float xs[kFinishChunks * 4];
    bool ok[kFinishChunks * 4];
#pragma unroll
    for (int ci = 0; ci < kFinishChunks; ++ci)
#pragma unroll
        for (int tile = 0; tile < 4; ++tile) {
            const int key = (first + ci) * kChunkKeys + wave * 64 + 16 * tile + n;
            ok[4 * ci + tile] = c == 0 && first + ci < last && key < u.sq.vis_len;
            xs[4 * ci + tile] = ok[4 * ci + tile] ? t.scores[u.unit * dm.max_vis + key] : 0.f;
        }
    put_moments(xs, ok);
}

// ---------------------------------------------------------------------------------------
// Eq.4-5 for bf16 / head_dim 128.  One workgroup per (KV head, sequence, layer).
//   phase 1: raw last-row logits of the G heads against every candidate text key on MFMA
//            (fp32 accumulation), into LDS.
//   phase 2: one wave per head.  Eq.5 is decided as the fp64 test exp((a_j - a_max)/sqrt(d)) >= alpha.
//            The fp32 logits settle every candidate that is not within kEliteMargin of the
//            threshold; the maximum and the few candidates inside the margin are recomputed as
//            exact fp64 dot products (bf16 products are exact, the sum is fp64) before deciding.
//            Then the ordered compaction of the elite positions and the elite-text columns of Eq.7.
// ---------------------------------------------------------------------------------------
constexpr int kEliteWaves = 8;      // phase 2 takes one head per wave
constexpr float kEliteMargin = 4e-3f;  // raw-logit units; fp32 accumulation of 128 bf16 products of this size errs by < 1e-3

__device__ __forceinline__ double dot64_wave(const bf16_t *a, const bf16_t *b, int lane) {
    const uint32_t ua = reinterpret_cast<const uint32_t *>(a)[lane], ub = reinterpret_cast<const uint32_t *>(b)[lane];
    const double p = (double)__uint_as_float(ua << 16) * (double)__uint_as_float(ub << 16) +
                     (double)__uint_as_float(ua & 0xffff0000u) * (double)__uint_as_float(ub & 0xffff0000u);
    return wave_sum(p);
}

__global__ __launch_bounds__(64 * kEliteWaves) void elite_mfma_kernel(Dims dm, DevTables t, int l0, LaunchLayers ll, air_strides st,
                                                         SeqArgs seqs, double alpha, double ln_alpha, int gb) {
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 15, c = lane >> 4;
    const int kvh = blockIdx.x, b = blockIdx.y, li = blockIdx.z;
    const int l = l0 + li;
    const air_seq sq = seqs.s[b];
    if (li == 0 && kvh == 0 && tid == 0) t.seq_tab[b] = sq;
    const int t0 = sq.vis_start + sq.vis_len;
    const int G = dm.G, W = dm.max_window, wl = sq.win_len;
    const bf16_t *qb = (const bf16_t *)ll.p[li].q + (int64_t)b * st.q_b;
    const bf16_t *k = (const bf16_t *)ll.p[li].k + (int64_t)b * st.kv_b + (int64_t)kvh * st.kv_h;
    const int ref = sq.win_start + wl - 1;
    extern __shared__ float s_dynf[];  // gb * max_window raw logits, then as many ints (elite lists)
    float *s_logit = s_dynf;
    int *s_elite = reinterpret_cast<int *>(s_dynf + (size_t)gb * W);
    const double inv_sqrt_d = 0.08838834764831845;  // 1 / sqrt(128), correctly rounded
    const float scale = 0.08838834764831845f;

    for (int g0 = 0; g0 < G; g0 += gb) {
        const int ng = min(gb, G - g0);
        // ---- phase 1: A = reference queries of heads g0 .. g0+ng-1 (MFMA row m = head), B = candidate keys
        uint4 qa[4];
        {
            const bf16_t *qr = qb + (int64_t)(kvh * G + g0 + (n < ng ? n : 0)) * st.q_h + (int64_t)(ref - t0) * st.q_t;
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                qa[sl] = make_uint4(0, 0, 0, 0);
                if (n < ng) qa[sl] = *reinterpret_cast<const uint4 *>(qr + 32 * sl + 8 * c);
            }
        }
        for (int j0 = wave * 16; j0 < wl; j0 += 16 * kEliteWaves) {
            const int j = j0 + n;
            uint4 kb[4];
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                kb[sl] = make_uint4(0, 0, 0, 0);
                if (j < wl) kb[sl] = *reinterpret_cast<const uint4 *>(k + (int64_t)(sq.win_start + j) * st.kv_t + 32 * sl + 8 * c);
            }
            f32x4 s4 = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
                s4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qa[sl]), __builtin_bit_cast(bf16x8, kb[sl]), s4, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (4 * c + i < ng && j < wl) s_logit[(size_t)(4 * c + i) * W + j] = s4[i];
        }
        __syncthreads();
        // ---- phase 2
        for (int hh = wave; hh < ng; hh += kEliteWaves) {
            const int h = kvh * G + g0 + hh;
            const int64_t hrow = ((int64_t)l * dm.B + b) * dm.Hq + h;
            const float *logit = s_logit + (size_t)hh * W;
            int *elite = s_elite + (size_t)hh * W;
            const bf16_t *q = qb + (int64_t)h * st.q_h;
            const bf16_t *qref = q + (int64_t)(ref - t0) * st.q_t;
            float m32 = -INFINITY;
            for (int j = lane; j < wl; j += 64) m32 = fmaxf(m32, logit[j]);
            m32 = wave_max(m32);
            // exact maximum: every candidate within the margin of the fp32 maximum is recomputed
            double amax = -INFINITY;
            for (int j0 = 0; j0 < wl; j0 += 64) {
                const int j = j0 + lane;
                unsigned long long near = __ballot(j < wl && logit[j] >= m32 - kEliteMargin);
                while (near) {
                    const int src = __ffsll(near) - 1;
                    near &= near - 1;
                    amax = fmax(amax, dot64_wave(qref, k + (int64_t)(sq.win_start + j0 + src) * st.kv_t, lane));
                }
            }
            int R = 0;
            for (int j0 = 0; j0 < wl; j0 += 64) {
                const int j = j0 + lane;
                // x > 0 <=> exp((a_j - a_max) / sqrt(d)) > alpha
                const double x = j < wl ? ((double)logit[j] - amax) * inv_sqrt_d - ln_alpha : -1.0;
                bool flag = j < wl && x > 0.0;
                unsigned long long unsure = __ballot(j < wl && fabs(x) <= (double)(kEliteMargin * scale));
                while (unsure) {
                    const int src = __ffsll(unsure) - 1;
                    unsure &= unsure - 1;
                    const double a = dot64_wave(qref, k + (int64_t)(sq.win_start + j0 + src) * st.kv_t, lane);
                    const bool f = exp((a - amax) * inv_sqrt_d) >= alpha;
                    if (lane == src) flag = f;
                }
                const unsigned long long bal = __ballot(flag);
                if (flag) {
                    const int pos = R + __popcll(bal & ((1ull << lane) - 1ull));
                    elite[pos] = sq.win_start + j;
                    t.elite_idx[hrow * W + pos] = sq.win_start + j;
                }
                R += __popcll(bal);
            }
            if (lane == 0) t.elite_cnt[hrow] = R;
            // elite-text columns of Eq.7: (max, sum-exp) of every elite row over the elite text keys.  The
            // R x R logits are formed on MFMA, 16 rows against 16 keys per tile; lane (n, c) of a tile holds
            // key n and rows 4c .. 4c+3, rows and keys past R re-read the last one.  Windows of more than 16
            // rows (alpha = 0 turns the whole span into rows) go over the keys twice (maximum, then sum);
            // up to 16 rows the one tile is kept.  The maximum is kept as the RAW dot product (before the
            // 1/sqrt(d) scale), the sum is of exp((a - max) / sqrt(d)).
            for (int rb = 0; rb < R; rb += 16) {
                uint4 qa2[4];
                {
                    const bf16_t *qr = q + (int64_t)(elite[min(rb + n, R - 1)] - t0) * st.q_t;
#pragma unroll
                    for (int sl = 0; sl < 4; ++sl) qa2[sl] = *reinterpret_cast<const uint4 *>(qr + 32 * sl + 8 * c);
                }
                float m4[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY}, z4[4] = {0.f, 0.f, 0.f, 0.f};
                f32x4 a4 = (f32x4){0.f, 0.f, 0.f, 0.f};
                for (int pass = 0; pass < 2; ++pass) {
                    for (int jb = 0; jb < R; jb += 16) {
                        if (pass == 0 || R > 16) {
                            const bf16_t *kr = k + (int64_t)elite[min(jb + n, R - 1)] * st.kv_t;
                            a4 = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int sl = 0; sl < 4; ++sl) {
                                const uint4 kb2 = *reinterpret_cast<const uint4 *>(kr + 32 * sl + 8 * c);
                                a4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qa2[sl]),
                                                                             __builtin_bit_cast(bf16x8, kb2), a4, 0, 0, 0);
                            }
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            // key jb + n of the elite list against row rb + 4c + i; the list is in position order, so
                            // with the causal option a row sees the keys up to its own place in it
                            const bool live = jb + n < R && (!dm.causal_text || jb + n <= rb + 4 * c + i);
                            if (pass == 0) m4[i] = fmaxf(m4[i], live ? a4[i] : -INFINITY);
                            else z4[i] += live ? expf((a4[i] - m4[i]) * scale) : 0.f;
                        }
                    }
                    if (pass == 0) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) m4[i] = max16(m4[i]);
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float z = sum16(z4[i]);
                    const int r = rb + 4 * c + i;
                    if (n == 0 && r < R) {
                        t.row_mtext[hrow * W + r] = m4[i];
                        t.row_ztext[hrow * W + r] = z;
                    }
                }
            }
        }
        __syncthreads();
    }
}

hipError_t launch_elite_mfma(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, const LaunchLayers &ll,
                             const air_strides &st, const SeqArgs &seqs, double alpha) {
    const size_t per_head = (size_t)dm.max_window * (sizeof(float) + sizeof(int));
    int gb = (int)(49152 / per_head);  // heads whose logits share the LDS
    gb = gb < 1 ? 1 : (gb > dm.G ? dm.G : gb);
    hipLaunchKernelGGL(elite_mfma_kernel, dim3(dm.Hkv, dm.B, nl), dim3(64 * kEliteWaves), gb * per_head, s, dm, t, l0, ll, st, seqs,
                       alpha, alpha > 0.0 ? log(alpha) : -INFINITY, gb);
    return hipGetLastError();
}

hipError_t launch_score_mfma(hipStream_t s, const Dims &dm, const DevTables &t, int pass, int l0, int nl,
                             const LaunchLayers &ll, const air_strides &st, const SeqArgs &seqs, int inline_rows, int many_rows) {
    if (pass == 1) {
        const dim3 grid((dm.n_chunks + kStreamChunks - 1) / kStreamChunks, dm.Hkv, nl * dm.B);
        if (dm.vis_window) {
            if (many_rows) hipLaunchKernelGGL((score_stream_kernel<true, true>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
            else hipLaunchKernelGGL((score_stream_kernel<true, false>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
        } else {
            if (many_rows) hipLaunchKernelGGL((score_stream_kernel<false, true>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
            else hipLaunchKernelGGL((score_stream_kernel<false, false>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
        }
    } else {
        const dim3 grid((dm.n_chunks + kFinishChunks - 1) / kFinishChunks, dm.Hkv, nl * dm.B);
        if (inline_rows && !dm.vis_window) {
            hipLaunchKernelGGL((score_finish_kernel<false, true, false>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
            return hipGetLastError();
        }
        // a wave per row when the launch has few units; with many units, 4 waves walk the rows
        hipLaunchKernelGGL(score_rows_mfma_kernel, dim3(dm.Hkv, dm.B, nl),
                           dim3(nl * dm.B * dm.Hkv >= 512 ? 256 : 64 * kRowWaves), 0, s, dm, t, l0, seqs);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (dm.vis_window) {
            if (many_rows) hipLaunchKernelGGL((score_finish_kernel<true, false, true>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
            else hipLaunchKernelGGL((score_finish_kernel<true, false, false>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
        } else {
            if (many_rows) hipLaunchKernelGGL((score_finish_kernel<false, false, true>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
            else hipLaunchKernelGGL((score_finish_kernel<false, false, false>), grid, dim3(256), 0, s, dm, t, l0, ll, st, seqs);
        }
    }
    return hipGetLastError();
}

}  // namespace air
