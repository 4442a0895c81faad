// Internal declarations shared by the translation units of libaircache.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "aircache.h"

namespace air {

constexpr int kChunkKeys = 256;       // visual keys per workgroup in the score passes
constexpr int kMaxLayersPerLaunch = 32;
constexpr int kMaxSplits = 16;        // largest split-K factor of the decode attention
constexpr int kCacheRowAlign = 32;    // layer regions of the compacted cache start on multiples of this
constexpr int kGatherRows = 32;       // rows copied per workgroup in the compaction gather
constexpr int kFinishChunks = 4;      // chunks finished (and summed into one moment entry) per workgroup of air_score's last kernel
constexpr int kStashRows = 32;        // window rows per unit up to which air_score stashes exponentials (one pass over K_v)

struct LayerPtrs {
    const void *q, *k, *v;
};

// Kernel-argument block: the per-layer tensor pointers of one launch and the per-layer
// count of tokens appended so far (decode only).
struct LaunchLayers {
    LayerPtrs p[kMaxLayersPerLaunch];
    int32_t appended[kMaxLayersPerLaunch];
};

// K and V tensor of one layer (the compacted cache itself when it is kept in place)
struct CachePtrs {
    void *k, *v;
};

struct SeqArgs {
    air_seq s[AIR_MAX_BATCH];
};

// Byte offsets of every table inside the workspace.
struct WsLayout {
    size_t seq_tab, elite_cnt, elite_idx, row_mtext, row_ztext, row_M, row_w, part, scores;
    size_t unit_st, unit_sk, s_t, s_k, budgets, base_len, layer_off, dec_cnt, unit_cnt, seq_cnt, moments, indices;
    size_t kcache, vcache, dec_o, dec_ml, stash, row_f, unit_R, len_off, dec_steps, cache_ptrs, by_length;
    size_t total;
    int32_t n_chunks;     // ceil(max_vis_len / kChunkKeys)
    int64_t pool_rows;    // rows of one (sequence, KV head) cache pool
};

// Shapes every kernel needs, passed by value.
struct Dims {
    int32_t L, Hq, Hkv, G, D, B;
    int32_t max_vis, max_window, n_chunks, max_steps;
    int32_t n_entries;   // moment entries per unit: one per workgroup of air_score's last kernel, ceil(n_chunks / kFinishChunks)
    int32_t vis_window;  // 1: the window rows are visual tokens (causal over the visual keys, no text columns)
    int32_t causal_text; // 1: an elite row sees only the elite text keys at or before its own position (Eq.7 with a causal mask)
    uint32_t inv_B;      // floor(2^32 / B) + 1 (unused for B = 1): division of a 16-bit index by B as one multiply
    int64_t pool_rows;
    // Eq.11 inside air_score: the last workgroup of a sequence to finish its unit does the allocation (the layers fit one wave)
    int32_t fuse_budget, budget_mode, min_keep;
    double retention;
};

struct DevTables {
    air_seq *seq_tab;
    int32_t *elite_cnt, *elite_idx;
    float *row_mtext, *row_ztext, *row_M, *row_w;
    float2 *part;
    float *scores;
    double *unit_st, *unit_sk, *s_t, *s_k, *moments;
    int32_t *budgets, *base_len, *layer_off, *dec_cnt, *indices;
    void *kcache, *vcache;
    float *dec_o, *stash, *row_f;
    int2 *len_off;    // (base_len, layer_off) of a (sequence, layer) side by side: one read for the decode kernel
    int4 *by_length;  // per sequence, the layers in order of falling cache length: (base_len, layer_off, layer, 0)
    int32_t *unit_cnt;  // per unit: workgroups of air_score's last kernel that have left their moment entry (zero between launches)
    int32_t *seq_cnt;   // per sequence: units whose statistics are complete (zero again once all L * H_kv have arrived)
    int32_t *unit_R;  // window rows of a unit (all heads of the group), left by the row-parameter kernel
    float2 *dec_ml;
    int32_t *dec_steps;  // tokens appended so far per unit when the device counts them (else null); one overflow flag after the last unit
    CachePtrs *cache_ptrs;  // in-place cache: K / V tensor of every layer, written by the compaction gather (else null)
    int64_t ip_kv_b, ip_kv_h;  // in-place cache: element strides between sequences and between KV heads of those tensors
};

// Where the workgroups of a decode launch exchange their split-K partials: per unit `stride` slots of
// (16 x head_dim partial outputs, (max, sum) per head) and one arrival counter.  The workspace's area is
// indexed by the context-wide unit (calls on different layers may overlap), the static one by the unit
// inside the launch.
struct DecodeExchange {
    float *o;
    float2 *ml;
    int32_t *cnt;
    int32_t local;   // 1: slots indexed by the unit inside the launch
    int32_t stride;  // slots per unit
};
constexpr size_t kStaticSlots = 1024;  // (unit, split) pairs per launch that the static exchange area holds

WsLayout make_layout(const air_config &cfg);

// ---- kernel launchers (each returns the hipError_t of its launch) ----
hipError_t launch_elite(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                        const LaunchLayers &ll, const air_strides &st, const SeqArgs &seqs, double alpha);
hipError_t launch_window_rows(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, const SeqArgs &seqs);
hipError_t launch_score_pass1(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                              const LaunchLayers &ll, const air_strides &st);
hipError_t launch_score_rows(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl);
hipError_t launch_score_pass2(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                              const LaunchLayers &ll, const air_strides &st);
hipError_t launch_stats(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl);
hipError_t launch_elite_mfma(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, const LaunchLayers &ll,
                             const air_strides &st, const SeqArgs &seqs, double alpha);
hipError_t launch_score_mfma(hipStream_t s, const Dims &dm, const DevTables &t, int pass, int l0, int nl,
                             const LaunchLayers &ll, const air_strides &st, const SeqArgs &seqs, int inline_rows, int many_rows);
hipError_t launch_budget(hipStream_t s, const Dims &dm, const DevTables &t, double retention, int mode,
                         int min_keep, int skip_allocation, const SeqArgs &seqs);
hipError_t launch_select(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, int threads, int direct_max);
hipError_t launch_gather(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl,
                         const LaunchLayers &ll, const air_strides &st, int wgs_per_unit);
hipError_t launch_gather_in_place(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, const LaunchLayers &ll,
                                  const air_strides &st);
hipError_t launch_decode(hipStream_t s, const Dims &dm, const DevTables &t, const DecodeExchange &x, int dtype, int l0,
                         int nl, int lbase, const LaunchLayers &ll, const void *q_new, const void *k_new,
                         const void *v_new, void *out, int splits, int waves, int tiles, int uniform_appended,
                         bool longest_first, bool column_halves);
// the exchange area inside the library's static device array, for the device that is current (looked up once per device)
hipError_t static_exchange(DecodeExchange *x);
hipError_t launch_zero_counters(hipStream_t s, int32_t *p, int n);

// The bf16 / head_dim 128 cache is laid out so that the decode kernel can feed it to MFMA straight
// from global memory, every load instruction of a wave reading 1 KB of consecutive memory, and so
// that one token touches few cache lines (appending a token costs by the line it writes).
//
// K' in tiles of 16 tokens, [4 slices][16 tokens][32 elements]: lane (token n, part c) of a wave finds
// the 16 bytes it feeds to MFMA for slice sl at byte 1024 sl + 64 n + 16 c of the tile.  A token's
// row is four runs of 64 bytes.
//
// V' transposed in blocks of 32 tokens, [8 column tiles][4 slot groups][16 columns][8 slots]: token t
// of the block sits in slot v_slot(t).  With this order the 8 probabilities a lane holds after the
// two 16-key score tiles of a block are exactly the 8 contraction slots it must supply, and lane
// (column n of tile j, group c) finds its 16 bytes at byte 1024 j + 256 c + 16 n of the block.
// A token touches 2 bytes in every 16 of one 256-byte run per column tile.
inline bool v_transposed(int dtype, int head_dim) { return dtype == AIR_BF16 && head_dim == 128; }
__host__ __device__ inline int v_slot(int t) { return ((t & 15) >> 2) * 8 + (t >> 4) * 4 + (t & 3); }
// element offsets from the unit's base of element e of K' row r / column col of V' row r
__host__ __device__ inline int64_t k_tiled(int64_t r, int e) {
    return (r >> 4) * 2048 + (e >> 5) * 512 + (r & 15) * 32 + (e & 31);
}
__host__ __device__ inline int64_t v_tiled(int64_t r, int col) {
    const int slot = v_slot((int)(r & 31));
    return (r >> 5) * 4096 + (col >> 4) * 512 + (slot >> 3) * 128 + (col & 15) * 8 + (slot & 7);
}

}  // namespace air
