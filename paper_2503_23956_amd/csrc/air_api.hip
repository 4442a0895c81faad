// C ABI of libaircache.so: context, workspace layout, argument validation, stage sequencing.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <initializer_list>
#include <string>
#include <vector>

#include "air_internal.h"

namespace air {

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static bool config_ok(const air_config &c) {
    if (c.n_layers < 1 || c.n_layers > AIR_MAX_LAYERS) return false;
    if (c.batch < 1 || c.batch > AIR_MAX_BATCH) return false;
    if (c.n_kv_heads < 1 || c.n_q_heads < c.n_kv_heads || c.n_q_heads % c.n_kv_heads) return false;
    if (c.n_q_heads / c.n_kv_heads > 16) return false;
    if ((int64_t)c.batch * c.n_kv_heads > 65535) return false;  // one layer's units must fit a grid dimension
    if (c.head_dim != 64 && c.head_dim != 128) return false;
    if (c.max_vis_len < 1 || c.max_nonvis_len < 1) return false;
    if (c.window_kind != AIR_WINDOW_TEXT && c.window_kind != AIR_WINDOW_VISUAL) return false;
    if (c.device_steps != 0 && c.device_steps != 1) return false;
    if (c.device_steps && !(c.dtype == AIR_BF16 && c.head_dim == 128)) return false;
    if (c.cache_in_place != 0 && c.cache_in_place != 1) return false;
    if (c.causal_text != 0 && c.causal_text != 1) return false;
    if (c.causal_text && c.window_kind == AIR_WINDOW_VISUAL) return false;  // a visual window has no text columns
    if (c.cache_in_place && !(c.dtype == AIR_BF16 && c.head_dim == 128)) return false;
    const bool vis_window = c.window_kind == AIR_WINDOW_VISUAL;
    if (c.max_window < 1 || c.max_window > AIR_MAX_TEXT) return false;
    if (c.max_window > (vis_window ? c.max_vis_len : c.max_nonvis_len)) return false;
    if (vis_window && c.alpha != 0.0) return false;  // every token of a visual window is a row: no Eq.5
    if (c.max_decode_steps < 0) return false;
    if (c.dtype != AIR_F32 && c.dtype != AIR_BF16) return false;
    if (c.budget_mode < AIR_BUDGET_STRENGTH_SKEW || c.budget_mode > AIR_BUDGET_SKEW) return false;
    if (c.min_keep < 0) return false;
    if (!(c.alpha >= 0.0 && c.alpha <= 1.0)) return false;
    if (!(c.retention > 0.0 && c.retention <= 1.0)) return false;
    return true;
}

static int64_t total_budget(const air_config &c, int n_vis) {
    int64_t k = (int64_t)floor(c.retention * (double)n_vis * (double)c.n_layers + 0.5);
    const int64_t lo = (int64_t)c.n_layers * (c.min_keep < n_vis ? c.min_keep : n_vis);
    const int64_t hi = (int64_t)c.n_layers * n_vis;
    return k < lo ? lo : (k > hi ? hi : k);
}

WsLayout make_layout(const air_config &c) {
    WsLayout w;
    memset(&w, 0, sizeof(w));
    const size_t L = c.n_layers, B = c.batch, Hq = c.n_q_heads, Hkv = c.n_kv_heads, D = c.head_dim;
    const size_t W = c.max_window, NV = c.max_vis_len;
    const size_t esz = c.dtype == AIR_BF16 ? 2 : 4;
    w.n_chunks = (int32_t)((NV + kChunkKeys - 1) / kChunkKeys);
    // rows of one (sequence, KV head) pool: every layer's system + text rows, its decode
    // appends and alignment slack, plus the kept visual rows of all layers together
    w.pool_rows = (int64_t)L * (c.max_nonvis_len + c.max_decode_steps + kCacheRowAlign - 1) +
                  total_budget(c, c.max_vis_len);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    w.seq_tab = take(B * sizeof(air_seq));
    w.elite_cnt = take(L * B * Hq * 4);
    w.elite_idx = take(L * B * Hq * W * 4);
    w.row_mtext = take(L * B * Hq * W * 4);
    w.row_ztext = take(L * B * Hq * W * 4);
    w.row_M = take(L * B * Hq * W * 4);
    w.row_w = take(L * B * Hq * W * 4);
    w.part = take(L * B * Hq * W * (size_t)w.n_chunks * 8);
    w.scores = take(L * B * Hkv * NV * 4);
    w.unit_st = take(L * B * Hkv * 8);
    w.unit_sk = take(L * B * Hkv * 8);
    w.s_t = take(B * L * 8);
    w.s_k = take(B * L * 8);
    w.budgets = take(B * L * 4);
    w.base_len = take(B * L * 4);
    w.layer_off = take(B * L * 4);
    w.dec_cnt = take(L * B * Hkv * 4);
    w.unit_cnt = take(L * B * Hkv * 4);
    w.seq_cnt = take(B * 4);
    w.dec_steps = take((L * B * Hkv + 1) * 4);
    w.moments = take(L * B * Hkv * (size_t)((w.n_chunks + kFinishChunks - 1) / kFinishChunks) * 4 * 8);
    w.indices = take(L * B * Hkv * NV * 4);
    // the cache pool, unless the cache is kept inside the prompt's own tensors
    w.kcache = take(c.cache_in_place ? 0 : B * Hkv * (size_t)w.pool_rows * D * esz);
    w.vcache = take(c.cache_in_place ? 0 : B * Hkv * (size_t)w.pool_rows * D * esz);
    w.cache_ptrs = take(L * sizeof(CachePtrs));
    w.dec_o = take(L * B * Hkv * kMaxSplits * 16 * D * 4);  // per (unit, split): 16 head rows x D
    w.dec_ml = take(L * B * Hq * kMaxSplits * 8);
    w.stash = v_transposed(c.dtype, c.head_dim) ? take(L * B * Hkv * (size_t)w.n_chunks * kStashRows * kChunkKeys * 4) : off;
    w.row_f = v_transposed(c.dtype, c.head_dim) ? take(L * B * Hkv * (size_t)kStashRows * w.n_chunks * 4) : off;
    w.unit_R = take(L * B * Hkv * 4);
    w.len_off = take(B * L * 8);
    w.by_length = take(B * L * 16);
    w.total = off;
    return w;
}

}  // namespace air

using namespace air;

// Eq.11 in the tail of air_score's last kernel: the MFMA score path, the layers within one wave, the KV heads of a layer
// within one round of sixteen loads
static bool can_fuse_budget(const air_config &c) {
    return v_transposed(c.dtype, c.head_dim) && c.n_layers <= 64 && c.n_kv_heads <= 16;
}

struct air_ctx {
    air_config cfg;
    WsLayout lay;
    Dims dm;
    DevTables tab;
    char *ws;
    bool have_seqs;
    bool budgets_ready;
    std::vector<air_seq> seqs;
    std::vector<char> decoded;  // device_steps: air_decode_attn has been called on the layer since its compaction
    std::vector<char> scored, compacted, fixed_idx;  // fixed_idx: the layer's kept indices were set by the caller
    std::vector<int32_t> appended;
    air_tuning tune;  // launch-shape overrides (air_set_tuning); all automatic after air_create
    std::vector<CachePtrs> ip_layers;
    // Eq.11 done in the tail of air_score (Dims::fuse_budget): layers scored that way since the reset; broken: a layer was
    // scored twice or with the fusion switched off, so air_budget launches its kernel; need_zero: the per-sequence
    // arrival counters may hold a partial count and are cleared in front of the next air_score
    int fused_count = 0;
    bool fused_broken = false, need_zero = false;  // in-place cache: the K / V tensor each compacted layer lives in
    std::string err;
};

static air_status fail(air_ctx *ctx, air_status st, const std::string &msg) {
    if (ctx) ctx->err = msg;
    return st;
}
static air_status hip_fail(air_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, AIR_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

extern "C" {

const char *air_version(void) { return "aircache-mi355x 0.1"; }

size_t air_workspace_bytes(const air_config *cfg) {
    if (!cfg || !config_ok(*cfg)) return 0;
    return make_layout(*cfg).total;
}

air_status air_create(const air_config *cfg, void *workspace, size_t workspace_bytes, air_ctx **out) {
    if (!cfg || !out) return AIR_ERR_INVALID_ARG;
    *out = nullptr;
    if (!config_ok(*cfg)) return AIR_ERR_SHAPE;
    WsLayout lay = make_layout(*cfg);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < lay.total) return AIR_ERR_WORKSPACE;
    air_ctx *c = new air_ctx();
    c->cfg = *cfg;
    c->lay = lay;
    c->ws = (char *)workspace;
    Dims &d = c->dm;
    d.L = cfg->n_layers;
    d.Hq = cfg->n_q_heads;
    d.Hkv = cfg->n_kv_heads;
    d.G = d.Hq / d.Hkv;
    d.D = cfg->head_dim;
    d.B = cfg->batch;
    d.max_vis = cfg->max_vis_len;
    d.max_window = cfg->max_window;
    d.n_chunks = lay.n_chunks;
    d.n_entries = (lay.n_chunks + kFinishChunks - 1) / kFinishChunks;
    d.max_steps = cfg->max_decode_steps;
    d.vis_window = cfg->window_kind == AIR_WINDOW_VISUAL ? 1 : 0;
    d.causal_text = cfg->causal_text;
    d.inv_B = cfg->batch > 1 ? (uint32_t)(0x100000000ull / (uint64_t)cfg->batch) + 1u : 0u;
    d.pool_rows = lay.pool_rows;
    d.fuse_budget = can_fuse_budget(*cfg) ? 1 : 0;
    d.budget_mode = cfg->budget_mode;
    d.min_keep = cfg->min_keep;
    d.retention = cfg->retention;
    DevTables &t = c->tab;
    char *w = c->ws;
    t.seq_tab = (air_seq *)(w + lay.seq_tab);
    t.elite_cnt = (int32_t *)(w + lay.elite_cnt);
    t.elite_idx = (int32_t *)(w + lay.elite_idx);
    t.row_mtext = (float *)(w + lay.row_mtext);
    t.row_ztext = (float *)(w + lay.row_ztext);
    t.row_M = (float *)(w + lay.row_M);
    t.row_w = (float *)(w + lay.row_w);
    t.part = (float2 *)(w + lay.part);
    t.scores = (float *)(w + lay.scores);
    t.unit_st = (double *)(w + lay.unit_st);
    t.unit_sk = (double *)(w + lay.unit_sk);
    t.s_t = (double *)(w + lay.s_t);
    t.s_k = (double *)(w + lay.s_k);
    t.budgets = (int32_t *)(w + lay.budgets);
    t.base_len = (int32_t *)(w + lay.base_len);
    t.layer_off = (int32_t *)(w + lay.layer_off);
    t.dec_cnt = (int32_t *)(w + lay.dec_cnt);
    t.unit_cnt = (int32_t *)(w + lay.unit_cnt);
    t.seq_cnt = (int32_t *)(w + lay.seq_cnt);
    t.moments = (double *)(w + lay.moments);
    t.indices = (int32_t *)(w + lay.indices);
    t.kcache = (void *)(w + lay.kcache);
    t.vcache = (void *)(w + lay.vcache);
    t.dec_o = (float *)(w + lay.dec_o);
    t.dec_ml = (float2 *)(w + lay.dec_ml);
    t.stash = (float *)(w + lay.stash);
    t.row_f = (float *)(w + lay.row_f);
    t.unit_R = (int32_t *)(w + lay.unit_R);
    t.len_off = (int2 *)(w + lay.len_off);
    t.by_length = (int4 *)(w + lay.by_length);
    t.dec_steps = cfg->device_steps ? (int32_t *)(w + lay.dec_steps) : nullptr;
    t.cache_ptrs = cfg->cache_in_place ? (CachePtrs *)(w + lay.cache_ptrs) : nullptr;
    t.ip_kv_b = t.ip_kv_h = 0;
    c->ip_layers.assign(d.L, CachePtrs{nullptr, nullptr});
    c->have_seqs = false;
    c->budgets_ready = false;
    memset(&c->tune, 0, sizeof(c->tune));
    c->tune.select_direct_max = -1;
    c->scored.assign(d.L, 0);
    c->compacted.assign(d.L, 0);
    c->fixed_idx.assign(d.L, 0);
    c->appended.assign(d.L, 0);
    c->decoded.assign(d.L, 0);
    // scores past a sequence's visual span and the small tables start at zero
    hipError_t e = static_exchange(nullptr);  // address of the static exchange area on this device, looked up once
    if (e == hipSuccess) e = hipMemset(w + lay.scores, 0, lay.unit_st - lay.scores);
    if (e == hipSuccess) e = hipMemset(w + lay.seq_tab, 0, lay.part - lay.seq_tab);
    if (e == hipSuccess) e = hipMemset(w + lay.unit_st, 0, lay.indices - lay.unit_st);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        delete c;
        return AIR_ERR_HIP;
    }
    *out = c;
    return AIR_OK;
}

air_status air_destroy(air_ctx *ctx) {
    if (!ctx) return AIR_ERR_INVALID_ARG;
    delete ctx;
    return AIR_OK;
}

air_status air_reset(air_ctx *ctx) {
    if (!ctx) return AIR_ERR_INVALID_ARG;
    ctx->have_seqs = false;
    ctx->budgets_ready = false;
    ctx->seqs.clear();
    ctx->scored.assign(ctx->dm.L, 0);
    ctx->compacted.assign(ctx->dm.L, 0);
    ctx->fixed_idx.assign(ctx->dm.L, 0);
    ctx->appended.assign(ctx->dm.L, 0);
    ctx->decoded.assign(ctx->dm.L, 0);
    if (ctx->fused_count > 0 && (ctx->fused_broken || ctx->fused_count != ctx->dm.L)) ctx->need_zero = true;
    ctx->fused_count = 0;
    ctx->fused_broken = false;
    return AIR_OK;
}

const char *air_last_error(const air_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

// layers per launch of the kernels that take per-layer tensor pointers: the units of a launch are one grid dimension (<= 65535)
static int layers_per_launch(const air_ctx *c) {
    const int64_t fit = 65535 / ((int64_t)c->dm.B * c->dm.Hkv);
    return (int)(fit < kMaxLayersPerLaunch ? fit : kMaxLayersPerLaunch);
}

static bool range_ok(const air_ctx *c, int32_t l0, int32_t l1) { return l0 >= 0 && l1 > l0 && l1 <= c->cfg.n_layers; }

static air_status check_strides(air_ctx *ctx, const air_strides *st, const air_layer *layers, int nl, bool need_q) {
    const int64_t vec = ctx->cfg.dtype == AIR_BF16 ? 8 : 4;  // elements per 16 bytes
    const int64_t D = ctx->cfg.head_dim;
    if (st->kv_t < D || st->kv_t % vec || st->kv_b % vec || st->kv_h % vec || st->kv_b < 0 || st->kv_h < 0)
        return fail(ctx, AIR_ERR_SHAPE, "k/v strides must be non-negative multiples of 16 bytes with token stride >= head_dim");
    if (need_q && (st->q_t < D || st->q_t % vec || st->q_b % vec || st->q_h % vec || st->q_b < 0 || st->q_h < 0))
        return fail(ctx, AIR_ERR_SHAPE, "q strides must be non-negative multiples of 16 bytes with token stride >= head_dim");
    for (int i = 0; i < nl; ++i) {
        if (!layers[i].k || !layers[i].v || (need_q && !layers[i].q_text))
            return fail(ctx, AIR_ERR_INVALID_ARG, "null tensor pointer in layers[]");
        if (((uintptr_t)layers[i].k & 15) || ((uintptr_t)layers[i].v & 15) || (need_q && ((uintptr_t)layers[i].q_text & 15)))
            return fail(ctx, AIR_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    }
    return AIR_OK;
}

static air_status check_seqs(air_ctx *ctx, const air_seq *seqs) {
    const air_config &c = ctx->cfg;
    for (int b = 0; b < c.batch; ++b) {
        const air_seq &s = seqs[b];
        const int text0 = s.vis_start + s.vis_len;
        if (s.vis_start < 0 || s.vis_len < 1 || s.vis_len > c.max_vis_len || s.seq_len <= text0)
            return fail(ctx, AIR_ERR_SHAPE, "air_seq: need vis_len in [1, max_vis_len] and at least one text token");
        if (s.seq_len - s.vis_len > c.max_nonvis_len)
            return fail(ctx, AIR_ERR_SHAPE, "air_seq: system + text tokens exceed max_nonvis_len");
        if (c.window_kind == AIR_WINDOW_VISUAL) {
            if (s.win_len < 1 || s.win_len > c.max_window || s.win_start < s.vis_start || s.win_start + s.win_len > text0)
                return fail(ctx, AIR_ERR_SHAPE, "air_seq: a visual window must lie inside the visual span and fit max_window");
        } else if (s.win_len < 1 || s.win_len > c.max_window || s.win_start < text0 || s.win_start + s.win_len > s.seq_len)
            return fail(ctx, AIR_ERR_SHAPE, "air_seq: candidate span must lie inside the text span and fit max_window");
    }
    return AIR_OK;
}

air_status air_score(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const air_layer *layers,
                     const air_strides *strides, const air_seq *seqs) {
    if (!ctx) return AIR_ERR_INVALID_ARG;
    if (!layers || !strides || !seqs) return fail(ctx, AIR_ERR_INVALID_ARG, "air_score: null argument");
    if (!range_ok(ctx, l0, l1)) return fail(ctx, AIR_ERR_INVALID_ARG, "air_score: bad layer range");
    air_status st = check_strides(ctx, strides, layers, l1 - l0, true);
    if (st != AIR_OK) return st;
    st = check_seqs(ctx, seqs);
    if (st != AIR_OK) return st;
    if (ctx->have_seqs && memcmp(ctx->seqs.data(), seqs, sizeof(air_seq) * ctx->cfg.batch) != 0)
        return fail(ctx, AIR_ERR_STATE, "air_score: seqs differ from the ones this context was first scored with");
    for (int l = l0; l < l1; ++l)
        if (ctx->compacted[l]) return fail(ctx, AIR_ERR_STATE, "air_score: layer already compacted");
    hipStream_t s = (hipStream_t)stream;
    SeqArgs sa;
    memset(&sa, 0, sizeof(sa));
    memcpy(sa.s, seqs, sizeof(air_seq) * ctx->cfg.batch);
    const int dt = ctx->cfg.dtype;
    const bool mfma = v_transposed(dt, ctx->cfg.head_dim);  // bf16, head_dim 128
    if (ctx->need_zero) {  // a prompt that was dropped half-way left partial counts of finished units
        hipError_t e = launch_zero_counters(s, ctx->tab.seq_cnt, ctx->dm.B);
        if (e != hipSuccess) return hip_fail(ctx, e, "air_score: clearing the arrival counters");
        ctx->need_zero = false;
    }
    const int lpl = layers_per_launch(ctx);
    int group = lpl;
    // The elite window (alpha > 0) leaves a unit a handful of rows: the finish kernel forms their
    // parameters itself.  A window that turns its whole span into rows gets the row-parameter kernel.
    const int inline_rows = ctx->cfg.alpha > 0.0 && !ctx->dm.vis_window && ctx->tune.score_rows_kernel != 1;
    // Windows that are known to exceed the stash (alpha = 0 turns the whole candidate span into rows)
    // read K_v twice: run the two kernels over groups of layers whose keys fit the memory-side cache.
    const int many_rows = mfma && ctx->cfg.alpha == 0.0 && (int64_t)ctx->dm.G * ctx->cfg.max_window > kStashRows;
    if (many_rows) {
        double layer_bytes = 0.0;
        for (int b = 0; b < ctx->cfg.batch; ++b) layer_bytes += (double)seqs[b].vis_len * ctx->cfg.n_kv_heads * 128 * 2;
        const double block = (double)(ctx->tune.score_block_mb > 0 ? ctx->tune.score_block_mb : 160) * 1048576.0;
        const int n_groups = (int)ceil(layer_bytes * (l1 - l0) / block);
        group = (l1 - l0 + (n_groups > 0 ? n_groups : 1) - 1) / (n_groups > 0 ? n_groups : 1);
        if (group < 1) group = 1;
        if (group > lpl) group = lpl;
    }
    for (int c0 = l0; c0 < l1; c0 += lpl) {
        const int nl = (l1 - c0 < lpl) ? l1 - c0 : lpl;
        LaunchLayers ll;
        memset(&ll, 0, sizeof(ll));
        for (int i = 0; i < nl; ++i) {
            ll.p[i].q = layers[c0 - l0 + i].q_text;
            ll.p[i].k = layers[c0 - l0 + i].k;
            ll.p[i].v = layers[c0 - l0 + i].v;
        }
        hipError_t e = ctx->dm.vis_window ? launch_window_rows(s, ctx->dm, ctx->tab, c0, nl, sa)
                       : mfma             ? launch_elite_mfma(s, ctx->dm, ctx->tab, c0, nl, ll, *strides, sa, ctx->cfg.alpha)
                                          : launch_elite(s, ctx->dm, ctx->tab, dt, c0, nl, ll, *strides, sa, ctx->cfg.alpha);
        if (e == hipSuccess && !mfma) {
            e = launch_score_pass1(s, ctx->dm, ctx->tab, dt, c0, nl, ll, *strides);
            if (e == hipSuccess) e = launch_score_rows(s, ctx->dm, ctx->tab, c0, nl);
            if (e == hipSuccess) e = launch_score_pass2(s, ctx->dm, ctx->tab, dt, c0, nl, ll, *strides);
            if (e == hipSuccess) e = launch_stats(s, ctx->dm, ctx->tab, c0, nl);
        }
        // MFMA path: stream kernel, then finish kernel, per group of layers (one group unless the
        // window is known to need the second read of K_v)
        for (int g0 = 0; mfma && e == hipSuccess && g0 < nl; g0 += group) {
            const int gn = (nl - g0 < group) ? nl - g0 : group;
            LaunchLayers lg;
            memset(&lg, 0, sizeof(lg));
            for (int i = 0; i < gn; ++i) lg.p[i] = ll.p[g0 + i];
            e = launch_score_mfma(s, ctx->dm, ctx->tab, 1, c0 + g0, gn, lg, *strides, sa, inline_rows, many_rows);
            if (e == hipSuccess) e = launch_score_mfma(s, ctx->dm, ctx->tab, 2, c0 + g0, gn, lg, *strides, sa, inline_rows, many_rows);
        }
        if (e != hipSuccess) return hip_fail(ctx, e, "air_score launch");
    }
    if (!ctx->have_seqs) {
        ctx->seqs.assign(seqs, seqs + ctx->cfg.batch);
        ctx->have_seqs = true;
    }
    for (int l = l0; l < l1; ++l) {
        if (ctx->scored[l] || !ctx->dm.fuse_budget) ctx->fused_broken = true;
        ctx->scored[l] = 1;
    }
    if (ctx->dm.fuse_budget) ctx->fused_count += l1 - l0;
    ctx->budgets_ready = false;
    return AIR_OK;
}

air_status air_budget(air_ctx *ctx, void *stream) {
    if (!ctx) return AIR_ERR_INVALID_ARG;
    for (int l = 0; l < ctx->cfg.n_layers; ++l)
        if (!ctx->scored[l]) return fail(ctx, AIR_ERR_STATE, "air_budget: not every layer has been scored");
    for (int l = 0; l < ctx->cfg.n_layers; ++l)
        if (ctx->compacted[l]) return fail(ctx, AIR_ERR_STATE, "air_budget: layers already compacted");
    // Where every layer went through air_score's last kernel once, with the allocation of Eq.11 in its tail, the
    // budgets and the layout tables are already on their way: nothing is launched here.
    const bool done_in_score = ctx->dm.fuse_budget && !ctx->fused_broken && ctx->fused_count == ctx->dm.L;
    if (!done_in_score) {
        SeqArgs sa;
        memset(&sa, 0, sizeof(sa));
        memcpy(sa.s, ctx->seqs.data(), sizeof(air_seq) * ctx->cfg.batch);
        hipError_t e = launch_budget((hipStream_t)stream, ctx->dm, ctx->tab, ctx->cfg.retention, ctx->cfg.budget_mode,
                                     ctx->cfg.min_keep, 0, sa);
        if (e != hipSuccess) return hip_fail(ctx, e, "air_budget launch");
    }
    ctx->fixed_idx.assign(ctx->dm.L, 0);
    ctx->budgets_ready = true;
    return AIR_OK;
}

air_status air_select_compact(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const air_layer *layers,
                              const air_strides *strides) {
    if (!ctx) return AIR_ERR_INVALID_ARG;
    if (!layers || !strides) return fail(ctx, AIR_ERR_INVALID_ARG, "air_select_compact: null argument");
    if (!range_ok(ctx, l0, l1)) return fail(ctx, AIR_ERR_INVALID_ARG, "air_select_compact: bad layer range");
    if (!ctx->budgets_ready) return fail(ctx, AIR_ERR_STATE, "air_select_compact: budgets not computed");
    for (int l = l0; l < l1; ++l) {
        if (ctx->appended[l] || ctx->decoded[l]) return fail(ctx, AIR_ERR_STATE, "air_select_compact: layer already decoded on");
        // budgets set by the caller do not need every layer scored, selecting a layer does
        if (!ctx->scored[l] && !ctx->fixed_idx[l])
            return fail(ctx, AIR_ERR_STATE, "air_select_compact: layer neither scored nor given fixed indices");
    }
    air_status st = check_strides(ctx, strides, layers, l1 - l0, false);
    if (st != AIR_OK) return st;
    const bool in_place = ctx->cfg.cache_in_place != 0;
    if (in_place) {
        // Every (sequence, KV head) must be a contiguous run of rows with room for the prompt and every token
        // decode may append, rounded up to whole 32-token blocks.  The budgets are on the device (no wait for
        // them here), so the room is checked for the largest budget there can be, the whole visual span.
        const int64_t D = ctx->cfg.head_dim;
        if (strides->kv_t != D || strides->kv_h % D)
            return fail(ctx, AIR_ERR_SHAPE, "air_select_compact (in place): token stride must equal head_dim and the head stride be whole rows");
        const int64_t rows_per_head = strides->kv_h / D;
        for (int b = 0; b < ctx->cfg.batch; ++b) {
            const int64_t need = ((int64_t)ctx->seqs[b].seq_len + ctx->cfg.max_decode_steps + kCacheRowAlign - 1) / kCacheRowAlign * kCacheRowAlign;
            if (rows_per_head < need)
                return fail(ctx, AIR_ERR_SHAPE, "air_select_compact (in place): a KV head of the prompt's tensors has " +
                                                    std::to_string(rows_per_head) + " rows, prompt + max_decode_steps need " + std::to_string(need));
        }
        if (ctx->cfg.batch > 1 && strides->kv_b < strides->kv_h * (ctx->cfg.n_kv_heads - 1) + rows_per_head * D)
            return fail(ctx, AIR_ERR_SHAPE, "air_select_compact (in place): sequences overlap in the prompt's tensors");
        bool any = false;
        for (int l = 0; l < ctx->cfg.n_layers; ++l) any = any || ctx->compacted[l];
        if (any && (ctx->tab.ip_kv_b != strides->kv_b || ctx->tab.ip_kv_h != strides->kv_h))
            return fail(ctx, AIR_ERR_STATE, "air_select_compact (in place): every layer must use the same strides");
        ctx->tab.ip_kv_b = strides->kv_b;
        ctx->tab.ip_kv_h = strides->kv_h;
    }
    hipStream_t s = (hipStream_t)stream;
    const int lpl = layers_per_launch(ctx);
    for (int c0 = l0; c0 < l1; c0 += lpl) {
        const int nl = (l1 - c0 < lpl) ? l1 - c0 : lpl;
        LaunchLayers ll;
        memset(&ll, 0, sizeof(ll));
        for (int i = 0; i < nl; ++i) {
            ll.p[i].k = layers[c0 - l0 + i].k;
            ll.p[i].v = layers[c0 - l0 + i].v;
            if (in_place) ctx->ip_layers[c0 + i] = CachePtrs{const_cast<void *>(ll.p[i].k), const_cast<void *>(ll.p[i].v)};
        }
        // selection over each run of layers whose indices the caller has not fixed
        hipError_t e = hipSuccess;
        for (int a = 0; a < nl && e == hipSuccess;) {
            if (ctx->fixed_idx[c0 + a]) {
                ++a;
                continue;
            }
            int z = a;
            while (z < nl && !ctx->fixed_idx[c0 + z]) ++z;
            e = launch_select(s, ctx->dm, ctx->tab, c0 + a, z - a, ctx->tune.select_threads, ctx->tune.select_direct_max);
            a = z;
        }
        if (e == hipSuccess)
            e = in_place ? launch_gather_in_place(s, ctx->dm, ctx->tab, c0, nl, ll, *strides)
                         : launch_gather(s, ctx->dm, ctx->tab, ctx->cfg.dtype, c0, nl, ll, *strides, ctx->tune.gather_wgs);
        if (e != hipSuccess) return hip_fail(ctx, e, "air_select_compact launch");
    }
    for (int l = l0; l < l1; ++l) ctx->compacted[l] = 1;
    return AIR_OK;
}

// Shape of one decode launch: `splits` workgroups of `waves` wavefronts per (layer, sequence, KV
// head); a wave works in iterations of 16 * tiles keys.  Measured on this machine: one workgroup streams
// about 100 GB/s (what one CU's vector memory path takes in), the launch as a whole about 6 TB/s, and a
// split costs about 3.7 us (partials written through to memory, an arrival counter, the last
// workgroup reading them back: four dependent trips).  So a unit is split only when the launch is so small
// that its time is one workgroup's streaming time and the split saves more of that than it costs.
// Four waves per workgroup beat eight at every cache length tried (112 units, 215 to 7400 keys: 10.4
// against 10.8 us at 10 % retention, 34.9 against 36.0 at 50 %, 75.3 against 78.2 with the full cache):
// the merge of the waves through LDS is shorter and the streaming is bound by the CU, not by the number of waves.
// air_set_tuning overrides the choice (tests, tuning).
static void decode_shape(const air_ctx *ctx, int n_layers_in_launch, int appended, bool halves_ok, int *splits, int *waves,
                         int *tiles) {
    constexpr int kEnoughWorkgroups = 256, kEnoughWaves = 1536;
    constexpr double kWorkgroupGBs = 100.0, kLaunchGBs = 6000.0, kSplitUs = 3.7;
    const air_config &c = ctx->cfg;
    double avg_len = 0.0;
    for (int b = 0; b < c.batch; ++b) {
        const air_seq &s = ctx->seqs[b];
        avg_len += (double)(s.seq_len - s.vis_len) + c.retention * (double)s.vis_len + appended + 1;
    }
    avg_len /= c.batch;
    const int64_t units = (int64_t)n_layers_in_launch * c.batch * c.n_kv_heads;
    // A launch of a handful of units (one layer of one sequence) is bound by what one CU can stream: the unit
    // is cut into splits of about one 32-key chunk per wave, which beats the exchange of the partials (4 units
    // of ~900 keys: 8.4 us against 9.9 us as single workgroups).
    // Short units of such a launch do better still as two workgroups each with half of V' and no exchange (the column
    // halves: four waves, 64-key chunks): 4 units, us per launch against the splits, 360 keys 5.8 / 7.7, 870 keys
    // 8.1 / 8.4, 1600 keys 11.3 / 9.8, 3800 keys 20.7 / 10.8.
    // (The rule goes by the prompt's own length, so that a decode run keeps one shape from its first step to its last.)
    const bool short_halves = units <= 16 && halves_ok && avg_len - appended < 896.0;
    const bool tiny_launch = units <= 16 && !short_halves;
    int kt = tiny_launch ? 2 : 4;
    if (ctx->tune.decode_tiles > 0) kt = ctx->tune.decode_tiles;
    const int64_t iters = (int64_t)((avg_len + 16.0 * kt - 1.0) / (16.0 * kt));
    // Waves per workgroup: enough for the launch to hold about 1536 waves, and beyond that one wave per 16
    // iterations of the unit, four at most (eight in a tiny launch).  Many short units run fastest with one wave
    // each (no merge, no barrier: 1792 units of ~600 keys 85 us against 97 us with four waves).
    const int w_max = tiny_launch ? 8 : 4;
    int w = 1;
    while (w < w_max && (units * w < kEnoughWaves || iters >= 16 * w)) w *= 2;
    if (ctx->tune.decode_waves > 0) w = ctx->tune.decode_waves;
    if (kt == 8 && w == 8) w = 4;
    int64_t s = 1;
    if (tiny_launch) {
        while (s < kMaxSplits && iters > 4 * s && units * s * 2 <= kEnoughWorkgroups) s *= 2;
    } else if (!short_halves) {
        const double unit_bytes = avg_len * 2.0 * c.head_dim * (c.dtype == AIR_BF16 ? 2.0 : 4.0);
        const double launch_us = (double)units * unit_bytes / (kLaunchGBs * 1e3);
        auto cost = [&](int64_t n) { return fmax(launch_us, unit_bytes / n / (kWorkgroupGBs * 1e3)) + (n > 1 ? kSplitUs : 0.0); };
        for (int64_t n = 2; n <= kMaxSplits && units * n <= kEnoughWorkgroups; n *= 2)
            if (cost(n) < cost(s)) s = n;
    }
    if (ctx->tune.decode_splits > 0) s = ctx->tune.decode_splits;
    *splits = (int)s;
    *waves = w;
    *tiles = kt;
}

// use_static: the split-K partials are exchanged through the library's static device array instead of the workspace
static air_status decode_attn(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const void *q_new, const void *k_new,
                              const void *v_new, void *out, bool use_static) {
    if (!ctx) return AIR_ERR_INVALID_ARG;
    if (!q_new || !k_new || !v_new || !out) return fail(ctx, AIR_ERR_INVALID_ARG, "air_decode_attn: null argument");
    if (((uintptr_t)q_new & 15) || ((uintptr_t)k_new & 15) || ((uintptr_t)v_new & 15) || ((uintptr_t)out & 15))
        return fail(ctx, AIR_ERR_INVALID_ARG, "air_decode_attn: tensors must be 16-byte aligned");
    if (!range_ok(ctx, l0, l1)) return fail(ctx, AIR_ERR_INVALID_ARG, "air_decode_attn: bad layer range");
    for (int l = l0; l < l1; ++l) {
        if (!ctx->compacted[l]) return fail(ctx, AIR_ERR_STATE, "air_decode_attn: layer not compacted");
        // with device-counted steps the kernel guards the capacity itself
        if (!ctx->cfg.device_steps && ctx->appended[l] >= ctx->cfg.max_decode_steps)
            return fail(ctx, AIR_ERR_STATE, "air_decode_attn: max_decode_steps exhausted");
    }
    hipStream_t s = (hipStream_t)stream;
    DecodeExchange xch;
    xch.o = ctx->tab.dec_o;
    xch.ml = ctx->tab.dec_ml;
    xch.cnt = ctx->tab.dec_cnt;
    xch.local = 0;
    xch.stride = kMaxSplits;
    if (use_static) {
        hipError_t e = static_exchange(&xch);
        if (e != hipSuccess) return hip_fail(ctx, e, "air_decode_attn_static: address of the static exchange area");
    }
    // The MFMA kernel takes any number of layers per launch when they have all appended the same number of
    // tokens (the usual case: the layers decode in step), as long as the grid fits; otherwise the per-layer
    // counts travel with the launch, kMaxLayersPerLaunch layers at a time.
    bool in_step = v_transposed(ctx->cfg.dtype, ctx->cfg.head_dim);
    for (int l = l0 + 1; l < l1 && in_step; ++l) in_step = ctx->appended[l] == ctx->appended[l0];
    const int64_t units_per_layer = (int64_t)ctx->dm.B * ctx->dm.Hkv;
    const int max_nl = in_step ? (int)(65535 / units_per_layer) : layers_per_launch(ctx);  // grid.y <= 65535
    // launch shapes first: a static exchange area that is too small must be found before anything is launched
    auto shape_of = [&](int c0, int nl, int *splits, int *waves, int *tiles) {
        // a recorded launch is replayed at every cache length: its shape is chosen for the middle of the decode
        const int hkv = ctx->dm.Hkv;
        const bool halves_ok = in_step && (hkv & (hkv - 1)) == 0 && ctx->tune.decode_halves != 1;
        decode_shape(ctx, nl, ctx->cfg.device_steps ? ctx->cfg.max_decode_steps / 2 : ctx->appended[c0], halves_ok, splits, waves,
                     tiles);
    };
    // Two workgroups per unit, each with all of K' and one half of the columns of V' (air_decode.hip), wherever a
    // launch of four-wave workgroups leaves half the CUs idle (with more workgroups than CUs it loses: 448 units
    // 47.8 against 42.4 us, 1280 units 256 against 250).  112 units, warm / cold cache: 215 keys per
    // unit 6.4 / 8.7 us against 6.5 / 8.4 with one workgroup per unit, 870 keys 9.6 / 11.6 against 10.7 / 13.3,
    // 3800 keys 33 / 45 against 35 / 55, 7400 keys 64 / 73 against 76 / 89.
    auto halves_of = [&](int nl, int splits, int waves, int tiles) {
        const int hkv = ctx->dm.Hkv;
        const bool can = in_step && (hkv & (hkv - 1)) == 0 && splits == 1 && waves == 4 && tiles == 4;
        const bool few = 2 * ((nl * units_per_layer + 7) & ~7) <= 256;
        return can && ctx->tune.decode_halves != 1 && (few || ctx->tune.decode_halves == 2);
    };
    for (int c0 = l0; use_static && c0 < l1; c0 += max_nl) {
        const int nl = (l1 - c0 < max_nl) ? l1 - c0 : max_nl;
        int splits = 1, waves = 1, tiles = 4;
        shape_of(c0, nl, &splits, &waves, &tiles);
        const bool exchanges = splits > 1 || !v_transposed(ctx->cfg.dtype, ctx->cfg.head_dim);  // the generic kernels always go through partials
        if (exchanges && (int64_t)nl * units_per_layer * splits > (int64_t)kStaticSlots)
            return fail(ctx, AIR_ERR_SHAPE, "air_decode_attn_static: the launch needs " +
                                                std::to_string((int64_t)nl * units_per_layer * splits) +
                                                " (unit, split) exchange slots, the static area holds " +
                                                std::to_string(kStaticSlots) + "; pass fewer layers per call");
    }
    for (int c0 = l0; c0 < l1; c0 += max_nl) {
        const int nl = (l1 - c0 < max_nl) ? l1 - c0 : max_nl;
        LaunchLayers ll;
        memset(&ll, 0, sizeof(ll));
        for (int i = 0; i < nl && !in_step; ++i) ll.appended[i] = ctx->appended[c0 + i];
        int splits = 1, waves = 1, tiles = 4;
        shape_of(c0, nl, &splits, &waves, &tiles);
        hipError_t e = hipSuccess;
        if (use_static) {
            xch.stride = splits;
            // the area keeps the last call's contents: the arrival counters of this launch start at zero
            if (splits > 1) e = launch_zero_counters(s, xch.cnt, (int)(nl * units_per_layer));
        }
        // A launch over every layer of many units of differing lengths takes them longest first (a table of the
        // layers by falling cache length per sequence, left by the budget kernel): the workgroups still running at
        // the end are then the short ones.  72B-shaped workload, 1280 units of 1475-2930 keys: 256 -> 248 us per step.
        const bool whole = in_step && c0 == 0 && nl == ctx->cfg.n_layers && splits == 1 && tiles == 4 && (waves == 1 || waves == 4) &&
                           v_transposed(ctx->cfg.dtype, ctx->cfg.head_dim) && !ctx->cfg.cache_in_place;
        const bool longest_first = whole && ctx->tune.decode_order != 1 &&
                                   (ctx->tune.decode_order == 2 || (int64_t)nl * units_per_layer >= 512);
        const bool column_halves = halves_of(nl, splits, waves, tiles);
        // with device-counted steps the two workgroups of a unit meet at the unit's arrival counter
        if (e == hipSuccess && use_static && column_halves && ctx->cfg.device_steps && splits == 1)
            e = launch_zero_counters(s, xch.cnt, (int)(nl * units_per_layer));
        if (e == hipSuccess)
            e = launch_decode(s, ctx->dm, ctx->tab, xch, ctx->cfg.dtype, c0, nl, c0 - l0, ll, q_new, k_new, v_new, out,
                              splits, waves, tiles, in_step ? ctx->appended[l0] : -1, longest_first, column_halves);
        if (e != hipSuccess) return hip_fail(ctx, e, "air_decode_attn launch");
    }
    for (int l = l0; l < l1; ++l) {
        if (ctx->cfg.device_steps) ctx->decoded[l] = 1;
        else ctx->appended[l] += 1;
    }
    return AIR_OK;
}

air_status air_decode_attn(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const void *q_new, const void *k_new,
                           const void *v_new, void *out) {
    return decode_attn(ctx, stream, l0, l1, q_new, k_new, v_new, out, false);
}

air_status air_decode_attn_static(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const void *q_new,
                                  const void *k_new, const void *v_new, void *out) {
    return decode_attn(ctx, stream, l0, l1, q_new, k_new, v_new, out, true);
}

air_status air_set_tuning(air_ctx *ctx, const air_tuning *tn) {
    if (!ctx || !tn) return AIR_ERR_INVALID_ARG;
    auto one_of = [](int v, std::initializer_list<int> ok) {
        for (int x : ok)
            if (v == x) return true;
        return false;
    };
    if (!one_of(tn->decode_splits, {0, 1, 2, 4, 8, 16}) || !one_of(tn->decode_waves, {0, 1, 2, 4, 8}) ||
        !one_of(tn->decode_tiles, {0, 2, 4, 8}) || tn->score_block_mb < 0 || tn->score_block_mb > 65536 ||
        !one_of(tn->score_rows_kernel, {0, 1}) || !one_of(tn->decode_order, {0, 1, 2}) || !one_of(tn->decode_halves, {0, 1, 2}) || !one_of(tn->budget_in_score, {0, 1}) || !one_of(tn->select_threads, {0, 256, 512}) ||
        tn->select_direct_max < -1 || tn->select_direct_max > 1024 || tn->gather_wgs < 0 || tn->gather_wgs > 64)
        return fail(ctx, AIR_ERR_INVALID_ARG, "air_set_tuning: a field holds a value outside its list");
    ctx->tune = *tn;
    // the allocation in the tail of air_score can be switched off (then air_budget launches its kernel); a switch
    // in the middle of a prompt leaves that prompt to the kernel as well
    const int fuse = can_fuse_budget(ctx->cfg) && tn->budget_in_score != 1 ? 1 : 0;
    if (fuse != ctx->dm.fuse_budget) {
        for (int l = 0; l < ctx->dm.L; ++l)
            if (ctx->scored[l]) ctx->fused_broken = true;
        ctx->dm.fuse_budget = fuse;
    }
    return AIR_OK;
}

static air_status d2h(air_ctx *ctx, void *dst, const void *src, size_t bytes);

// tokens appended so far to every layer of sequence b = 0..B-1 (device-counted steps): host [B][L];
// fails when a step ran with the cache full
static air_status device_steps(air_ctx *ctx, std::vector<int32_t> &steps) {
    const int L = ctx->dm.L, B = ctx->dm.B, Hkv = ctx->dm.Hkv;
    std::vector<int32_t> raw((size_t)L * B * Hkv + 1);
    air_status st = d2h(ctx, raw.data(), ctx->tab.dec_steps, raw.size() * 4);
    if (st != AIR_OK) return st;
    bool any_compacted = false;  // until a layer is compacted again the flag is the previous prompt's
    for (int l = 0; l < L; ++l) any_compacted = any_compacted || ctx->compacted[l];
    if (any_compacted && raw.back() != 0)
        return fail(ctx, AIR_ERR_STATE, "a decode step ran with the cache full (max_decode_steps exhausted)");
    steps.assign((size_t)B * L, 0);
    for (int l = 0; l < L; ++l)
        for (int b = 0; b < B; ++b) steps[(size_t)b * L + l] = raw[((size_t)l * B + b) * Hkv];  // the same for every KV head
    return AIR_OK;
}

// ---------------------------------------------------------------------------------------
// inspection
// ---------------------------------------------------------------------------------------
static air_status d2h(air_ctx *ctx, void *dst, const void *src, size_t bytes) {
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(ctx, e, "device to host copy");
    return AIR_OK;
}

air_status air_get_scores(air_ctx *ctx, int32_t l, float *host) {
    if (!ctx || !host) return AIR_ERR_INVALID_ARG;
    if (l < 0 || l >= ctx->cfg.n_layers) return fail(ctx, AIR_ERR_INVALID_ARG, "bad layer");
    if (!ctx->scored[l]) return fail(ctx, AIR_ERR_STATE, "layer not scored");
    const size_t n = (size_t)ctx->dm.B * ctx->dm.Hkv * ctx->dm.max_vis;
    return d2h(ctx, host, ctx->tab.scores + (size_t)l * n, n * 4);  // the device's own buffer, padding included
}

air_status air_get_elite(air_ctx *ctx, int32_t l, int32_t *counts, int32_t *indices) {
    if (!ctx || !counts || !indices) return AIR_ERR_INVALID_ARG;
    if (l < 0 || l >= ctx->cfg.n_layers) return fail(ctx, AIR_ERR_INVALID_ARG, "bad layer");
    if (!ctx->scored[l]) return fail(ctx, AIR_ERR_STATE, "layer not scored");
    const size_t n = (size_t)ctx->dm.B * ctx->dm.Hq;
    air_status st = d2h(ctx, counts, ctx->tab.elite_cnt + (size_t)l * n, n * 4);
    if (st != AIR_OK) return st;
    return d2h(ctx, indices, ctx->tab.elite_idx + (size_t)l * n * ctx->dm.max_window, n * ctx->dm.max_window * 4);
}

air_status air_get_stats(air_ctx *ctx, double *s_t, double *s_k) {
    if (!ctx || !s_t || !s_k) return AIR_ERR_INVALID_ARG;
    if (!ctx->budgets_ready) return fail(ctx, AIR_ERR_STATE, "air_get_stats: run air_budget first");
    const size_t n = (size_t)ctx->dm.B * ctx->dm.L;
    air_status st = d2h(ctx, s_t, ctx->tab.s_t, n * 8);
    if (st != AIR_OK) return st;
    return d2h(ctx, s_k, ctx->tab.s_k, n * 8);
}

air_status air_get_budgets(air_ctx *ctx, int32_t *host) {
    if (!ctx || !host) return AIR_ERR_INVALID_ARG;
    if (!ctx->budgets_ready) return fail(ctx, AIR_ERR_STATE, "budgets not computed");
    return d2h(ctx, host, ctx->tab.budgets, (size_t)ctx->dm.B * ctx->dm.L * 4);
}

air_status air_set_budgets(air_ctx *ctx, const int32_t *host) {
    if (!ctx || !host) return AIR_ERR_INVALID_ARG;
    if (!ctx->have_seqs) return fail(ctx, AIR_ERR_STATE, "air_set_budgets: score at least one layer first");
    for (int l = 0; l < ctx->cfg.n_layers; ++l)
        if (ctx->compacted[l]) return fail(ctx, AIR_ERR_STATE, "air_set_budgets: layers already compacted");
    const int L = ctx->dm.L;
    for (int b = 0; b < ctx->dm.B; ++b) {
        const air_seq &s = ctx->seqs[b];
        int64_t rows = 0;
        for (int l = 0; l < L; ++l) {
            const int k = host[(size_t)b * L + l];
            if (k < 0 || k > s.vis_len) return fail(ctx, AIR_ERR_SHAPE, "air_set_budgets: budget outside [0, vis_len]");
            const int64_t cap = (int64_t)(s.seq_len - s.vis_len) + k + ctx->dm.max_steps;
            rows += (cap + kCacheRowAlign - 1) / kCacheRowAlign * kCacheRowAlign;
        }
        if (!ctx->cfg.cache_in_place && rows > ctx->dm.pool_rows)
            return fail(ctx, AIR_ERR_SHAPE, "air_set_budgets: budgets exceed the cache pool");
    }
    SeqArgs sa;
    memset(&sa, 0, sizeof(sa));
    memcpy(sa.s, ctx->seqs.data(), sizeof(air_seq) * ctx->cfg.batch);
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(ctx->tab.budgets, host, (size_t)ctx->dm.B * L * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = launch_budget(nullptr, ctx->dm, ctx->tab, ctx->cfg.retention, ctx->cfg.budget_mode,
                                           ctx->cfg.min_keep, 1, sa);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) return hip_fail(ctx, e, "air_set_budgets");
    ctx->fixed_idx.assign(ctx->dm.L, 0);
    ctx->budgets_ready = true;
    return AIR_OK;
}

air_status air_get_indices(air_ctx *ctx, int32_t l, int32_t *host) {
    if (!ctx || !host) return AIR_ERR_INVALID_ARG;
    if (l < 0 || l >= ctx->cfg.n_layers) return fail(ctx, AIR_ERR_INVALID_ARG, "bad layer");
    if (!ctx->compacted[l]) return fail(ctx, AIR_ERR_STATE, "layer not compacted");
    const size_t n = (size_t)ctx->dm.B * ctx->dm.Hkv * ctx->dm.max_vis;
    return d2h(ctx, host, ctx->tab.indices + (size_t)l * n, n * 4);
}

air_status air_set_indices(air_ctx *ctx, int32_t l, const int32_t *host) {
    if (!ctx || !host) return AIR_ERR_INVALID_ARG;
    if (l < 0 || l >= ctx->cfg.n_layers) return fail(ctx, AIR_ERR_INVALID_ARG, "bad layer");
    if (!ctx->budgets_ready) return fail(ctx, AIR_ERR_STATE, "air_set_indices: budgets not computed");
    if (ctx->compacted[l]) return fail(ctx, AIR_ERR_STATE, "air_set_indices: layer already compacted");
    const int L = ctx->dm.L, B = ctx->dm.B, Hkv = ctx->dm.Hkv, NV = ctx->dm.max_vis;
    std::vector<int32_t> budgets((size_t)B * L);
    air_status st = d2h(ctx, budgets.data(), ctx->tab.budgets, budgets.size() * 4);
    if (st != AIR_OK) return st;
    for (int b = 0; b < B; ++b) {
        const int k = budgets[(size_t)b * L + l], n = ctx->seqs[b].vis_len;
        for (int h = 0; h < Hkv; ++h) {
            const int32_t *row = host + ((size_t)b * Hkv + h) * NV;
            for (int i = 0; i < k; ++i)
                if (row[i] < 0 || row[i] >= n || (i > 0 && row[i] <= row[i - 1]))
                    return fail(ctx, AIR_ERR_INVALID_ARG, "air_set_indices: indices must be strictly ascending inside the visual span");
        }
    }
    const size_t n = (size_t)B * Hkv * NV;
    hipError_t e = hipMemcpy(ctx->tab.indices + (size_t)l * n, host, n * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(ctx, e, "air_set_indices");
    ctx->fixed_idx[l] = 1;
    return AIR_OK;
}

air_status air_get_lengths(air_ctx *ctx, int32_t *host) {
    if (!ctx || !host) return AIR_ERR_INVALID_ARG;
    if (!ctx->budgets_ready) return fail(ctx, AIR_ERR_STATE, "budgets not computed");
    const int L = ctx->dm.L;
    air_status st = d2h(ctx, host, ctx->tab.base_len, (size_t)ctx->dm.B * L * 4);
    if (st != AIR_OK) return st;
    std::vector<int32_t> steps;
    if (ctx->cfg.device_steps) {
        st = device_steps(ctx, steps);
        if (st != AIR_OK) return st;
    }
    for (int b = 0; b < ctx->dm.B; ++b)
        for (int l = 0; l < L; ++l)
            // a layer that is not compacted yet has appended nothing (its device count is from the prompt before)
            host[(size_t)b * L + l] += !ctx->cfg.device_steps ? ctx->appended[l] : (ctx->compacted[l] ? steps[(size_t)b * L + l] : 0);
    return AIR_OK;
}

air_status air_get_cache(air_ctx *ctx, int32_t l, int32_t b, int32_t h, void *k_host, void *v_host, int32_t max_rows) {
    if (!ctx || !k_host || !v_host) return AIR_ERR_INVALID_ARG;
    if (l < 0 || l >= ctx->cfg.n_layers || b < 0 || b >= ctx->dm.B || h < 0 || h >= ctx->dm.Hkv)
        return fail(ctx, AIR_ERR_INVALID_ARG, "bad (layer, sequence, head)");
    if (!ctx->compacted[l]) return fail(ctx, AIR_ERR_STATE, "layer not compacted");
    int32_t base = 0, off = 0;
    air_status st = d2h(ctx, &base, ctx->tab.base_len + (size_t)b * ctx->dm.L + l, 4);
    if (st != AIR_OK) return st;
    st = d2h(ctx, &off, ctx->tab.layer_off + (size_t)b * ctx->dm.L + l, 4);
    if (st != AIR_OK) return st;
    int32_t app = ctx->appended[l];
    if (ctx->cfg.device_steps) {
        st = d2h(ctx, &app, ctx->tab.dec_steps + ((size_t)l * ctx->dm.B + b) * ctx->dm.Hkv + h, 4);
        if (st != AIR_OK) return st;
    }
    const int32_t len = base + app;
    if (len > max_rows) return fail(ctx, AIR_ERR_SHAPE, "air_get_cache: max_rows too small");
    const size_t esz = ctx->cfg.dtype == AIR_BF16 ? 2 : 4;
    const size_t rb = (size_t)ctx->dm.D * esz;
    // row of the unit's first cache row, in units of rows from the base the cache is read from
    const char *kbase = (const char *)ctx->tab.kcache, *vbase = (const char *)ctx->tab.vcache;
    size_t row0 = ((size_t)b * ctx->dm.Hkv + h) * (size_t)ctx->dm.pool_rows + off;
    if (ctx->cfg.cache_in_place) {
        kbase = (const char *)ctx->ip_layers[l].k;
        vbase = (const char *)ctx->ip_layers[l].v;
        row0 = ((size_t)b * ctx->tab.ip_kv_b + (size_t)h * ctx->tab.ip_kv_h) / ctx->dm.D;
    }
    if (!v_transposed(ctx->cfg.dtype, ctx->dm.D)) {
        st = d2h(ctx, k_host, kbase + row0 * rb, (size_t)len * rb);
        if (st != AIR_OK) return st;
        return d2h(ctx, v_host, vbase + row0 * rb, (size_t)len * rb);
    }
    // tiled K' and block-transposed V': fetch whole 32-token blocks and put the tokens back in row order
    const int D = ctx->dm.D;
    const size_t n_blk = ((size_t)len + 31) / 32;
    std::vector<uint16_t> raw(n_blk * 32 * D);
    st = d2h(ctx, raw.data(), kbase + row0 * rb, raw.size() * 2);
    if (st != AIR_OK) return st;
    uint16_t *kh = (uint16_t *)k_host;
    for (int r = 0; r < len; ++r)
        for (int col = 0; col < D; ++col) kh[(size_t)r * D + col] = raw[k_tiled(r, col)];
    st = d2h(ctx, raw.data(), vbase + row0 * rb, raw.size() * 2);
    if (st != AIR_OK) return st;
    uint16_t *vh = (uint16_t *)v_host;
    for (int r = 0; r < len; ++r)
        for (int col = 0; col < D; ++col)
            vh[(size_t)r * D + col] = raw[v_tiled(r, col)];
    return AIR_OK;
}

}  // extern "C"
