/*
 * aircache.h - C ABI of the AirCache hot path for MI355X (gfx950).
 *
 * AirCache (arxiv 2503.23956) compresses the visual part of an LVLM's KV cache once, after
 * prefill, and decodes over the shorter cache.  This library is the data-parallel part of
 * that method (Alg.1 and the decode attention of Sec.3.1):
 *
 *   air_score          Alg.1 first loop:  elite observation window (Eq.4-5), cross-modal
 *                      attention (Eq.6-7), importance I_v (Eq.8), strength and skewness
 *                      (Eq.9-10) of every layer in a range.
 *   air_budget         Eq.11: per-layer budgets from the strength / skewness of all layers.
 *   air_select_compact Alg.1 second loop: top-k by importance, gather of K / V rows into
 *                      the compacted cache.
 *   air_decode_attn    Eq.2 append + softmax(q K'^T / sqrt(d)) V' over the compacted cache.
 *
 * Conventions
 *   - Every tensor pointer is DEVICE memory unless its comment says "host".  Descriptor
 *     arrays (air_layer[], air_seq[]) and getter outputs are HOST memory.
 *   - The caller owns every input tensor and the workspace; the library borrows them for
 *     the duration of the enqueued work and never allocates or frees device memory.
 *   - The four stage calls only enqueue work on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream).  They do not synchronise.  The getters synchronise.
 *   - Every call returns an air_status.  Arguments are validated before anything is
 *     launched, so an error return implies that no device memory was written.
 *     air_last_error() gives a text for the last failure on that context.
 *   - Same inputs give bitwise the same outputs (no floating-point atomics anywhere).
 *   - A context is not thread-safe: the caller serialises the calls on one context.  Contexts are
 *     independent of each other.  Calls that overlap on the device (different streams) must not
 *     touch the same layers of one context.
 *   - Token layout of a prompt: [system | visual | text] (Eq.3; the system prompt is never
 *     scored and always kept).  Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - head_dim is 64 or 128; the innermost (head_dim) axis of every tensor is contiguous.
 */
#ifndef AIRCACHE_H
#define AIRCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct air_ctx air_ctx; /* opaque */

typedef enum {
    AIR_OK = 0,
    AIR_ERR_INVALID_ARG = 1, /* null pointer, bad enum, bad layer range                      */
    AIR_ERR_SHAPE = 2,       /* shape outside what the kernels support or the config allows */
    AIR_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or too small                   */
    AIR_ERR_STATE = 4,       /* stages called out of order, decode capacity exhausted       */
    AIR_ERR_HIP = 5          /* a HIP runtime call failed; see air_last_error               */
} air_status;

typedef enum { AIR_F32 = 0, AIR_BF16 = 1 } air_dtype;

/* How Eq.11 weighs the layers (the paper's allocation and its ablations, Tab.5). */
typedef enum {
    AIR_BUDGET_STRENGTH_SKEW = 0, /* r_l = (s't + s'k)/2 * r  (Eq.11) */
    AIR_BUDGET_UNIFORM = 1,
    AIR_BUDGET_STRENGTH = 2,
    AIR_BUDGET_SKEW = 3
} air_budget_mode;

/* Which tokens serve as the observation window (Sec.3.3; window rows of the ablation table, Tab.5). */
typedef enum {
    AIR_WINDOW_TEXT = 0,  /* candidate span inside the text span, Eq.5 picks the rows (alpha = 0: all of it) */
    AIR_WINDOW_VISUAL = 1 /* the "visual window" ablation: the span lies inside the visual span (the paper
                             takes the last visual tokens) and every token of it is a row; there is no Eq.5
                             (alpha must be 0).  Row r at visual index p_r is normalised over the visual keys
                             i <= p_r (the attention it had in prefill, restricted to the visual keys as
                             Eq.7 is); no text key takes part, so Eq.9 is 1 for every layer.             */
} air_window_kind;

#define AIR_MAX_BATCH 64   /* sequences per context                       */
#define AIR_MAX_LAYERS 256 /* layers per context                          */
#define AIR_MAX_TEXT 4096  /* text tokens per sequence (candidate span)   */

typedef struct {
    int32_t n_layers, n_q_heads, n_kv_heads, head_dim, batch;
    int32_t max_vis_len;      /* largest visual span in the batch                          */
    int32_t max_nonvis_len;   /* largest (system + text) token count in the batch          */
    int32_t max_window;       /* largest candidate span (win_len) in the batch             */
    int32_t max_decode_steps; /* tokens that air_decode_attn may append per layer          */
    int32_t dtype;            /* air_dtype of Q, K, V, the compacted cache and the output  */
    int32_t budget_mode;      /* air_budget_mode                                            */
    int32_t min_keep;         /* lower bound on kept visual tokens per layer (>= 0)        */
    double alpha;             /* relevance threshold of Eq.5, in [0,1]; the paper uses 0.9 */
    double retention;         /* r: fraction of visual tokens kept overall, in (0,1]       */
    int32_t window_kind;      /* air_window_kind; 0 = the paper's text windows              */
    int32_t device_steps;     /* 0: the host counts the tokens air_decode_attn has appended and passes the
                                 count with every launch.  1 (bf16, head_dim 128 only): the count lives in
                                 device memory and advances with every decode launch that RUNS, so that a
                                 decode step captured in a HIP graph can be replayed; see air_decode_attn */
    int32_t cache_in_place;   /* 0: the compacted cache lives in the workspace.  1 (bf16, head_dim 128 only):
                                 air_select_compact compacts every layer INSIDE the prompt's own K / V tensors
                                 (App. A names the full-size cache kept until every layer is scored as the
                                 method's memory cost; this mode at least adds no second copy to it): the
                                 workspace then holds no cache pool, the layer's K / V tensors become its cache
                                 (the caller keeps them alive and no longer reads them), and decode appends
                                 into them.  Needs token stride == head_dim (each (sequence, KV head) a
                                 contiguous run of rows) and, per head, rows for the prompt plus
                                 max_decode_steps rounded up to a multiple of 32 (head stride / head_dim)    */
    int32_t causal_text;      /* 0: Eq.7 as printed, every elite row sees every elite text key.  1: an elite row
                                 sees only the elite text keys at or before its own position (what it saw in
                                 the model's causal prefill); visual keys are never masked.  Text windows only */
} air_config;

/* One prompt.  system = [0, vis_start), visual = [vis_start, vis_start+vis_len),
 * text = [vis_start+vis_len, seq_len).  [win_start, win_start+win_len) is the candidate
 * span of Eq.5, inside the text span; its last token is the reference row of Eq.4.
 * win_len == text length and alpha = 0.9 is the paper's elite window; alpha = 0 turns
 * the span into a plain continuous observation window (Tab.5).  With AIR_WINDOW_VISUAL the
 * span lies inside the visual span instead and all of it is the window. */
typedef struct {
    int32_t seq_len, vis_start, vis_len, win_start, win_len;
} air_seq;

/* One layer's tensors (device pointers). */
typedef struct {
    const void *q_text; /* [B][H_q ][text][d]: queries of the text span; row j = text token j
                           (AIR_WINDOW_VISUAL: [B][H_q][win_len][d], row j = token win_start + j) */
    const void *k;      /* [B][H_kv][seq ][d]                                                  */
    const void *v;      /* [B][H_kv][seq ][d]                                                  */
} air_layer;

/* Element strides shared by all layers of a call (innermost axis has stride 1). */
typedef struct {
    int64_t q_b, q_h, q_t;    /* q_text: batch, head, token */
    int64_t kv_b, kv_h, kv_t; /* k and v: batch, head, token */
} air_strides;

/* Bytes of device workspace a context with this config needs (0 on invalid config). */
size_t air_workspace_bytes(const air_config *cfg);

/* Create a context over a caller-allocated device workspace (256-byte aligned, at least
 * air_workspace_bytes(cfg)).  Clears its bookkeeping tables on the default stream and
 * waits for that.  The context itself is a small host object freed by air_destroy. */
air_status air_create(const air_config *cfg, void *workspace, size_t workspace_bytes, air_ctx **out);
air_status air_destroy(air_ctx *ctx);

/* Launch-shape overrides for tests and tuning.  They change how the work is cut into workgroups and
 * never a result; every shape they can force is a shape the library may choose by itself.  A field left
 * at 0 (select_direct_max: at -1) leaves that choice to the library, which is the state after air_create.
 * Not part of the method: no passage of the paper stands behind this call.  Nothing in the library reads
 * the environment. */
typedef struct {
    int32_t decode_splits;     /* workgroups per (layer, sequence, KV head) of air_decode_attn: 1, 2, 4, 8 or 16 */
    int32_t decode_waves;      /* wavefronts per workgroup of air_decode_attn: 1, 2, 4 or 8                     */
    int32_t decode_tiles;      /* 16-key tiles per loop iteration of a wave: 2, 4 or 8                          */
    int32_t score_block_mb;    /* MB of K_v scored per pair of passes when a window needs two passes: 1..65536   */
    int32_t score_rows_kernel; /* 1: the elite window's row parameters by their own kernel                       */
    int32_t select_threads;    /* workgroup size of the selection kernel: 256 or 512                             */
    int32_t select_direct_max; /* largest deciding bin that is ranked directly, 0..1024 (0: always the radix
                                  passes); -1: the library's default                                            */
    int32_t gather_wgs;        /* workgroups per unit of the compaction gather: 1..64                            */
    int32_t decode_order;      /* order of the units of a decode launch over all layers: 1 by layer, 2 longest
                                  cache first (where the launch shape has that variant)                         */
    int32_t decode_halves;     /* two workgroups per unit with one half of the columns of V' each, in decode launches
                                  whose shape has that variant: 1 never, 2 whatever the number of units (the library
                                  takes it up to 128 units per launch)                                               */
    int32_t budget_in_score;   /* 1: air_score never does the allocation of Eq.11 in the tail of its last kernel
                                  (air_budget then launches the budget kernel, as it does beyond 64 layers)       */
} air_tuning;
/* AIR_ERR_INVALID_ARG (and no change) if a field holds a value outside its list. */
air_status air_set_tuning(air_ctx *ctx, const air_tuning *tuning);

/* Forget the prompt: the context returns to its state after air_create (no layer scored,
 * no budgets, empty caches) so that the next prompt of the same shape can be compressed.
 * Host bookkeeping only; nothing is enqueued and device memory is left as it is. */
air_status air_reset(air_ctx *ctx);

/* Alg.1, first loop (Eq.4-10) for layers [l0, l1).  layers: host array of l1-l0 entries;
 * seqs: host array of cfg.batch entries, the same for every call on this context (the
 * first call fixes it).  Fills importance scores and per-layer strength / skewness. */
air_status air_score(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const air_layer *layers,
                     const air_strides *strides, const air_seq *seqs);

/* Eq.11 for every sequence.  All layers must have been scored (else AIR_ERR_STATE).  Where every layer went
 * through air_score exactly once since the reset, on the bf16 / head_dim 128 path with at most 64 layers and 16 KV
 * heads, the last kernel of air_score has done the allocation in its tail and this call launches nothing; it is
 * still the call that makes the budgets available to air_select_compact.  Call it on the stream air_score ran on
 * (or one ordered behind it). */
air_status air_budget(air_ctx *ctx, void *stream);

/* Alg.1, second loop for layers [l0, l1): top-k_l visual tokens per (sequence, KV head)
 * by importance (ties to the lower token index), then K' = [K_sys ; K_v[idx] ; K_t] and
 * V' likewise into the compacted cache inside the workspace.  Needs air_budget (or
 * air_set_budgets).  After the enqueued work has run the caller may free the prompt K/V.
 * With cfg.cache_in_place the rows are instead compacted inside layers[].k / layers[].v themselves (see
 * air_config): those tensors ARE the cache afterwards and must stay alive; AIR_ERR_SHAPE if their strides or
 * rows per head do not allow it (checked for the largest budget there can be, without waiting for the device). */
air_status air_select_compact(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const air_layer *layers,
                              const air_strides *strides);

/* One decode step for layers [l0, l1): appends k_new / v_new to each layer's compacted
 * cache (Eq.2), then out[h] = softmax(q_h K'^T / sqrt(d)) V' over the whole cache
 * including the new token.  All tensors dense: q_new, out [l1-l0][B][H_q][d];
 * k_new, v_new [l1-l0][B][H_kv][d].  At most max_decode_steps calls per layer.
 * The call enqueues kernel launches only (no copy, no memset, no allocation, no host wait), so it
 * can be recorded into a HIP graph.  With cfg.device_steps the recorded step advances the cache by
 * itself on every replay; the host then cannot check the capacity: a step that runs with the cache
 * full appends nothing, leaves `out` as it is and raises a flag that makes air_get_lengths fail
 * with AIR_ERR_STATE.  air_select_compact starts a layer's count at zero again. */
air_status air_decode_attn(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const void *q_new,
                           const void *k_new, const void *v_new, void *out);

/* air_decode_attn for callers that must not allocate and whose workspace must not serve as scratch: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * results (bit for bit) as air_decode_attn; the one difference is where the workgroups of a unit exchange
 * their split-K partials and arrival counters: in a fixed array of 8.1 MiB inside the library's device image
 * (every GPU the library runs on holds its copy until the process ends) instead of the workspace.  The call
 * allocates nothing and calls no allocating routine.
 *   - Limit: a launch that exchanges partials may have at most 1024 (unit, split) pairs, unit = (layer,
 *     sequence, KV head) of the call; beyond that the call returns AIR_ERR_SHAPE before anything is launched
 *     (pass fewer layers per call).  Launches with one workgroup per unit exchange nothing and have no limit.
 *   - The array is shared by every context and call on one GPU and keeps the last call's contents; the call
 *     clears the counters it needs with a small kernel first.  Calls that overlap on one GPU (two streams,
 *     two contexts, two threads) race on it: serialise them. */
air_status air_decode_attn_static(air_ctx *ctx, void *stream, int32_t l0, int32_t l1, const void *q_new,
                                  const void *k_new, const void *v_new, void *out);

/* ---- inspection (tests, debugging): these synchronise the device ---- */
/* importance scores of layer l: host [B][H_kv][max_vis_len], the device buffer as it is (entries past a
 * sequence's vis_len are never written by the library: zero on a context that has seen one prompt) */
air_status air_get_scores(air_ctx *ctx, int32_t l, float *host);
/* elite window of layer l: counts host [B][H_q]; indices host [B][H_q][max_window] (absolute token positions) */
air_status air_get_elite(air_ctx *ctx, int32_t l, int32_t *counts, int32_t *indices);
/* per-layer strength and skewness: host [B][L] each */
air_status air_get_stats(air_ctx *ctx, double *s_t, double *s_k);
/* budgets k[b][l]: host [B][L] */
air_status air_get_budgets(air_ctx *ctx, int32_t *host);
/* replace the budgets (stage-isolated tests); every entry in [0, vis_len of b] */
air_status air_set_budgets(air_ctx *ctx, const int32_t *host);
/* kept visual indices of layer l: host [B][H_kv][max_vis_len], ascending, first k[b][l] valid */
air_status air_get_indices(air_ctx *ctx, int32_t l, int32_t *host);
/* Fix the kept visual indices of layer l instead of selecting them (same layout as air_get_indices;
 * the first k[b][l] entries of every row must be strictly ascending and inside [0, vis_len of b]):
 * air_select_compact then only gathers that layer.  With budgets of 1 this keeps the single token of
 * a chosen importance rank, the one-token-at-a-time study of Sec.4.3 (Fig.4); it also isolates the
 * gather for tests.  Needs budgets; computing or setting budgets again forgets the fixed indices. */
air_status air_set_indices(air_ctx *ctx, int32_t l, const int32_t *host);
/* current cache length (system + kept + text + appended) per (b, l): host [B][L] */
air_status air_get_lengths(air_ctx *ctx, int32_t *host);
/* rows [0, length) of the compacted cache of (layer l, sequence b, KV head h) in token
 * order, element type = cfg.dtype: host [max_rows][d] each; fails if length > max_rows */
air_status air_get_cache(air_ctx *ctx, int32_t l, int32_t b, int32_t h, void *k_host, void *v_host,
                         int32_t max_rows);

const char *air_last_error(const air_ctx *ctx);
const char *air_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AIRCACHE_H */
