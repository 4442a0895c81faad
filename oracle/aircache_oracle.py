"""CPU oracle of the AirCache hot path (arxiv 2503.23956).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
the HIP library must compute.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does, and it
shares no code with the HIP path.

Each function follows one passage of the paper; the equations are numbered in
order of appearance in Sec.3 (Eq.1 projections, Eq.2 decode append, Eq.3 token
concatenation, Eq.4 text-only attention, Eq.5 elite index set, Eq.6 gathered
queries/keys, Eq.7 cross-modal attention, Eq.8 importance, Eq.9 strength,
Eq.10 skewness, Eq.11 layer budget; Alg.1 is the two-loop procedure).

Readings taken where the paper leaves a choice (all listed in the design notes):
heads are scored per query head and averaged over the query heads that share a
KV head; the scale is 1/sqrt(head_dim); Eq.7's softmax runs over the visual
keys plus that head's elite text keys with no mask (a causal mask over the elite
text keys is an option, off by default); system-prompt tokens are
never scored and always kept; Eq.10 uses the sample standard deviation; the
a row whose
standard deviation is at most 1e-6 of its mean has zero spread (skewness 0); the
cross-layer normalisation is by shares; budgets are integerised by largest
remainder after clamping to [min_keep, N_v]; ties in top-k go to the lower
token index and kept tokens stay in position order.

Pins (tests/test_oracle_*.py): row sums and torch.softmax for Eq.7; the alpha=0
and alpha=1 special cases and the explicit-softmax form of Eq.5; scipy's
adjusted skewness and closed forms for Eq.10; sum / bound / monotonicity /
uniform invariants for Eq.11; brute-force and stable-argsort top-k;
torch scaled_dot_product_attention and the 100 %-retention identity for decode;
causal scaled_dot_product_attention over the visual span, unit row sums and the
one-hot closed form for the visual observation window.
The whole pipeline has no printed worked example in the paper to compare with:
end-to-end values are "parity unpinned" beyond those per-step pins.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

BUDGET_STRENGTH_SKEW = 0
BUDGET_UNIFORM = 1
BUDGET_STRENGTH = 2
BUDGET_SKEW = 3


@dataclass(frozen=True)
class Segments:
    """[system | visual | text] spans of one prompt and the candidate span of Eq.5."""

    seq_len: int
    vis_start: int
    vis_len: int
    win_start: int
    win_len: int

    @property
    def text_start(self) -> int:
        return self.vis_start + self.vis_len


# ---------------------------------------------------------------------------
# Eq.4-5: text-only attention, last row, elite index set
# ---------------------------------------------------------------------------
def last_row_logits(q_ref: np.ndarray, k_cand: np.ndarray) -> np.ndarray:
    """Scaled logits of the reference (last candidate) query against the candidate text keys (Eq.4, last row)."""
    d = q_ref.shape[-1]
    return (k_cand @ q_ref) / math.sqrt(d)


def elite_set(logits: np.ndarray, alpha: float) -> np.ndarray:
    """Eq.5: candidates whose last-row attention is at least alpha times the row maximum.

    The softmax normaliser is common to both sides and cancels, so the test is
    exp(s_j - max s) >= alpha.  alpha = 0 keeps every candidate, alpha = 1 keeps
    only the maxima.  Returns ascending positions inside the candidate span.
    """
    rel = np.exp(logits - logits.max())
    return np.nonzero(rel >= alpha)[0]


# ---------------------------------------------------------------------------
# Eq.6-8: cross-modal attention of the elite window and importance scores
# ---------------------------------------------------------------------------
def head_importance(q_text_h: np.ndarray, k_h: np.ndarray, seg: Segments, alpha: float,
                    return_attn: bool = False, causal_text: bool = False):
    """Importance of the visual tokens seen by one query head (Eq.4-8).

    q_text_h: [n_text][d] queries of the text span of this query head.
    k_h     : [seq_len][d] keys of the KV head this query head reads.
    causal_text: Eq.7 as printed has no mask (the default).  With this flag an elite row sees only the
        elite text keys at or before its own position, as it did in the model's causal prefill; the
        visual keys all precede every text token and are never masked.
    Returns (I_h [vis_len], elite positions as absolute token indices
    [, A_vtk [R][vis_len + R]]).
    """
    d = k_h.shape[-1]
    t0 = seg.text_start
    cand = np.arange(seg.win_start, seg.win_start + seg.win_len)
    ref = cand[-1]
    s_last = last_row_logits(q_text_h[ref - t0], k_h[cand])
    elite = cand[elite_set(s_last, alpha)]
    q_e = q_text_h[elite - t0]                                  # Q_tk   (Eq.6)
    k_ve = np.concatenate([k_h[seg.vis_start:t0], k_h[elite]])  # K_vtk  (Eq.6)
    s = (q_e @ k_ve.T) / math.sqrt(d)
    if causal_text:  # elite key j (a text token) is visible to elite row r only if it does not come after it
        later = elite[None, :] > elite[:, None]
        s[:, seg.vis_len:] = np.where(later, -np.inf, s[:, seg.vis_len:])
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    a = p / p.sum(axis=1, keepdims=True)                        # A_vtk  (Eq.7)
    imp = a[:, : seg.vis_len].sum(axis=0) / a.shape[0]          # I_v    (Eq.8)
    if return_attn:
        return imp, elite, a
    return imp, elite


def head_importance_visual_window(q_win_h: np.ndarray, k_h: np.ndarray, seg: Segments,
                                  return_attn: bool = False):
    """Importance under a visual observation window (the "visual window" row of the ablation
    table of Sec.4.3: the last continuous visual tokens serve as the reference).

    The candidate span [win_start, win_start + win_len) lies INSIDE the visual span and every
    token of it is a window row (there is no Eq.5 for this window).  The paper gives no
    equation for it; the reading taken is the attention these rows had in prefill, restricted
    to the visual keys as Eq.7 is: row r (visual index p_r) sees the visual keys i <= p_r
    (causal), no text key (all text comes later), and Eq.8 averages the rows.

    q_win_h: [win_len][d] queries of the window tokens of this query head (row j = token win_start + j).
    k_h    : [seq_len][d] keys of the KV head this query head reads.
    Returns I_h [vis_len] (, A [win_len][vis_len]).
    """
    d = k_h.shape[-1]
    k_v = k_h[seg.vis_start:seg.text_start]
    p_row = np.arange(seg.win_start, seg.win_start + seg.win_len) - seg.vis_start
    s = (q_win_h[: seg.win_len] @ k_v.T) / math.sqrt(d)
    s = np.where(np.arange(seg.vis_len)[None, :] <= p_row[:, None], s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    a = p / p.sum(axis=1, keepdims=True)
    imp = a.sum(axis=0) / a.shape[0]
    if return_attn:
        return imp, a
    return imp


def layer_importance_visual_window(q_win: np.ndarray, k: np.ndarray, seg: Segments):
    """Per-KV-head importance of one layer of one sequence under the visual observation window:
    head_importance_visual_window per query head, then the mean over the query heads of a KV head.
    q_win: [H_q][win_len][d], k: [H_kv][seq_len][d].  Returns (I [H_kv][vis_len], window positions
    per query head, for symmetry with layer_importance)."""
    hq, hkv = q_win.shape[0], k.shape[0]
    g = hq // hkv
    imp = np.zeros((hkv, seg.vis_len), dtype=np.float64)
    rows = np.arange(seg.win_start, seg.win_start + seg.win_len)
    for h in range(hq):
        imp[h // g] += head_importance_visual_window(q_win[h], k[h // g], seg)
    imp /= g
    return imp, [rows.copy() for _ in range(hq)]


def layer_importance(q_text: np.ndarray, k: np.ndarray, seg: Segments, alpha: float, causal_text: bool = False):
    """Per-KV-head importance of one layer of one sequence.

    q_text: [H_q][n_text][d], k: [H_kv][seq_len][d] (fp64 values of the stored tensors).
    Each query head has its own elite window; a KV head's importance is the
    plain mean over the query heads that share it.
    Returns (I [H_kv][vis_len], list over query heads of elite index arrays).
    """
    hq, hkv = q_text.shape[0], k.shape[0]
    g = hq // hkv
    imp = np.zeros((hkv, seg.vis_len), dtype=np.float64)
    elites = []
    for h in range(hq):
        i_h, e_h = head_importance(q_text[h], k[h // g], seg, alpha, causal_text=causal_text)
        imp[h // g] += i_h
        elites.append(e_h)
    imp /= g
    return imp, elites


# ---------------------------------------------------------------------------
# Eq.9-10: strength and skewness
# ---------------------------------------------------------------------------
def strength(imp: np.ndarray) -> float:
    """Eq.9: attention mass on the visual tokens."""
    return float(np.sum(imp))


# Relative resolution below which a row's spread counts as zero in Eq.10 (see skewness).
ZERO_SPREAD_REL = 1e-6


def skewness(imp: np.ndarray) -> float:
    """Eq.10: adjusted sample skewness with the sample (n-1) standard deviation.

    Fewer than three tokens, or zero spread, give 0.  Eq.10 divides by sigma^3 and the paper
    does not say what a layer whose visual tokens all score alike gets; the reading taken is
    0, and "alike" is taken at the resolution at which two scores count as equal anywhere
    else in the method's contract (1e-6 relative): sigma <= 1e-6 |mu| is zero spread.  An
    exact test (sigma > 0) would not do: the mean of n equal values is in general not that
    value in floating point, so a constant row would get +-1 instead of 0, and the skewness
    of rounding noise is not a property of the layer.
    """
    n = imp.shape[0]
    if n < 3:
        return 0.0
    mu = float(np.sum(imp)) / n
    c = imp - mu
    var = float(np.sum(c * c)) / (n - 1)
    sigma = math.sqrt(var)
    if not sigma > ZERO_SPREAD_REL * abs(mu):
        return 0.0
    z = c / sigma
    return n / ((n - 1.0) * (n - 2.0)) * float(np.sum(z * z * z))


def layer_stats(imp: np.ndarray) -> Tuple[float, float]:
    """(s_t, s_k) of one layer of one sequence: Eq.9 / Eq.10 per KV head, then the mean over KV heads."""
    hkv = imp.shape[0]
    st = [strength(imp[h]) for h in range(hkv)]
    sk = [skewness(imp[h]) for h in range(hkv)]
    s_t = 0.0
    s_k = 0.0
    for h in range(hkv):  # fixed left-to-right order
        s_t += st[h]
        s_k += sk[h]
    return s_t / hkv, s_k / hkv


# ---------------------------------------------------------------------------
# Eq.11 / Alg.1 second loop: layer budgets
# ---------------------------------------------------------------------------
def total_budget(retention: float, n_vis: int, n_layers: int, min_keep: int = 1) -> int:
    k_tot = int(math.floor(retention * n_vis * n_layers + 0.5))
    lo = n_layers * min(min_keep, n_vis)
    return max(lo, min(k_tot, n_layers * n_vis))


def layer_weights(s_t: Sequence[float], s_k: Sequence[float], mode: int = BUDGET_STRENGTH_SKEW) -> List[float]:
    """Budget shares w_l with sum 1.  Eq.11 with share normalisation:
    s'_t = L*s_t/sum(s_t), s'_k = L*max(s_k,0)/sum(max(s_k,0)), r_hat_l = (s'_t+s'_k)/2 * r,
    so that N_v*r_hat_l = w_l * (r*N_v*L) with w_l = (a_l + b_l)/2.
    Plain left-to-right fp64 sums."""
    n = len(s_t)
    sum_t = 0.0
    sum_k = 0.0
    for l in range(n):
        sum_t += s_t[l]
        sum_k += max(s_k[l], 0.0)
    w = []
    for l in range(n):
        a = s_t[l] / sum_t if sum_t > 0.0 else 1.0 / n
        b = max(s_k[l], 0.0) / sum_k if sum_k > 0.0 else 1.0 / n
        if mode == BUDGET_UNIFORM:
            w.append(1.0 / n)
        elif mode == BUDGET_STRENGTH:
            w.append(a)
        elif mode == BUDGET_SKEW:
            w.append(b)
        else:
            w.append(0.5 * (a + b))
    return w


def layer_budgets(s_t: Sequence[float], s_k: Sequence[float], retention: float, n_vis: int,
                  mode: int = BUDGET_STRENGTH_SKEW, min_keep: int = 1) -> List[int]:
    """Integer number of visual tokens kept per layer (Eq.11, Alg.1 second loop).

    1. shares w_l (layer_weights);
    2. K_tot = floor(r*N_v*L + 1/2), kept inside [L*min_keep, L*N_v];
    3. real allocation x_l proportional to w_l, clamped to [min_keep, N_v]:
       repeat { x_l = w_l / W_free * K_free on the free layers; if none is out
       of range stop; pin the side (above N_v / below min_keep) with the larger
       total violation to its bound and take it out of the free set };
    4. k_l = floor(x_l); the K_tot - sum(k_l) leftover tokens go one each to
       the layers with the largest fractional parts (ties: lower layer).
    """
    n = len(s_t)
    lo = float(min(min_keep, n_vis))
    hi = float(n_vis)
    w = layer_weights(s_t, s_k, mode)
    k_tot = total_budget(retention, n_vis, n, min_keep)
    x = [0.0] * n
    free = [True] * n
    k_free = float(k_tot)
    for _ in range(n + 1):
        w_free = 0.0
        n_free = 0
        for l in range(n):
            if free[l]:
                w_free += w[l]
                n_free += 1
        if n_free == 0:
            break
        over = 0.0
        under = 0.0
        for l in range(n):
            if free[l]:
                x[l] = (w[l] / w_free) * k_free if w_free > 0.0 else k_free / n_free
                if x[l] > hi:
                    over += x[l] - hi
                elif x[l] < lo:
                    under += lo - x[l]
        if over == 0.0 and under == 0.0:
            break
        pin_hi = over >= under
        for l in range(n):
            if free[l]:
                if pin_hi and x[l] > hi:
                    x[l] = hi
                    free[l] = False
                    k_free -= hi
                elif (not pin_hi) and x[l] < lo:
                    x[l] = lo
                    free[l] = False
                    k_free -= lo
    k = [0] * n
    frac = [0.0] * n
    tot = 0
    for l in range(n):
        fl = math.floor(x[l])
        fl = max(int(lo), min(int(fl), n_vis))
        k[l] = fl
        frac[l] = x[l] - fl
        tot += fl
    left = k_tot - tot
    while left > 0:
        best = -1
        for l in range(n):
            if k[l] < n_vis and (best < 0 or frac[l] > frac[best]):
                best = l
        if best < 0:
            break
        k[best] += 1
        frac[best] = -1.0
        left -= 1
    return k


# ---------------------------------------------------------------------------
# Alg.1 second loop: top-k selection and compaction
# ---------------------------------------------------------------------------
def select_topk(imp_row: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest importance scores, ties to the lower index, returned ascending."""
    order = np.argsort(-imp_row, kind="stable")
    return np.sort(order[:k])


def compact_rows(seg: Segments, idx: np.ndarray) -> np.ndarray:
    """Token positions of the compacted cache of one KV head: system, kept visual (ascending), all text."""
    return np.concatenate([
        np.arange(0, seg.vis_start),
        seg.vis_start + idx,
        np.arange(seg.text_start, seg.seq_len),
    ])


def compact(k_h: np.ndarray, v_h: np.ndarray, seg: Segments, idx: np.ndarray):
    """K', V' of one KV head (Alg.1: kept visual rows followed by the text rows; system rows first)."""
    rows = compact_rows(seg, idx)
    return k_h[rows], v_h[rows]


# ---------------------------------------------------------------------------
# Eq.2 + standard attention over the compacted cache
# ---------------------------------------------------------------------------
def decode_attn(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray) -> np.ndarray:
    """softmax(q K'^T / sqrt(d)) V' for the G query heads of one KV head.

    q: [G][d]; k_cache, v_cache: [T][d] (already holding the appended token, Eq.2).
    """
    d = q.shape[-1]
    s = (q @ k_cache.T) / math.sqrt(d)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ v_cache


def decode_layer(q: np.ndarray, k_caches: Sequence[np.ndarray], v_caches: Sequence[np.ndarray]) -> np.ndarray:
    """One layer of one sequence: q [H_q][d]; caches per KV head [T][d].  Query head h reads KV head h // G."""
    hq, hkv = q.shape[0], len(k_caches)
    g = hq // hkv
    out = np.zeros_like(q, dtype=np.float64)
    for kv in range(hkv):
        out[kv * g:(kv + 1) * g] = decode_attn(q[kv * g:(kv + 1) * g], k_caches[kv], v_caches[kv])
    return out


# ---------------------------------------------------------------------------
# Whole method on one sequence (Alg.1), used by the parity tests
# ---------------------------------------------------------------------------
@dataclass
class CompressResult:
    scores: List[np.ndarray]        # per layer [H_kv][vis_len]
    elites: List[List[np.ndarray]]  # per layer, per query head
    s_t: List[float]
    s_k: List[float]
    budgets: List[int]
    indices: List[List[np.ndarray]]  # per layer, per KV head, ascending visual indices


def compress_sequence(q_text_layers, k_layers, seg: Segments, alpha: float, retention: float,
                      mode: int = BUDGET_STRENGTH_SKEW, min_keep: int = 1) -> CompressResult:
    """Alg.1 for one sequence.  q_text_layers[l]: [H_q][n_text][d], k_layers[l]: [H_kv][seq_len][d]."""
    scores, elites, s_t, s_k = [], [], [], []
    for q_text, k in zip(q_text_layers, k_layers):  # first loop
        imp, el = layer_importance(q_text, k, seg, alpha)
        a, b = layer_stats(imp)
        scores.append(imp)
        elites.append(el)
        s_t.append(a)
        s_k.append(b)
    budgets = layer_budgets(s_t, s_k, retention, seg.vis_len, mode, min_keep)
    indices = []
    for imp, kl in zip(scores, budgets):            # second loop
        indices.append([select_topk(imp[h], kl) for h in range(imp.shape[0])])
    return CompressResult(scores, elites, s_t, s_k, budgets, indices)
