"""Shared machinery of the GPU parity tests: run the HIP path and the oracle on the same seeded inputs.

Tolerances (the bar the task states):
  * elite index sets, budgets (given the same statistics), compacted rows: bit-exact;
  * fp32 importance scores: 1e-5 relative (plus 1e-30 absolute for entries that underflow);
  * selected index sets: identical, except that candidates whose oracle score lies within
    1e-6 relative of the oracle's k-th largest score may be swapped for one another;
  * decode outputs: 2e-2 absolute for bf16, 1e-4 absolute for fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

import synth
from oracle import aircache_oracle as O

SCORE_RTOL = 1e-5
SCORE_ATOL = 1e-30
STAT_RTOL = 1e-5
SWAP_RTOL = 1e-6
DECODE_ATOL = {"bf16": 2e-2, "f32": 1e-4}


def seg_of(s) -> O.Segments:
    return O.Segments(s.seq_len, s.vis_start, s.vis_len, s.win_start, s.win_len)


@dataclass
class OracleRun:
    scores: List[List[np.ndarray]] = field(default_factory=list)   # [l][b] -> [H_kv][vis_len]
    elites: List[List[List[np.ndarray]]] = field(default_factory=list)  # [l][b][h]
    s_t: Optional[np.ndarray] = None  # [B][L]
    s_k: Optional[np.ndarray] = None
    budgets: Optional[np.ndarray] = None  # [B][L]


def oracle_score_layer(w, li, seqs, alpha, causal_text=False):
    """Oracle importance + stats of one generated layer for every sequence."""
    out_scores, out_elites, st, sk = [], [], [], []
    for b, s in enumerate(seqs):
        q = synth.storage_to_f64(li.q_text[b][:, : s.n_text])
        k = synth.storage_to_f64(li.k[b][:, : s.seq_len])
        imp, el = O.layer_importance(q, k, seg_of(s), alpha, causal_text)
        a, c = O.layer_stats(imp)
        out_scores.append(imp)
        out_elites.append(el)
        st.append(a)
        sk.append(c)
    return out_scores, out_elites, st, sk


def oracle_score_layer_visual_window(w, q_win, li, seqs):
    """The same for the visual observation window; q_win [B][H_q][>=win_len][d] holds the window rows' queries."""
    out_scores, out_elites, st, sk = [], [], [], []
    for b, s in enumerate(seqs):
        q = synth.storage_to_f64(q_win[b][:, : s.win_len])
        k = synth.storage_to_f64(li.k[b][:, : s.seq_len])
        imp, rows = O.layer_importance_visual_window(q, k, seg_of(s))
        a, c = O.layer_stats(imp)
        out_scores.append(imp)
        out_elites.append(rows)
        st.append(a)
        sk.append(c)
    return out_scores, out_elites, st, sk


def oracle_budgets(s_t, s_k, seqs, retention, mode=0, min_keep=1):
    """[B][L] budgets from [B][L] statistics."""
    return np.array([O.layer_budgets(list(s_t[b]), list(s_k[b]), retention, s.vis_len, mode, min_keep)
                     for b, s in enumerate(seqs)], dtype=np.int32)


def check_scores(gpu_scores: np.ndarray, oracle_scores: List[np.ndarray], seqs, tag=""):
    """gpu_scores [B][H_kv][max_vis] vs oracle list over b of [H_kv][vis_len]."""
    worst = 0.0
    for b, s in enumerate(seqs):
        g = gpu_scores[b][:, : s.vis_len].astype(np.float64)
        o = oracle_scores[b]
        err = np.abs(g - o) / (SCORE_RTOL * np.abs(o) + SCORE_ATOL)
        worst = max(worst, float(err.max()))
        assert err.max() <= 1.0, f"{tag} b={b}: score error {err.max():.3g}x tolerance at {np.unravel_index(err.argmax(), err.shape)}"
        assert np.all(gpu_scores[b][:, s.vis_len:] == 0.0), f"{tag} b={b}: padding scores not zero"
    return worst * SCORE_RTOL


def check_elite(cnt: np.ndarray, idx: np.ndarray, oracle_elites, tag=""):
    for b in range(cnt.shape[0]):
        for h in range(cnt.shape[1]):
            want = oracle_elites[b][h]
            got = idx[b, h, : cnt[b, h]]
            assert cnt[b, h] == len(want) and np.array_equal(got, want), f"{tag} b={b} h={h}: elite {got} != {want}"


def check_selection(gpu_idx: np.ndarray, oracle_scores_row: np.ndarray, k: int, tag=""):
    """Index set of one (layer, sequence, KV head).  Returns the number of tolerated swaps."""
    assert gpu_idx.shape[0] == k
    if k == 0:
        return 0
    assert np.all(np.diff(gpu_idx) > 0), f"{tag}: indices not strictly ascending"
    assert gpu_idx[0] >= 0 and gpu_idx[-1] < oracle_scores_row.shape[0], f"{tag}: index out of range"
    want = O.select_topk(oracle_scores_row, k)
    if np.array_equal(gpu_idx, want):
        return 0
    a, g = set(want.tolist()), set(gpu_idx.tolist())
    only_o, only_g = sorted(a - g), sorted(g - a)
    assert len(only_o) == len(only_g)
    tau = np.sort(oracle_scores_row)[::-1][k - 1]
    for i in only_o + only_g:
        rel = abs(oracle_scores_row[i] - tau) / tau
        assert rel < SWAP_RTOL, f"{tag}: token {i} swapped across the top-{k} boundary, oracle score {rel:.3g} relative away from it"
    return len(only_o)
