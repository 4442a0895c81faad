"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no worked numeric example, so the pins are closed forms,
hand-worked small cases, invariants, library routines (torch.softmax,
scipy.stats.skew, torch scaled_dot_product_attention) and brute force on tiny
inputs.  Each is chosen so that a plausible slip in the oracle (a dropped term,
a wrong sign or index, a transposed operand, a wrong normaliser) fails it.
"""
import math

import numpy as np
import pytest
import scipy.stats
import torch

from oracle import aircache_oracle as O


def _seg(n_sys, n_vis, n_text, win=None):
    win = n_text if win is None else win
    L = n_sys + n_vis + n_text
    return O.Segments(L, n_sys, n_vis, L - win, win)


# ---------------------------------------------------------------------------
# Eq.4-5
# ---------------------------------------------------------------------------
def test_last_row_logits_explicit_loops():
    rng = np.random.default_rng(1)
    q = rng.standard_normal(6)
    k = rng.standard_normal((5, 6))
    got = O.last_row_logits(q, k)
    for j in range(5):
        acc = 0.0
        for c in range(6):
            acc += q[c] * k[j, c]
        assert got[j] == pytest.approx(acc / math.sqrt(6.0), rel=1e-14)


def test_elite_alpha_zero_keeps_all_alpha_one_keeps_argmax():
    # Sec.3.3 below Eq.5: alpha = 0 retains all text tokens, alpha = 1 only the top-scoring one
    s = np.array([0.3, -1.0, 2.5, 2.4999, 0.0])
    assert O.elite_set(s, 0.0).tolist() == [0, 1, 2, 3, 4]
    assert O.elite_set(s, 1.0).tolist() == [2]


def test_elite_matches_explicit_softmax_threshold():
    rng = np.random.default_rng(2)
    for trial in range(200):
        n = int(rng.integers(2, 40))
        s = rng.standard_normal(n) * 2.0
        alpha = float(rng.uniform(0.05, 0.99))
        a = torch.softmax(torch.from_numpy(s), dim=0).numpy()
        margin = np.abs(a - alpha * a.max()) / a.max()
        if margin.min() < 1e-9:  # borderline by rounding: skip
            continue
        want = np.nonzero(a >= alpha * a.max())[0]
        assert O.elite_set(s, alpha).tolist() == want.tolist()
        # closed form: s_j >= s_max + ln(alpha)
        want2 = np.nonzero(s >= s.max() + math.log(alpha))[0]
        assert O.elite_set(s, alpha).tolist() == want2.tolist()


def test_elite_is_independent_of_extra_softmax_keys():
    # the normaliser of Eq.4 cancels in Eq.5: appending lower-scoring keys to the row changes nothing
    rng = np.random.default_rng(3)
    s = rng.standard_normal(12)
    extra = s.min() - 1.0 - rng.uniform(0, 3, size=7)
    a = torch.softmax(torch.from_numpy(np.concatenate([s, extra])), dim=0).numpy()
    alpha = 0.5
    want = np.nonzero(a[:12] >= alpha * a.max())[0]
    assert O.elite_set(s, alpha).tolist() == want.tolist()


# ---------------------------------------------------------------------------
# Eq.6-8
# ---------------------------------------------------------------------------
def _brute_head_importance(q_text, k, seg, alpha):
    """Eq.4-8 with explicit python loops and math.exp (tiny inputs only)."""
    d = k.shape[1]
    t0 = seg.text_start
    cand = list(range(seg.win_start, seg.win_start + seg.win_len))
    ref = cand[-1]
    s_last = []
    for j in cand:
        s_last.append(sum(q_text[ref - t0][c] * k[j][c] for c in range(d)) / math.sqrt(d))
    z = sum(math.exp(x) for x in s_last)
    att = [math.exp(x) / z for x in s_last]
    elite = [cand[i] for i in range(len(cand)) if att[i] >= alpha * max(att)]
    keys = list(range(seg.vis_start, t0)) + elite
    imp = [0.0] * seg.vis_len
    for r in elite:
        logits = [sum(q_text[r - t0][c] * k[j][c] for c in range(d)) / math.sqrt(d) for j in keys]
        zz = sum(math.exp(x) for x in logits)
        for i in range(seg.vis_len):
            imp[i] += math.exp(logits[i]) / zz / len(elite)
    return imp, elite


@pytest.mark.parametrize("alpha", [0.0, 0.5, 0.9, 1.0])
def test_head_importance_brute_force(alpha):
    rng = np.random.default_rng(10)
    seg = _seg(2, 7, 5, win=4)
    k = rng.standard_normal((seg.seq_len, 4))
    q_text = rng.standard_normal((5, 4)) * 1.5
    imp, elite = O.head_importance(q_text, k, seg, alpha)
    want, want_elite = _brute_head_importance(q_text, k, seg, alpha)
    assert elite.tolist() == want_elite
    np.testing.assert_allclose(imp, want, rtol=1e-12)


def test_softmax_domain_and_scale_closed_form():
    # one elite row (alpha = 1); scaled logits ln3, 0 on two visual keys and 0 on the elite text key
    # => attention 3/5, 1/5, 1/5; I_v = [0.6, 0.2]; strength 0.8.  Pins the 1/sqrt(d) scale and
    # that the elite text key sits in the denominator of Eq.7.
    d = 4
    q = np.zeros((1, d))
    q[0, 0] = 2.0
    k = np.zeros((3, d))
    k[0, 0] = math.sqrt(d) * math.log(3.0) / 2.0
    seg = _seg(0, 2, 1)
    imp, elite, a = O.head_importance(q, k, seg, 1.0, return_attn=True)
    assert elite.tolist() == [2]
    np.testing.assert_allclose(a[0], [0.6, 0.2, 0.2], rtol=1e-14)
    np.testing.assert_allclose(imp, [0.6, 0.2], rtol=1e-14)
    assert O.strength(imp) == pytest.approx(0.8, rel=1e-14)


def test_cross_modal_rows_sum_to_one_and_match_torch_softmax():
    rng = np.random.default_rng(11)
    seg = _seg(3, 50, 9)
    d = 8
    k = rng.standard_normal((seg.seq_len, d))
    q_text = rng.standard_normal((9, d)) * 2
    imp, elite, a = O.head_importance(q_text, k, seg, 0.3, return_attn=True)
    assert a.shape == (len(elite), seg.vis_len + len(elite))
    np.testing.assert_allclose(a.sum(axis=1), 1.0, atol=1e-12)
    k_ve = np.concatenate([k[3:53], k[elite]])
    logits = torch.from_numpy(q_text[elite - seg.text_start] @ k_ve.T / math.sqrt(d))
    np.testing.assert_allclose(a, torch.softmax(logits, dim=1).numpy(), rtol=1e-12)
    np.testing.assert_allclose(imp, a[:, :50].mean(axis=0), rtol=1e-13)
    # strength + mass on the elite text columns = 1
    assert O.strength(imp) + a[:, 50:].sum() / len(elite) == pytest.approx(1.0, abs=1e-12)
    assert 0.0 < O.strength(imp) < 1.0


def test_identical_visual_keys_give_uniform_importance():
    rng = np.random.default_rng(12)
    seg = _seg(1, 20, 4)
    k = rng.standard_normal((seg.seq_len, 6))
    k[1:21] = k[1]
    q_text = rng.standard_normal((4, 6))
    imp, _ = O.head_importance(q_text, k, seg, 0.0)
    np.testing.assert_allclose(imp, imp[0], rtol=1e-13)
    assert imp[0] == pytest.approx(O.strength(imp) / 20, rel=1e-13)


def test_visual_permutation_permutes_importance_and_system_tokens_are_ignored():
    rng = np.random.default_rng(13)
    seg = _seg(4, 30, 6)
    k = rng.standard_normal((seg.seq_len, 8))
    q_text = rng.standard_normal((6, 8))
    imp, el = O.head_importance(q_text, k, seg, 0.7)
    perm = rng.permutation(30)
    k2 = k.copy()
    k2[4:34] = k[4:34][perm]
    k2[:4] = rng.standard_normal((4, 8)) * 50  # system keys never enter the compress pass
    imp2, el2 = O.head_importance(q_text, k2, seg, 0.7)
    assert el.tolist() == el2.tolist()
    np.testing.assert_allclose(imp2, imp[perm], rtol=1e-12)


def test_common_key_shift_leaves_importance_unchanged():
    # adding one vector to every key adds a per-row constant to the logits: softmax rows and
    # the elite set are unchanged
    rng = np.random.default_rng(14)
    seg = _seg(0, 25, 7)
    k = rng.standard_normal((seg.seq_len, 8))
    q_text = rng.standard_normal((7, 8))
    imp, el = O.head_importance(q_text, k, seg, 0.6)
    imp2, el2 = O.head_importance(q_text, k + rng.standard_normal(8), seg, 0.6)
    assert el.tolist() == el2.tolist()
    np.testing.assert_allclose(imp2, imp, rtol=1e-10)


def test_candidate_span_restricts_the_window():
    rng = np.random.default_rng(15)
    seg = _seg(2, 12, 10, win=3)
    k = rng.standard_normal((seg.seq_len, 4))
    q_text = rng.standard_normal((10, 4))
    _, el = O.head_importance(q_text, k, seg, 0.0)
    assert el.tolist() == [seg.seq_len - 3, seg.seq_len - 2, seg.seq_len - 1]


def test_gqa_grouping_reads_the_right_kv_head():
    # KV head 1 has identical visual keys: every query head reading it must give a uniform row;
    # KV head 0 is random.  Query heads 0,1,2 read KV head 0 and 3,4,5 read KV head 1.
    rng = np.random.default_rng(16)
    seg = _seg(1, 16, 5)
    k = rng.standard_normal((2, seg.seq_len, 4))
    k[1, 1:17] = k[1, 1]
    q_text = rng.standard_normal((6, 5, 4))
    imp, elites = O.layer_importance(q_text, k, seg, 0.5)
    assert len(elites) == 6
    np.testing.assert_allclose(imp[1], imp[1, 0], rtol=1e-13)
    assert np.ptp(imp[0]) > 1e-3
    # mean over the group with equal weight per head
    heads = [O.head_importance(q_text[h], k[0], seg, 0.5)[0] for h in range(3)]
    np.testing.assert_allclose(imp[0], (heads[0] + heads[1] + heads[2]) / 3.0, rtol=1e-13)


# ---------------------------------------------------------------------------
# Visual observation window (ablation table of Sec.4.3)
# ---------------------------------------------------------------------------
def _vis_seg(n_sys, n_vis, n_text, win_first, win):
    return O.Segments(n_sys + n_vis + n_text, n_sys, n_vis, n_sys + win_first, win)


@pytest.mark.parametrize("win_first,win", [(44, 6), (17, 5), (0, 4), (49, 1)])
def test_visual_window_matches_causal_sdpa_over_the_visual_span(win_first, win):
    # library route: causal attention of ALL visual queries over the visual keys with V = identity
    # returns the attention matrix itself; the window rows of it, averaged, are Eq.8
    rng = np.random.default_rng(40 + win)
    n_vis, d = 50, 8
    seg = _vis_seg(3, n_vis, 7, win_first, win)
    k = rng.standard_normal((seg.seq_len, d))
    q_all = rng.standard_normal((n_vis, d))  # queries of every visual token
    a_full = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q_all)[None], torch.from_numpy(k[3:3 + n_vis])[None],
        torch.eye(n_vis, dtype=torch.float64)[None], is_causal=True)[0].numpy()
    want = a_full[win_first:win_first + win].mean(axis=0)
    got, a = O.head_importance_visual_window(q_all[win_first:win_first + win], k, seg, return_attn=True)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(a.sum(axis=1), 1.0, rtol=1e-13)   # every row is a distribution over visual keys
    assert np.all(got[win_first + win:] == 0.0)                   # nothing after the window is ever seen
    assert abs(O.strength(got) - 1.0) < 1e-12                     # Eq.9 is identically 1 for this window


def test_visual_window_closed_forms():
    rng = np.random.default_rng(44)
    n_vis, d = 36, 4
    k = rng.standard_normal((2 + n_vis + 5, d))
    # a single row at the first visual token sees only itself: one-hot importance, skewness sqrt(N_v)
    imp = O.head_importance_visual_window(rng.standard_normal((1, d)), k, _vis_seg(2, n_vis, 5, 0, 1))
    assert imp[0] == 1.0 and np.all(imp[1:] == 0.0)
    assert abs(O.skewness(imp) - math.sqrt(n_vis)) < 1e-12
    # identical visual keys: row p spreads 1/(p+1) over keys 0..p
    k[2:2 + n_vis] = k[2]
    seg = _vis_seg(2, n_vis, 5, n_vis - 3, 3)
    imp = O.head_importance_visual_window(rng.standard_normal((3, d)), k, seg)
    want = np.zeros(n_vis)
    for p in (n_vis - 3, n_vis - 2, n_vis - 1):
        want[: p + 1] += 1.0 / (p + 1) / 3.0
    np.testing.assert_allclose(imp, want, rtol=1e-13)
    # the scale is 1/sqrt(head_dim): two keys, one row at the second, logits (0, ln 3 * sqrt d) -> (1/4, 3/4)
    k2 = np.zeros((1 + 2 + 1, d)); k2[2, 0] = 1.0
    q = np.zeros((1, d)); q[0, 0] = math.log(3.0) * math.sqrt(d)
    imp = O.head_importance_visual_window(q, k2, O.Segments(4, 1, 2, 2, 1))
    np.testing.assert_allclose(imp, [0.25, 0.75], rtol=1e-13)


def test_visual_window_layer_is_mean_over_the_group_and_reads_the_right_kv_head():
    rng = np.random.default_rng(45)
    seg = _vis_seg(1, 20, 4, 16, 4)
    k = rng.standard_normal((2, seg.seq_len, 4))
    q_win = rng.standard_normal((4, 4, 4))
    imp, rows = O.layer_importance_visual_window(q_win, k, seg)
    assert [r.tolist() for r in rows] == [[17, 18, 19, 20]] * 4
    for kv in range(2):
        heads = [O.head_importance_visual_window(q_win[h], k[kv], seg) for h in (2 * kv, 2 * kv + 1)]
        np.testing.assert_allclose(imp[kv], (heads[0] + heads[1]) / 2.0, rtol=1e-13)


def test_causal_text_option_masks_later_elite_keys_only():
    # Eq.7 with the optional causal mask over the elite text keys: every row equals causal scaled-dot-product attention
    # of that text token over [visual keys ; elite text keys] (torch, fp64, explicit mask); the last elite row sees every
    # key either way; with a single elite row the option changes nothing; visual columns are never masked
    import torch

    rng = np.random.default_rng(26)
    d, n_vis, n_text, ns = 16, 40, 12, 2
    seg = O.Segments(ns + n_vis + n_text, ns, n_vis, ns + n_vis, n_text)
    k = rng.standard_normal((seg.seq_len, d))
    q = rng.standard_normal((n_text, d)) * 0.3  # mild logits: several tokens pass the threshold
    imp_c, elite, a_c = O.head_importance(q, k, seg, 0.2, return_attn=True, causal_text=True)
    imp_u, elite_u, a_u = O.head_importance(q, k, seg, 0.2, return_attn=True)
    assert np.array_equal(elite, elite_u) and len(elite) >= 3
    keys = np.concatenate([k[seg.vis_start:seg.text_start], k[elite]])
    mask = np.ones((len(elite), n_vis + len(elite)), dtype=bool)
    mask[:, n_vis:] = elite[None, :] <= elite[:, None]
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q[elite - seg.text_start])[None], torch.from_numpy(keys)[None], torch.eye(n_vis + len(elite), dtype=torch.float64)[None],
        attn_mask=torch.from_numpy(mask)[None]).numpy()[0]  # V = identity: the output is the attention matrix itself
    np.testing.assert_allclose(a_c, want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(a_c.sum(axis=1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(a_c[-1], a_u[-1], rtol=1e-13)       # the last elite row sees every elite key
    assert np.all(a_c[:, n_vis:][~mask[:, n_vis:]] == 0.0) and np.all(a_c[:, :n_vis] > 0.0)
    assert np.all(a_c[:-1, :n_vis] >= a_u[:-1, :n_vis])            # mass taken from masked keys goes to the visible ones
    np.testing.assert_allclose(imp_c, a_c[:, :n_vis].mean(axis=0), rtol=1e-13)
    one_c = O.head_importance(q, k, seg, 1.0, causal_text=True)[0]  # alpha = 1: a single elite row
    one_u = O.head_importance(q, k, seg, 1.0)[0]
    assert np.array_equal(one_c, one_u)


# ---------------------------------------------------------------------------
# Eq.9-10
# ---------------------------------------------------------------------------
def test_skewness_matches_scipy_adjusted():
    rng = np.random.default_rng(20)
    for n in (3, 4, 17, 576, 7290):
        x = rng.gamma(0.3, size=n)
        assert O.skewness(x) == pytest.approx(scipy.stats.skew(x, bias=False), rel=1e-10)


def test_skewness_closed_forms():
    # one-hot vector of length n: adjusted skewness = sqrt(n) exactly
    for n in (9, 576, 7290):
        x = np.zeros(n)
        x[n // 3] = 1.0
        assert O.skewness(x) == pytest.approx(math.sqrt(n), rel=1e-12)
    # 0/1 vector with m ones out of n: (1-2p)/sqrt(p(1-p)) * sqrt(n(n-1))/(n-2)
    n, m = 1000, 50
    x = np.zeros(n)
    x[:m] = 1.0
    p = m / n
    want = (1 - 2 * p) / math.sqrt(p * (1 - p)) * math.sqrt(n * (n - 1)) / (n - 2)
    assert O.skewness(x) == pytest.approx(want, rel=1e-12)


def test_skewness_invariances_and_degenerate_cases():
    rng = np.random.default_rng(21)
    x = rng.gamma(0.5, size=300)
    assert O.skewness(3.5 * x + 2.0) == pytest.approx(O.skewness(x), rel=1e-9)
    assert O.skewness(-x) == pytest.approx(-O.skewness(x), rel=1e-12)
    assert O.skewness(np.full(10, 0.25)) == 0.0
    assert O.skewness(np.array([1.0, 2.0])) == 0.0


def test_skewness_zero_spread_is_taken_at_the_resolution_of_the_scores():
    # Eq.10 at sigma -> 0 (reading: 0).  A constant row must give 0 whatever its value and length: the mean of
    # n equal values is not that value in floating point for most values, and an exact "sigma > 0" test then
    # returns +-1 (the skewness of n copies of one rounding error)
    for n in (3, 576, 1000, 2304, 7290, 16384):
        for val in (0.9 / n, 0.37 / n, 1.0 / 3.0, 1e-30):
            assert O.skewness(np.full(n, val)) == 0.0
    # spreads below 1e-6 of the mean are zero spread; above it the definition applies unchanged
    rng = np.random.default_rng(23)
    base = 0.9 / 7290
    noise = rng.standard_normal(7290)
    for rel in (1e-12, 1e-9, 1e-7):
        assert O.skewness(base * (1.0 + rel * noise)) == 0.0
    for rel in (1e-5, 1e-3, 1e-1):
        x = base * (1.0 + rel * rng.exponential(size=7290))
        assert O.skewness(x) == pytest.approx(scipy.stats.skew(x, bias=False), rel=1e-6)
        assert O.skewness(x) > 1.0  # an exponential tail: the skewness is 2 in the limit, and it is not cut off


def test_identical_visual_keys_give_uniform_importance_and_zero_skewness():
    # all visual keys equal: every row of Eq.7 spreads its visual mass evenly, I_v = s_t / N_v, Eq.10 -> 0
    rng = np.random.default_rng(24)
    d, hq, hkv, ns, nv, nt = 32, 4, 2, 3, 700, 12
    k = rng.standard_normal((hkv, ns + nv + nt, d))
    k[:, ns:ns + nv] = k[:, ns:ns + 1]
    q = rng.standard_normal((hq, nt, d))
    seg = O.Segments(ns + nv + nt, ns, nv, ns + nv, nt)
    imp, _ = O.layer_importance(q, k, seg, 0.9)
    s_t, s_k = O.layer_stats(imp)
    assert s_k == 0.0
    assert 0.0 < s_t < 1.0
    np.testing.assert_allclose(imp, np.broadcast_to(imp.sum(axis=1, keepdims=True) / nv, imp.shape), rtol=1e-12)


def test_layer_stats_is_mean_over_kv_heads():
    rng = np.random.default_rng(22)
    imp = rng.gamma(0.4, size=(3, 40)) / 100
    s_t, s_k = O.layer_stats(imp)
    assert s_t == pytest.approx(imp.sum() / 3, rel=1e-13)
    assert s_k == pytest.approx(np.mean([scipy.stats.skew(r, bias=False) for r in imp]), rel=1e-10)


# ---------------------------------------------------------------------------
# Eq.11 / budgets
# ---------------------------------------------------------------------------
def test_budget_hand_worked_cases():
    # shares a = b = [.25, .75]; K_tot = round(0.1*100*2) = 20
    assert O.layer_budgets([0.2, 0.6], [1.0, 3.0], 0.10, 100) == [5, 15]
    # r_hat_l = (s'_t + s'_k)/2 * r with s' = L*share: layer 1 keeps N_v * r_hat = 100 * 1.5 * 0.1
    # lower clamp: x = [0.5, 9.5] -> layer 0 pinned at min_keep = 1, the rest to layer 1
    assert O.layer_budgets([0.05, 0.95], [0.05, 0.95], 0.5, 10) == [1, 9]
    # upper clamp: K_tot = 18, x = [4.5, 13.5] -> layer 1 pinned at N_v = 10, layer 0 gets 8
    assert O.layer_budgets([0.25, 0.75], [0.25, 0.75], 0.9, 10) == [8, 10]
    # largest remainder, ties to the lower layer: 10 tokens over three equal layers
    assert O.layer_budgets([1, 1, 1], [1, 1, 1], 10 / 300, 100) == [4, 3, 3]
    # negative skewness is clamped to 0 before normalising: b = [0, 1], a = [.5, .5] -> w = [.25, .75]
    assert O.layer_budgets([0.5, 0.5], [-1.0, 2.0], 0.1, 100) == [5, 15]
    # mixed strength and skew: a = [.5,.5], b = [.2,.8] -> w = [.35,.65]; K_tot = 40
    assert O.layer_budgets([0.3, 0.3], [1.0, 4.0], 0.2, 100) == [14, 26]


def test_budget_hand_worked_fixture():
    # tests/golden/eq11_hand_worked.txt: allocations derived on paper from Eq.11 (the derivation is in the file)
    import os

    path = os.path.join(os.path.dirname(__file__), "golden", "eq11_hand_worked.txt")
    n = 0
    for line in open(path):
        if not line.strip() or line.startswith("#"):
            continue
        s_t, s_k, r, n_vis, min_keep, want, _ = [f.strip() for f in line.split("|")]
        got = O.layer_budgets([float(x) for x in s_t.split(",")], [float(x) for x in s_k.split(",")], float(r), int(n_vis),
                              O.BUDGET_STRENGTH_SKEW, int(min_keep))
        assert got == [int(x) for x in want.split(",")], line
        n += 1
    assert n == 10


def test_budget_modes():
    s_t, s_k = [0.1, 0.3], [3.0, 1.0]
    assert O.layer_budgets(s_t, s_k, 0.1, 100, O.BUDGET_UNIFORM) == [10, 10]
    assert O.layer_budgets(s_t, s_k, 0.1, 100, O.BUDGET_STRENGTH) == [5, 15]
    assert O.layer_budgets(s_t, s_k, 0.1, 100, O.BUDGET_SKEW) == [15, 5]
    assert O.layer_budgets(s_t, s_k, 0.1, 100, O.BUDGET_STRENGTH_SKEW) == [10, 10]


def test_budget_invariants_random():
    rng = np.random.default_rng(30)
    for trial in range(300):
        L = int(rng.integers(1, 40))
        n_vis = int(rng.integers(1, 3000))
        r = float(rng.choice([0.01, 0.05, 0.1, 0.25, 0.5, 0.9, 1.0]))
        min_keep = int(rng.integers(0, 4))
        s_t = rng.uniform(0.01, 1.0, L) ** 3
        s_k = rng.normal(5, 8, L)
        k = O.layer_budgets(list(s_t), list(s_k), r, n_vis, min_keep=min_keep)
        k_tot = O.total_budget(r, n_vis, L, min_keep)
        assert sum(k) == k_tot
        assert all(min(min_keep, n_vis) <= x <= n_vis for x in k)
        if r == 1.0:
            assert k == [n_vis] * L


def test_budget_total_rounding():
    assert O.total_budget(0.10, 7290, 28) == 20412
    assert O.total_budget(0.10, 576, 2) == 115      # 115.2 -> 115
    assert O.total_budget(0.05, 2305, 28) == 3227   # 3227.0
    assert O.total_budget(0.001, 100, 4, min_keep=1) == 4  # floor is min_keep per layer
    assert O.total_budget(0.001, 100, 4, min_keep=0) == 0


def test_budget_identical_layers_and_monotonicity():
    k = O.layer_budgets([0.4] * 7, [2.0] * 7, 0.1, 1000)
    assert sum(k) == 700 and max(k) - min(k) <= 1
    rng = np.random.default_rng(31)
    for trial in range(100):
        L = int(rng.integers(2, 20))
        s_t = list(rng.uniform(0.05, 1.0, L))
        s_k = list(rng.uniform(0.0, 20.0, L))
        base = O.layer_budgets(s_t, s_k, 0.1, 2000)
        l = int(rng.integers(0, L))
        s_t2 = list(s_t)
        s_t2[l] *= 1.5
        assert O.layer_budgets(s_t2, s_k, 0.1, 2000)[l] >= base[l]


def test_budget_proportionality_without_clamps():
    # with no clamp active every k_l is within one token of w_l * K_tot
    rng = np.random.default_rng(32)
    s_t = list(rng.uniform(0.2, 0.9, 28))
    s_k = list(rng.uniform(5, 30, 28))
    w = O.layer_weights(s_t, s_k)
    assert sum(w) == pytest.approx(1.0, abs=1e-12)
    k = O.layer_budgets(s_t, s_k, 0.1, 7290)
    for kl, wl in zip(k, w):
        assert abs(kl - wl * 20412) < 1.0


# ---------------------------------------------------------------------------
# top-k and compaction
# ---------------------------------------------------------------------------
def test_topk_brute_force_and_ties():
    rng = np.random.default_rng(40)
    for trial in range(200):
        n = int(rng.integers(1, 60))
        x = rng.integers(0, 8, size=n).astype(np.float64) / 8  # many ties
        k = int(rng.integers(0, n + 1))
        want = sorted(sorted(range(n), key=lambda i: (-x[i], i))[:k])
        assert O.select_topk(x, k).tolist() == want
    x = np.array([0.5, 0.9, 0.5, 0.9, 0.1])
    assert O.select_topk(x, 3).tolist() == [0, 1, 3]  # tie between 0 and 2 -> lower index
    assert O.select_topk(x, 5).tolist() == [0, 1, 2, 3, 4]
    assert O.select_topk(x, 0).tolist() == []


def test_compaction_keeps_system_and_text_and_copies_rows():
    rng = np.random.default_rng(41)
    seg = _seg(3, 10, 4)
    k = rng.standard_normal((seg.seq_len, 5))
    v = rng.standard_normal((seg.seq_len, 5))
    idx = np.array([1, 4, 9])
    rows = O.compact_rows(seg, idx)
    assert rows.tolist() == [0, 1, 2, 4, 7, 12, 13, 14, 15, 16]
    kc, vc = O.compact(k, v, seg, idx)
    assert np.array_equal(kc, k[rows]) and np.array_equal(vc, v[rows])


# ---------------------------------------------------------------------------
# decode attention
# ---------------------------------------------------------------------------
def test_decode_attn_matches_torch_sdpa():
    rng = np.random.default_rng(50)
    hq, hkv, t, d = 6, 2, 37, 16
    q = rng.standard_normal((hq, d))
    kc = [rng.standard_normal((t, d)) for _ in range(hkv)]
    vc = [rng.standard_normal((t, d)) for _ in range(hkv)]
    got = O.decode_layer(q, kc, vc)
    tq = torch.from_numpy(q)[None, :, None, :]
    tk = torch.from_numpy(np.stack(kc))[None].repeat_interleave(hq // hkv, dim=1)
    tv = torch.from_numpy(np.stack(vc))[None].repeat_interleave(hq // hkv, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0].numpy()
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_decode_single_key_returns_value_and_full_retention_is_identity():
    rng = np.random.default_rng(51)
    q = rng.standard_normal((3, 8))
    k1, v1 = rng.standard_normal((1, 8)), rng.standard_normal((1, 8))
    np.testing.assert_allclose(O.decode_attn(q, k1, v1), np.repeat(v1, 3, axis=0), rtol=1e-14)
    seg = _seg(2, 9, 3)
    k = rng.standard_normal((seg.seq_len, 8))
    v = rng.standard_normal((seg.seq_len, 8))
    kc, vc = O.compact(k, v, seg, O.select_topk(rng.random(9), 9))
    assert np.array_equal(kc, k) and np.array_equal(vc, v)
    assert np.array_equal(O.decode_attn(q, kc, vc), O.decode_attn(q, k, v))


# ---------------------------------------------------------------------------
# whole method on a planted example
# ---------------------------------------------------------------------------
def test_compress_sequence_recovers_planted_salient_tokens():
    """Keys aligned with the text queries must be the ones kept; the layer with the sharper head
    effect and the larger visual mass must get the larger budget."""
    rng = np.random.default_rng(60)
    hq, hkv, d, n_vis, n_text = 4, 2, 16, 200, 6
    seg = _seg(2, n_vis, n_text)
    u = np.zeros(d)
    u[0] = 1.0
    planted = [np.sort(rng.choice(n_vis, c, replace=False)) for c in (5, 60)]
    q_layers, k_layers = [], []
    for l, boost in enumerate((8.0, 2.0)):
        k = rng.standard_normal((hkv, seg.seq_len, d)) * 0.1
        k[:, seg.vis_start + planted[l]] += boost * u
        k[:, seg.text_start:] += (0.0 if l == 0 else 3.0) * u  # layer 1 looks at its text keys instead
        q = rng.standard_normal((hq, n_text, d)) * 0.1 + 4.0 * u
        q_layers.append(q)
        k_layers.append(k)
    res = O.compress_sequence(q_layers, k_layers, seg, 0.9, 0.2)
    assert sum(res.budgets) == 80
    assert res.s_t[0] > res.s_t[1] and res.s_k[0] > res.s_k[1]
    assert res.budgets[0] > res.budgets[1]
    for h in range(hkv):
        assert set(planted[0]).issubset(set(res.indices[0][h]))   # 5 planted, more than 5 kept
        assert set(res.indices[1][h]).issubset(set(planted[1]))   # 60 planted, fewer kept
        assert len(res.indices[0][h]) == res.budgets[0]
        assert np.all(np.diff(res.indices[1][h]) > 0)


def test_oracle_answer_for_the_tiny_workload_has_not_drifted():
    # tests/golden/tiny_pipeline.txt is written by tests/golden/make_tiny_pipeline.py from the oracle alone;
    # it guards the oracle against unintended changes (it is not a pin against the paper, which prints no example)
    import importlib.util
    import os

    here = os.path.join(os.path.dirname(__file__), "golden")
    spec = importlib.util.spec_from_file_location("make_tiny_pipeline", os.path.join(here, "make_tiny_pipeline.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = open(os.path.join(here, "tiny_pipeline.txt")).read().splitlines()
    now = mod.tiny_pipeline_lines()
    assert len(stored) == len(now)
    for a, b in zip(stored, now):
        ta, tb = a.split(), b.split()
        assert len(ta) == len(tb), (a, b)
        for x, y in zip(ta, tb):
            if ":" in x and "e" in x:  # index:score pairs
                assert x.split(":")[0] == y.split(":")[0], (a, b)
                assert float(x.split(":")[1]) == pytest.approx(float(y.split(":")[1]), rel=1e-10), (a, b)
            elif "e-" in x or "e+" in x:
                assert float(x) == pytest.approx(float(y), rel=1e-10), (a, b)
            else:
                assert x == y, (a, b)

