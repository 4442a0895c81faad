"""HIP path vs CPU oracle, stage by stage, on the same seeded inputs (through the C ABI)."""
import gc

import numpy as np
import pytest

import synth
from oracle import aircache_oracle as O
from tests import parity_util as P

pytestmark = pytest.mark.gpu


def _run_case(w, retention, *, alpha=None, steps=2, layer_chunk=None, token_major=False, budget_mode=0,
              min_keep=1, check_decode_units=None, verbose=True, visual_window=None, tuning=None, oracle_steps=None,
              causal_text=False):
    """Full pipeline on the GPU, checked stage by stage against the oracle.

    Stages after the budget are fed the oracle's budgets when the GPU's differ from them (the
    difference itself is checked separately), so that every stage is compared on equal inputs.

    visual_window = (first, length): the visual observation window of the ablation table; the span
    starts `first` tokens into the visual span (negative: counted from its end).  The generator has no
    queries for visual tokens, so the first `length` rows of its text queries stand in for them.
    """
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device, to_host

    dev = torch.device("cuda:0")
    alpha = w.alpha if alpha is None else alpha
    seqs = w.seqs()
    if visual_window is not None:
        import dataclasses
        first, length = visual_window
        assert all(length <= s.n_text and length <= s.vis_len for s in seqs)
        seqs = [dataclasses.replace(s, win_start=s.vis_start + (first if first >= 0 else s.vis_len + first), win_len=length)
                for s in seqs]
        alpha = 0.0
    L, B, Hkv, G, d = w.n_layers, w.batch, w.n_kv_heads, w.group, w.head_dim
    cfg = config_for(w, retention, alpha=alpha, budget_mode=budget_mode, min_keep=min_keep, max_decode_steps=max(steps, 1),
                     seqs=seqs, window_kind=0 if visual_window is None else A.AIR_WINDOW_VISUAL, causal_text=int(causal_text))
    ac = A.AirCache(cfg, dev)
    if tuning:
        ac.air_set_tuning(**tuning)  # launch shapes the library would not pick for this size by itself
    tag = f"[{w.name} r={retention} alpha={alpha}]"

    # ---- inputs: generate layer by layer, upload, run the oracle's first loop on the host copy
    q_dev, k_dev, v_dev, host_kv = [], [], [], []
    orc = P.OracleRun()
    s_t = np.zeros((B, L))
    s_k = np.zeros((B, L))
    for l in range(L):
        li = synth.layer_inputs(w, l, seqs)
        if token_major:  # [B][T][H][d] memory order, indexed as [B][H][T][d] through strides
            q_dev.append(to_device(np.ascontiguousarray(li.q_text.transpose(0, 2, 1, 3)), dev).permute(0, 2, 1, 3))
            k_dev.append(to_device(np.ascontiguousarray(li.k.transpose(0, 2, 1, 3)), dev).permute(0, 2, 1, 3))
            v_dev.append(to_device(np.ascontiguousarray(li.v.transpose(0, 2, 1, 3)), dev).permute(0, 2, 1, 3))
        else:
            q_dev.append(to_device(li.q_text, dev))
            k_dev.append(to_device(li.k, dev))
            v_dev.append(to_device(li.v, dev))
        if visual_window is None:
            sc, el, a, c = P.oracle_score_layer(w, li, seqs, alpha, causal_text)
        else:
            sc, el, a, c = P.oracle_score_layer_visual_window(w, li.q_text, li, seqs)
        orc.scores.append(sc)
        orc.elites.append(el)
        s_t[:, l] = a
        s_k[:, l] = c
        host_kv.append((li.k, li.v))
    orc.s_t, orc.s_k = s_t, s_k
    orc.budgets = P.oracle_budgets(s_t, s_k, seqs, retention, budget_mode, min_keep)

    # ---- air_score
    chunk = layer_chunk or L
    for l0 in range(0, L, chunk):
        l1 = min(L, l0 + chunk)
        ac.air_score(l0, l1, q_dev[l0:l1], k_dev[l0:l1], v_dev[l0:l1], seqs)
    worst = 0.0
    for l in range(L):
        cnt, idx = ac.air_get_elite(l)
        P.check_elite(cnt, idx, orc.elites[l], f"{tag} layer {l}")
        worst = max(worst, P.check_scores(ac.air_get_scores(l), orc.scores[l], seqs, f"{tag} layer {l}"))

    # ---- air_budget
    ac.air_budget()
    g_st, g_sk = ac.air_get_stats()
    np.testing.assert_allclose(g_st, s_t, rtol=P.STAT_RTOL, err_msg=f"{tag} strength")
    np.testing.assert_allclose(g_sk, s_k, rtol=P.STAT_RTOL, atol=1e-9, err_msg=f"{tag} skewness")
    g_bud = ac.air_get_budgets()
    # integer work is bit-exact given the same statistics
    same_stats = P.oracle_budgets(g_st, g_sk, seqs, retention, budget_mode, min_keep)
    assert np.array_equal(g_bud, same_stats), f"{tag} budgets differ from the oracle's allocation of the GPU's own statistics"
    assert np.array_equal(g_bud.sum(axis=1), orc.budgets.sum(axis=1))
    budget_moves = int(np.abs(g_bud - orc.budgets).sum())
    assert np.abs(g_bud - orc.budgets).max() <= 1, f"{tag} budgets off by more than one token: {g_bud - orc.budgets}"
    if budget_moves:
        ac.air_set_budgets(orc.budgets)
    bud = orc.budgets

    # ---- air_select_compact
    for l0 in range(0, L, chunk):
        l1 = min(L, l0 + chunk)
        ac.air_select_compact(l0, l1, k_dev[l0:l1], v_dev[l0:l1])
    swaps = 0
    gpu_idx = []
    for l in range(L):
        gi = ac.air_get_indices(l)
        gpu_idx.append(gi)
        for b in range(B):
            for h in range(Hkv):
                swaps += P.check_selection(gi[b, h, : bud[b, l]], orc.scores[l][b][h], int(bud[b, l]),
                                           f"{tag} layer {l} b={b} kv={h}")
    lens = ac.air_get_lengths()
    for b, s in enumerate(seqs):
        assert np.array_equal(lens[b], (s.seq_len - s.vis_len) + bud[b])

    # compaction: rows bit-identical to the source rows of [system ; kept ; text]
    units = check_decode_units or [(l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)]
    caches = {}
    for (l, b, h) in units:
        s = seqs[b]
        rows = O.compact_rows(P.seg_of(s), gpu_idx[l][b, h, : bud[b, l]])
        kk, vv = ac.air_get_cache(l, b, h, len(rows))
        hk, hv = host_kv[l]
        assert np.array_equal(kk, hk[b, h][rows]), f"{tag} K' rows differ at layer {l} b={b} kv={h}"
        assert np.array_equal(vv, hv[b, h][rows]), f"{tag} V' rows differ at layer {l} b={b} kv={h}"
        caches[(l, b, h)] = (synth.storage_to_f64(kk), synth.storage_to_f64(vv))

    # ---- air_decode_attn: every step runs on the GPU; the oracle is consulted on `oracle_steps` (default: all),
    # its cache rebuilt from the compacted rows plus every token appended so far (Eq.2)
    worst_dec = 0.0
    out = torch.empty((L, B, w.n_q_heads, d), dtype=q_dev[0].dtype, device=dev)
    check_at = set(range(steps)) if oracle_steps is None else set(oracle_steps)
    assert all(0 <= t < steps for t in check_at)
    for step in range(steps):
        qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
        qn, kn, vn = np.stack(qs), np.stack(ks), np.stack(vs)
        dq, dk, dv = to_device(qn, dev), to_device(kn, dev), to_device(vn, dev)
        for l0 in range(0, L, chunk):
            l1 = min(L, l0 + chunk)
            ac.air_decode_attn(l0, l1, dq[l0:l1], dk[l0:l1], dv[l0:l1], out[l0:l1])
        k64, v64 = synth.storage_to_f64(kn), synth.storage_to_f64(vn)
        for (l, b, h) in units:
            kc, vc = caches[(l, b, h)]
            if isinstance(kc, np.ndarray):  # compacted rows first, appended rows after them, joined when needed
                kc, vc = [kc], [vc]
            kc.append(k64[l, b, h][None])  # Eq.2
            vc.append(v64[l, b, h][None])
            caches[(l, b, h)] = (kc, vc)
        if step not in check_at:
            continue
        got = synth.storage_to_f64(to_host(out))
        assert not np.any(np.isnan(got))
        q64 = synth.storage_to_f64(qn)
        for (l, b, h) in units:
            kc, vc = caches[(l, b, h)]
            kc, vc = [np.concatenate(kc)], [np.concatenate(vc)]
            caches[(l, b, h)] = (kc, vc)
            want = O.decode_attn(q64[l, b, h * G:(h + 1) * G], kc[0], vc[0])
            err = np.abs(got[l, b, h * G:(h + 1) * G] - want).max()
            worst_dec = max(worst_dec, float(err))
            assert err <= P.DECODE_ATOL[w.dtype], f"{tag} decode step {step} layer {l} b={b} kv={h}: abs err {err:.3g}"
    for key, (kc, vc) in caches.items():
        if not isinstance(kc, np.ndarray):
            caches[key] = (np.concatenate(kc), np.concatenate(vc))
    if steps:
        lens2 = ac.air_get_lengths()
        assert np.array_equal(lens2, lens + steps)
        (l, b, h) = units[-1]
        kk, vv = ac.air_get_cache(l, b, h, int(lens2[b, l]))
        assert np.array_equal(synth.storage_to_f64(kk), caches[(l, b, h)][0]), "appended K rows differ"
        assert np.array_equal(synth.storage_to_f64(vv), caches[(l, b, h)][1]), "appended V rows differ"
    if verbose:
        print(f"{tag} worst score rel err {worst:.2e}; budget moves {budget_moves}; tolerated swaps {swaps}; "
              f"worst decode abs err {worst_dec:.2e}", flush=True)
    ac.close()
    del ac, q_dev, k_dev, v_dev
    gc.collect()
    torch.cuda.empty_cache()
    return dict(score_err=worst, budget_moves=budget_moves, swaps=swaps, decode_err=worst_dec, budgets=bud,
                vis_len=[s.vis_len for s in seqs])


def test_config1_tiny_fp32_elite_window():
    _run_case(synth.get_workload(1), 0.10, alpha=0.9, steps=1)


def test_config1_tiny_fp32_continuous_window():
    # the last-16 continuous observation window of Tab.5: alpha = 0 keeps the whole candidate span
    _run_case(synth.get_workload(1), 0.10, alpha=0.0, steps=1)


@pytest.mark.parametrize("retention", [0.01, 0.10, 0.50, 1.00])
def test_small_bf16_retention_sweep(retention):
    # several key chunks and a ragged tail (1500 = 5*256 + 220), G = 7, 3 layers
    w = synth.get_workload(2).scaled(n_layers=3, n_vis=1500, n_text=40, decode_steps=3)
    _run_case(w, retention, steps=3)


def test_small_ragged_batch_token_major_layout():
    w = synth.get_workload(3).scaled(batch=3, n_layers=2, n_vis=700, n_text=48)
    _run_case(w, 0.10, steps=2, token_major=True)


def test_layer_chunked_calls_match():
    w = synth.get_workload(2).scaled(n_layers=5, n_vis=600, n_text=32)
    _run_case(w, 0.25, steps=2, layer_chunk=2)


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_budget_modes(mode):
    w = synth.get_workload(2).scaled(n_layers=6, n_vis=520, n_text=24)
    _run_case(w, 0.10, steps=0, budget_mode=mode)


def test_all_text_window_alpha_zero():
    # every text token is a window row (Tab.5 "all text tokens"): many rows per head
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=520, n_text=24)
    _run_case(w, 0.10, alpha=0.0, steps=1)


@pytest.mark.parametrize("first,length", [(-32, 32), (-4, 4), (200, 40), (0, 3)])
def test_visual_window_bf16(first, length):
    # "Visual window (32)" of the ablation table on the MFMA kernels: G * 32 rows take the recompute path,
    # G * 4 = 28 rows the stash path; a window in the middle of the span (200..239 of 1500, across no chunk
    # boundary but with five chunks wholly behind it) and one at its very start (rows that see 1-3 keys)
    # exercise the empty partials.  Eq.9 is 1 for every layer, so the budgets rest on the skewness alone.
    w = synth.get_workload(2).scaled(n_layers=3, n_vis=1500, n_text=48, decode_steps=1)
    r = _run_case(w, 0.10, steps=1, visual_window=(first, length))
    assert r["score_err"] <= P.SCORE_RTOL


def test_visual_window_across_a_chunk_boundary_and_ragged_batch():
    # rows 750 .. 773 of 780 straddle the chunk boundary at 768: the last chunk is empty for the first 18 rows
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=780, n_text=48, decode_steps=1)
    _run_case(w, 0.10, steps=1, visual_window=(-30, 24))
    # visual spans of different lengths in one batch
    w = synth.get_workload(3).scaled(batch=3, n_layers=2, n_vis=780, n_text=48)
    _run_case(w, 0.10, steps=1, visual_window=(-30, 24))


def test_visual_window_fp32_generic_path():
    _run_case(synth.get_workload(1), 0.10, steps=1, visual_window=(-16, 16))
    _run_case(synth.get_workload(1).scaled(n_vis=300), 0.10, steps=1, visual_window=(250, 12))


def test_one_token_at_a_time_harness_and_fixed_indices():
    """Sec.4.3, Fig.4 as a mechanism: keep only the visual token of importance rank j in every layer
    (budgets of 1, indices fixed by the caller), decode over [system ; that token ; text].  One layer keeps
    the library's own selection, to check that fixed and selected layers mix in one call."""
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device, to_host
    from paper_2503_23956_amd.diagnostics import importance_ranking, single_rank_indices

    dev = torch.device("cuda:0")
    w = synth.get_workload(2).scaled(n_layers=3, n_vis=700, n_text=32, decode_steps=1)
    seqs = w.seqs()
    L, B, Hkv, G, d = w.n_layers, w.batch, w.n_kv_heads, w.group, w.head_dim
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    oracle_imp = [P.oracle_score_layer(w, li, seqs, w.alpha)[0] for li in layers]  # [l][b] -> [H_kv][vis_len]
    qs, ks, vs = zip(*[synth.decode_inputs(w, l, 0) for l in range(L)])
    qn, kn, vn = np.stack(qs), np.stack(ks), np.stack(vs)
    ac = A.AirCache(config_for(w, 0.10, max_decode_steps=1, seqs=seqs), dev)
    for rank in (0, 1, 7, 699):
        ac.air_reset()
        ac.air_score(0, L, q, k, v, seqs)
        ac.air_budget()
        ac.air_set_budgets(np.ones((B, L), dtype=np.int32))
        want_tok = np.zeros((L, B, Hkv), dtype=np.int64)
        for l in range(L):
            for b in range(B):
                for h in range(Hkv):  # the oracle's token of this rank: its top-(j+1) set minus its top-j set
                    imp = oracle_imp[l][b][h]
                    (tok,) = set(O.select_topk(imp, rank + 1).tolist()) - set(O.select_topk(imp, rank).tolist())
                    want_tok[l, b, h] = tok
            if l != 1:  # layer 1 is left to the library's own top-1 selection
                idx = np.zeros((B, Hkv, ac.cfg.max_vis_len), dtype=np.int32)
                idx[:, :, 0] = want_tok[l]
                ac.air_set_indices(l, idx)
            if rank < 2:  # well-separated ranks: the GPU's scores rank the same token there
                got = single_rank_indices(ac.air_get_scores(l), [s.vis_len for s in seqs], rank)
                assert np.array_equal(got[:, :, 0], want_tok[l])
        ac.air_select_compact(0, L, k, v)
        out = torch.empty((L, B, w.n_q_heads, d), dtype=q[0].dtype, device=dev)
        ac.air_decode_attn(0, L, to_device(qn, dev), to_device(kn, dev), to_device(vn, dev), out)
        got_out = synth.storage_to_f64(to_host(out))
        for l in range(L):
            gi = ac.air_get_indices(l)
            for b, s in enumerate(seqs):
                for h in range(Hkv):
                    tok = int(want_tok[l, b, h]) if l != 1 else int(O.select_topk(oracle_imp[l][b][h], 1)[0])
                    assert gi[b, h, 0] == tok
                    rows = O.compact_rows(P.seg_of(s), np.array([tok]))
                    kk, vv = ac.air_get_cache(l, b, h, len(rows) + 1)  # the decode step has appended one row
                    assert np.array_equal(kk[:-1], layers[l].k[b, h][rows]) and np.array_equal(vv[:-1], layers[l].v[b, h][rows])
                    assert np.array_equal(kk[-1], kn[l, b, h]) and np.array_equal(vv[-1], vn[l, b, h])
                    kc, vc = synth.storage_to_f64(kk), synth.storage_to_f64(vv)
                    want = O.decode_attn(synth.storage_to_f64(qn[l, b, h * G:(h + 1) * G]), kc, vc)
                    assert np.abs(got_out[l, b, h * G:(h + 1) * G] - want).max() <= P.DECODE_ATOL[w.dtype]
    # misuse is caught on the host
    ac.air_reset()
    ac.air_score(0, L, q, k, v, seqs)
    with pytest.raises(A.AirError) as e:
        ac.air_set_indices(0, np.zeros((B, Hkv, ac.cfg.max_vis_len), dtype=np.int32))  # no budgets yet
    assert e.value.status == A.binding.AIR_ERR_STATE
    ac.air_budget()
    bad = np.zeros((B, Hkv, ac.cfg.max_vis_len), dtype=np.int32)  # budgets > 1: zeros are not ascending
    with pytest.raises(A.AirError) as e:
        ac.air_set_indices(0, bad)
    assert e.value.status == A.binding.AIR_ERR_INVALID_ARG
    bad[:, :, :] = np.arange(ac.cfg.max_vis_len) + 699  # ascending, but the second entry is past the visual span
    with pytest.raises(A.AirError) as e:
        ac.air_set_indices(0, bad)
    assert e.value.status == A.binding.AIR_ERR_INVALID_ARG
    ac.close()


def test_generic_path_other_storage_combinations():
    # the fp32-ALU kernels serve every storage type / head_dim pair that the MFMA kernels do not:
    # fp32 with head_dim 128, bf16 with head_dim 64 (G = 7, several key chunks, decode across a split)
    _run_case(synth.get_workload(1).scaled(head_dim=128), 0.10, alpha=0.9, steps=2)
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=700, n_text=40, head_dim=64, decode_steps=3)
    _run_case(w, 0.10, steps=3)


def test_all_text_window_with_more_rows_than_one_staging_round():
    # 7 heads x 160 text tokens = 1120 window rows per unit: the finish kernel stages its row parameters
    # in rounds of 512, and the elite-text block of Eq.7 is 160 x 160 per head
    w = synth.get_workload(2).scaled(n_layers=1, n_vis=600, n_text=160, decode_steps=1)
    _run_case(w, 0.10, alpha=0.0, steps=1)


def test_elite_window_row_parameters_by_their_own_kernel():
    """The elite window's row parameters are formed inside the finish kernel; the separate row-parameter
    kernel (the path of the windows that turn their whole span into rows) must give the same on it, with the
    rows in the stash (alpha 0.9) and beyond it (alpha 0.05: most text tokens are elite)."""
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=1100, n_text=48, decode_steps=1)
    _run_case(w, 0.10, steps=1, tuning=dict(score_rows_kernel=1))
    _run_case(w, 0.10, alpha=0.05, steps=1, tuning=dict(score_rows_kernel=1))


def test_elite_window_with_more_rows_than_the_stash_holds():
    # a low threshold makes most text tokens elite: the finish kernel recomputes the logits and forms the
    # parameters of several hundred rows itself
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=1100, n_text=48, decode_steps=1)
    _run_case(w, 0.10, alpha=0.05, steps=1)


@pytest.mark.parametrize("case", ["elite_few_rows", "low_threshold", "continuous_16", "all_text", "fp32_elite", "fp32_continuous"])
def test_causal_mask_over_the_elite_text_keys(case):
    """Eq.7 with the optional causal mask (an elite row sees the elite text keys at or before its position only):
    one tile of rows, rows beyond the stash, more than 16 rows per head (two passes over the key tiles), and the
    generic kernels with up to 8 and with more elite rows per head."""
    if case in ("fp32_elite", "fp32_continuous"):
        _run_case(synth.get_workload(1), 0.10, alpha=0.9 if case == "fp32_elite" else 0.0, steps=1, causal_text=True)
        return
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=1100, n_text=48, decode_steps=1)
    if case == "elite_few_rows":
        _run_case(w, 0.10, alpha=0.5, steps=1, causal_text=True)
    elif case == "low_threshold":
        _run_case(w, 0.10, alpha=0.05, steps=1, causal_text=True)
    elif case == "continuous_16":
        import dataclasses
        _run_case(dataclasses.replace(w, window=16), 0.10, alpha=0.0, steps=1, causal_text=True)
    else:
        _run_case(w, 0.10, alpha=0.0, steps=1, causal_text=True)


def test_unified_span_without_a_modality_distinction():
    """The unified variant of the paper's vision-only / unified comparison (Sec.4.3): every prompt token in
    front of the observation window is a candidate.  Nothing in the path looks at a token's modality, so
    the variant is a sequence descriptor whose compressible span starts at token 0 and ends where the
    window starts (no system tokens, the whole text span as the window)."""
    w = synth.get_workload(2).scaled(n_layers=2, n_sys=0, n_vis=1500, n_text=48, window=0, decode_steps=2)
    s = w.seqs()[0]
    assert s.vis_start == 0 and s.vis_start + s.vis_len == s.win_start and s.win_start + s.win_len == s.seq_len
    _run_case(w, 0.25, steps=2)             # elite rows of the window
    _run_case(w, 0.10, alpha=0.0, steps=1)  # every window token a row, as the continuous-window baselines do


def test_degenerate_sizes():
    # fewer than three visual tokens (skewness 0), one text token, one-token window, min_keep 0
    w = synth.get_workload(1).scaled(n_vis=2, n_text=1, window=1, n_sys=1)
    _run_case(w, 0.5, steps=1, min_keep=0)
    w = synth.get_workload(1).scaled(n_vis=257, n_text=3, window=2, n_sys=0)
    _run_case(w, 0.02, steps=1)


def test_degenerate_sizes_bf16_mfma_path():
    # the same degenerate shapes on the bf16 / head_dim 128 kernels: a cache of a handful of rows that
    # grows through its first token block, one text token, fewer than three visual tokens
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=2, n_text=1, n_sys=1, decode_steps=40)
    _run_case(w, 0.5, steps=40, min_keep=0)
    w = synth.get_workload(2).scaled(n_layers=1, n_vis=33, n_text=2, n_sys=0, decode_steps=3)
    _run_case(w, 0.03, steps=3)


def test_decode_many_steps_cross_token_blocks():
    # appended tokens cross several 32-token block boundaries of the cache
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=300, n_text=21, decode_steps=70)
    _run_case(w, 0.10, steps=70)


def test_decode_long_cache_multiple_iterations_per_split():
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=3000, n_text=40, decode_steps=2)
    _run_case(w, 1.00, steps=2)


@pytest.mark.parametrize("splits,waves,tiles", [(4, 8, 4), (1, 2, 2), (2, 4, 2), (1, 1, 8), (16, 1, 4), (2, 2, 8), (1, 1, 4)])
def test_decode_forced_launch_shapes(splits, waves, tiles):
    # every compiled launch shape of the decode kernel (split-K exchange, 32-key double-buffered chunks,
    # 128-key chunks) against the oracle, with appends that cross token-block and split boundaries
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=900, n_text=37, decode_steps=36)
    _run_case(w, 0.25, steps=36, tuning=dict(decode_splits=splits, decode_waves=waves, decode_tiles=tiles))


@pytest.mark.parametrize("base,batch,n_layers,n_vis,retention", [(2, 1, 3, 900, 0.25), (2, 1, 2, 2600, 1.00), (2, 1, 5, 300, 0.05),
                                                                 (3, 3, 2, 1100, 0.25)])
def test_decode_column_halves(base, batch, n_layers, n_vis, retention):
    # two workgroups per unit, each with all of K' and one half of the columns of V' and of the output: against the
    # oracle (12, 20 and 24 units: a grid rounded up to whole groups of 16 workgroups; 8 units: an exact one; one sequence
    # and a ragged batch of three), with appends
    # that cross token blocks, and bit for bit against one workgroup per unit (same arithmetic per output column)
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device, to_host

    steps = 36
    w = synth.get_workload(base).scaled(batch=batch, n_layers=n_layers, n_vis=n_vis, n_text=37, decode_steps=steps)
    shape = dict(decode_splits=1, decode_waves=4, decode_tiles=4)
    _run_case(w, retention, steps=steps, oracle_steps=[0, 1, 31, 32, 35], tuning=dict(shape, decode_halves=2))
    dev = torch.device("cuda:0")
    seqs = w.seqs()
    L = w.n_layers
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q, k, v = ([to_device(getattr(li, name), dev) for li in layers] for name in ("q_text", "k", "v"))
    outs = []
    for halves in (1, 2):
        ac = A.AirCache(config_for(w, retention, seqs=seqs, max_decode_steps=steps), dev)
        ac.air_set_tuning(**shape, decode_halves=halves)
        ac.air_score(0, L, q, k, v, seqs)
        ac.air_budget()
        ac.air_select_compact(0, L, k, v)
        out = torch.empty((L, w.batch, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
        res = []
        for step in range(steps):
            qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
            ac.air_decode_attn(0, L, *(to_device(np.stack(x), dev) for x in (qs, ks, vs)), out)
            res.append(to_host(out).copy())
        lens = ac.air_get_lengths()
        res.append([ac.air_get_cache(l, b, h, int(lens[b, l])) for l in range(L) for b in range(w.batch) for h in range(w.n_kv_heads)])
        outs.append(res)
        ac.close()
    for step in range(steps):
        assert np.array_equal(outs[0][step].view(np.uint16), outs[1][step].view(np.uint16)), f"step {step}"
    for (k1, v1), (k2, v2) in zip(outs[0][steps], outs[1][steps]):
        assert np.array_equal(k1, k2) and np.array_equal(v1, v2)


def test_decode_longest_cache_first_after_caller_set_budgets():
    # budgets handed in by the caller (reversed per sequence, so that the order by length is not the order by layer)
    # go through the same layout code: the table by falling length must follow them
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device, to_host

    dev = torch.device("cuda:0")
    w = synth.get_workload(3).scaled(batch=2, n_layers=6, n_vis=1200, n_text=40, decode_steps=3)
    seqs = w.seqs()
    L = w.n_layers
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q, k, v = ([to_device(getattr(li, name), dev) for li in layers] for name in ("q_text", "k", "v"))
    outs = []
    for order in (1, 2):
        ac = A.AirCache(config_for(w, 0.20, seqs=seqs, max_decode_steps=3), dev)
        ac.air_set_tuning(decode_splits=1, decode_waves=4, decode_tiles=4, decode_order=order, decode_halves=1)
        ac.air_score(0, L, q, k, v, seqs)
        ac.air_budget()
        bud = ac.air_get_budgets()[:, ::-1].copy()
        assert len(set(bud[0].tolist())) > 1
        ac.air_set_budgets(bud)
        ac.air_select_compact(0, L, k, v)
        out = torch.empty((L, w.batch, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
        res = []
        for step in range(3):
            qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
            ac.air_decode_attn(0, L, *(to_device(np.stack(x), dev) for x in (qs, ks, vs)), out)
            res.append(to_host(out).copy())
        assert np.array_equal(ac.air_get_lengths(), bud + np.array([[s.seq_len - s.vis_len] for s in seqs]) + 3)
        outs.append(res)
        ac.close()
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


@pytest.mark.parametrize("waves", [1, 4])
def test_decode_longest_cache_first(waves):
    # a launch over all layers that takes its units by falling cache length (the table the budget kernel leaves,
    # also after caller-set budgets): ragged batch, layers of clearly different budgets, against the oracle
    w = synth.get_workload(3).scaled(batch=3, n_layers=5, n_vis=1500, n_text=40, decode_steps=34)
    _run_case(w, 0.20, steps=34, oracle_steps=[0, 1, 33],
              tuning=dict(decode_splits=1, decode_waves=waves, decode_tiles=4, decode_order=2))


@pytest.mark.parametrize("side", [+1, -1])
def test_elite_threshold_within_fp32_resolution_of_a_candidate(side):
    # Eq.5 with alpha placed a relative 1e-9 above / below exp(s_j - s_max) of a real candidate: fp32
    # logits cannot tell the two sides apart, so the kernel has to take the decision from its fp64
    # recomputation, and the elite sets must still equal the oracle's for every head
    w = synth.get_workload(2).scaled(n_layers=1, n_vis=300, n_text=48, decode_steps=1)
    seqs = w.seqs()
    s = seqs[0]
    li = synth.layer_inputs(w, 0, seqs)
    q = synth.storage_to_f64(li.q_text[0])
    k = synth.storage_to_f64(li.k[0])
    t0 = s.vis_start + s.vis_len
    logits = O.last_row_logits(q[0, s.win_start + s.win_len - 1 - t0], k[0, s.win_start:s.win_start + s.win_len])
    second = np.sort(logits)[-2]
    alpha = float(np.exp(second - logits.max()) * (1.0 + side * 1e-9))
    assert 0.0 < alpha < 1.0
    want = 1 if side > 0 else 2  # the runner-up of head 0 falls just outside / just inside
    assert len(O.elite_set(logits, alpha)) == want
    _run_case(w, 0.10, alpha=alpha, steps=0)


def test_topk_exact_ties_go_to_the_lower_index(monkeypatch):
    # Half of the visual keys are copies of the layer's most important key (one 256-key chunk, so the
    # copies' scores are equal bit for bit): the budget boundary falls inside the group of equal
    # scores, and the kept copies must be exactly the ones with the lowest token indices, as in the oracle
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=200, n_text=24, decode_steps=1)
    seqs = w.seqs()
    s = seqs[0]
    real = synth.layer_inputs

    def with_copies(wl, layer, sq=None):
        li = real(wl, layer, sq)
        imp = P.oracle_score_layer(wl, li, seqs, wl.alpha)[0][0]  # [H_kv][vis_len] of sequence 0
        src = s.vis_start + int(np.argmax(imp.sum(axis=0)))
        k, v = li.k.copy(), li.v.copy()
        for i in range(1, 200, 2):  # every odd visual position
            k[:, :, s.vis_start + i] = k[:, :, src]
            v[:, :, s.vis_start + i] = v[:, :, src]
        return type(li)(li.q_text, k, v)

    # the boundary does fall inside the tie group for at least one (layer, KV head)
    straddles = 0
    for layer in range(w.n_layers):
        imp = P.oracle_score_layer(w, with_copies(w, layer, seqs), seqs, w.alpha)[0][0]
        for h in range(w.n_kv_heads):
            kth = np.sort(imp[h])[-60]
            straddles += int(np.sum(imp[h] == kth) > 1 and np.sum(imp[h] > kth) < 60 < np.sum(imp[h] >= kth))
    assert straddles > 0
    monkeypatch.setattr(synth, "layer_inputs", with_copies)
    res = _run_case(w, 0.30, steps=1)
    assert res["swaps"] == 0


@pytest.mark.parametrize("cap", [0, 8])
def test_select_radix_fallback(cap):
    # the selection kernel ranks the deciding 12-bit bin directly when it is small; a cap of 0 (or one
    # that the bin exceeds) sends every row through the four radix passes instead
    w = synth.get_workload(2).scaled(n_layers=3, n_vis=5000, n_text=40, decode_steps=1)
    _run_case(w, 0.10, steps=1, tuning=dict(select_direct_max=cap))


@pytest.mark.parametrize("threads,n_vis,cap", [(256, 1500, None), (256, 9000, None), (256, 5000, 0), (512, 1500, None)])
def test_select_workgroup_sizes(threads, n_vis, cap):
    # both workgroup sizes of the selection kernel, whatever the launch would choose by itself: rows kept
    # in registers (1500, 5000 scores), a row walked in sweeps (9000 scores with 256 threads), the radix passes
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=n_vis, n_text=40, decode_steps=1)
    _run_case(w, 0.10, steps=1, tuning=dict(select_threads=threads, select_direct_max=-1 if cap is None else cap))


def test_maximum_candidate_span():
    # 4096 text tokens, the largest candidate span the boundary accepts: the elite kernel then keeps
    # the logits of one head at a time in LDS
    w = synth.get_workload(2).scaled(n_layers=1, n_vis=300, n_text=4096, decode_steps=1)
    _run_case(w, 0.10, steps=1)


def test_visual_span_beyond_one_selection_sweep():
    # 40000 visual tokens (a long video): the selection kernel walks the row in three sweeps of 16384
    # scores instead of keeping it in registers, and a window row has 157 chunk partials (more than one
    # per lane of the wave that combines them)
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=40000, n_text=32, decode_steps=2)
    units = [(0, 0, 0), (1, 0, w.n_kv_heads - 1)]
    _run_case(w, 0.05, steps=2, check_decode_units=units)


def test_maximum_batch():
    # 64 ragged sequences, the largest batch the boundary accepts (the sequence table travels as a kernel argument)
    w = synth.get_workload(3).scaled(batch=64, n_layers=2, n_vis=260, n_text=20, decode_steps=2)
    _run_case(w, 0.10, steps=2)


def test_more_units_per_layer_than_a_launch_of_32_layers_can_hold():
    # 64 sequences x 40 KV heads = 2560 units per layer: a grid dimension holds 25 layers of them, so the 27
    # layers go out in two launches per kernel (one query head per KV head on the way)
    w = synth.get_workload(3).scaled(batch=64, n_layers=27, n_q_heads=40, n_kv_heads=40, n_vis=40, n_text=4,
                                     decode_steps=1)
    units = [(0, 0, 0), (26, 63, 39), (25, 31, 7)]
    _run_case(w, 0.25, steps=1, check_decode_units=units, verbose=True)


def test_seeded_random_shapes():
    # a seeded sweep over other input seeds, sizes, batches, retentions and thresholds than the named cases use
    import dataclasses

    rng = np.random.default_rng(12345)
    for it in range(16):
        n_vis, n_text, L = int(rng.integers(200, 5000)), int(rng.integers(4, 200)), int(rng.integers(1, 5))
        ret = float(rng.choice([0.01, 0.05, 0.1, 0.25, 0.5, 1.0]))
        alpha = float(rng.choice([0.9, 0.9, 0.5, 0.99, 0.0]))
        base = int(rng.choice([2, 3]))
        B = 1 if base == 2 else int(rng.integers(1, 5))
        w = synth.get_workload(base).scaled(cfg_id=100 + it, batch=B, n_layers=L, n_vis=n_vis, n_text=n_text, decode_steps=3)
        if alpha == 0.0 and n_text > 64:
            w = dataclasses.replace(w, window=32)
        _run_case(w, ret, alpha=alpha, steps=3, verbose=False)


def test_budget_allocation_random_configurations():
    """Eq.11 with its clamps under seeded random depths, retentions, floors and allocation modes (the clamp at N_v
    at high retention, the floor at low retention with a large min_keep, both in one allocation): the budgets
    must be the oracle's allocation of the same statistics in every case."""
    rng = np.random.default_rng(4242)
    both_clamps = 0
    for it in range(24):
        base = int(rng.choice([1, 2]))
        n_vis, n_text, L = int(rng.integers(8, 700)), int(rng.integers(2, 40)), int(rng.integers(1, 20))
        ret = float(rng.choice([0.005, 0.02, 0.1, 0.3, 0.6, 0.9, 0.97, 1.0]))
        mode, min_keep = int(rng.integers(0, 4)), int(rng.choice([0, 1, 1, 5, 50]))
        B = int(rng.integers(1, 4))
        w = synth.get_workload(base).scaled(cfg_id=500 + it, batch=B, n_layers=L, n_vis=n_vis, n_text=n_text, window=0,
                                            decode_steps=1, jitter=0.2 if B > 1 else 0.0)
        r = _run_case(w, ret, steps=1, budget_mode=mode, min_keep=min_keep, verbose=False)
        for b, n in enumerate(r["vis_len"]):  # allocations in which some layers sit at N_v and others at the floor
            both_clamps += int(min_keep < n and np.any(r["budgets"][b] == n) and np.any(r["budgets"][b] == min(min_keep, n)))
    assert both_clamps >= 1
    # deeper than one wave has lanes: the workgroup-wide form of the allocation
    for L, ret, min_keep in ((70, 0.1, 1), (100, 0.97, 0), (129, 0.02, 5)):
        w = synth.get_workload(1).scaled(cfg_id=600 + L, n_layers=L, n_vis=96, n_text=6, window=0, decode_steps=1)
        _run_case(w, ret, steps=1, min_keep=min_keep, verbose=False)


def test_config2_full_size():
    _run_case(synth.get_workload(2), 0.10, steps=2)


def _sample_units(w, n, seed):
    rng = np.random.default_rng(seed)
    units = set()
    while len(units) < n:
        units.add((int(rng.integers(w.n_layers)), int(rng.integers(w.batch)), int(rng.integers(w.n_kv_heads))))
    return sorted(units)


def _spaced_steps(n):
    """First, last and six evenly spaced decode steps in between."""
    return sorted(set(int(round(i * (n - 1) / 7)) for i in range(8)))


@pytest.mark.parametrize("retention", [0.05, 0.10, 0.25])
def test_config3_batched_ragged_full_size(retention):
    # 16 ragged sequences; scores, budgets and index sets of every unit; compaction and decode on a sample of
    # units: all 256 steps run on the GPU, the oracle checks the first, the last and six spaced ones
    w = synth.get_workload(3)
    _run_case(w, retention, steps=w.decode_steps, oracle_steps=_spaced_steps(w.decode_steps),
              check_decode_units=_sample_units(w, 64, 3))


def test_config4_video_full_size():
    w = synth.get_workload(4)  # 512 decode steps
    _run_case(w, 0.10, steps=w.decode_steps, oracle_steps=_spaced_steps(w.decode_steps),
              check_decode_units=_sample_units(w, 48, 4))


def test_config5_72b_stress_full_size():
    # 80 layers (three launches per stage), G = 8, 16384 visual tokens (one full select sweep), 256 decode steps
    w = synth.get_workload(5)
    _run_case(w, 0.10, steps=w.decode_steps, oracle_steps=_spaced_steps(w.decode_steps),
              check_decode_units=_sample_units(w, 48, 5))


@pytest.mark.parametrize("retention", [0.01, 0.02, 0.05, 0.25, 0.50])
def test_config5_shape_retention_sweep(retention):
    # the other retentions of the 72B-shaped workload's sweep, on 6 of its layers at full width
    w = synth.get_workload(5).scaled(n_layers=6, decode_steps=40)
    _run_case(w, retention, steps=40, oracle_steps=[0, 1, 20, 39], check_decode_units=_sample_units(w, 24, 6))


def test_two_runs_give_bitwise_equal_results():
    """Same inputs, same outputs, bit for bit: scores, statistics, budgets, kept indices, cache rows and decode
    outputs of two independent contexts (the selection kernel counts with LDS atomics, whose order varies from
    run to run; nothing may depend on it).  A ragged batch, so that several launch paths take part."""
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device, to_host

    dev = torch.device("cuda:0")
    w = synth.get_workload(3).scaled(batch=3, n_layers=4, n_vis=2600, n_text=60, decode_steps=5)
    seqs = w.seqs()
    L, B, Hkv = w.n_layers, w.batch, w.n_kv_heads
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    dec = []
    for step in range(5):
        qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
        dec.append(tuple(to_device(np.stack(x), dev) for x in (qs, ks, vs)))

    def one_run(tuning):
        ac = A.AirCache(config_for(w, 0.10, seqs=seqs, max_decode_steps=5), dev)
        ac.air_set_tuning(**tuning)
        ac.air_score(0, L, q, k, v, seqs)
        ac.air_budget()
        ac.air_select_compact(0, L, k, v)
        res = dict(scores=[ac.air_get_scores(l) for l in range(L)], stats=ac.air_get_stats(), budgets=ac.air_get_budgets(),
                   indices=[], outs=[])
        bud = res["budgets"]
        for l in range(L):
            idx = ac.air_get_indices(l)
            res["indices"].append([idx[b, :, : bud[b, l]].copy() for b in range(B)])
        out = torch.empty((L, B, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
        for step in range(5):
            ac.air_decode_attn(0, L, *dec[step], out)
            res["outs"].append(to_host(out).copy())
        lens = ac.air_get_lengths()
        res["cache"] = [ac.air_get_cache(l, b, h, int(lens[b, l])) for l in (0, L - 1) for b in range(B) for h in (0, Hkv - 1)]
        ac.close()
        return res

    def same(a, b):
        if isinstance(a, (list, tuple)):
            return len(a) == len(b) and all(same(x, y) for x, y in zip(a, b))
        return np.array_equal(a.view(np.uint8) if a.dtype != np.uint8 else a, b.view(np.uint8) if b.dtype != np.uint8 else b)

    for tuning in (dict(), dict(decode_splits=4, decode_waves=4, decode_tiles=2), dict(select_direct_max=0, select_threads=256)):
        r1, r2 = one_run(tuning), one_run(tuning)
        for key in r1:
            assert same(r1[key], r2[key]), f"{key} differs between two runs ({tuning})"
    # the order in which a decode launch takes its units (by layer, or longest cache first) changes no bit either
    for waves in (1, 4):
        shape = dict(decode_splits=1, decode_waves=waves, decode_tiles=4)
        r1, r2 = one_run(dict(shape, decode_order=1)), one_run(dict(shape, decode_order=2))
        for key in r1:
            assert same(r1[key], r2[key]), f"{key} differs between the two unit orders ({waves} waves)"


def test_allocation_in_the_tail_of_scoring_equals_the_budget_kernel():
    """Up to 64 layers air_score's last kernel does Eq.11 itself (the last unit of a sequence to finish); beyond that,
    or with the tuning switch, air_budget launches the budget kernel.  Both must leave the same statistics, budgets
    and layout, also when the layers are scored in several calls, when a layer is scored twice (the kernel takes
    over) and when a prompt is dropped half-way (its partial arrival counts must not leak into the next one)."""
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device

    dev = torch.device("cuda:0")
    w = synth.get_workload(3).scaled(batch=3, n_layers=5, n_vis=1300, n_text=48, decode_steps=1)
    seqs = w.seqs()
    L = w.n_layers
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q, k, v = ([to_device(getattr(li, name), dev) for li in layers] for name in ("q_text", "k", "v"))

    def state(ac):
        ac.air_budget()
        ac.air_select_compact(0, L, k, v)  # the layout tables are what the gather and the lengths follow
        bud = ac.air_get_budgets()
        idx = [ac.air_get_indices(l) for l in range(L)]
        return dict(stats=ac.air_get_stats(), budgets=bud, lengths=ac.air_get_lengths(),
                    idx=[[idx[l][b, :, : bud[b, l]] for b in range(w.batch)] for l in range(L)])

    def same(a, b):
        for key in a:
            xs, ys = (a[key], b[key]) if isinstance(a[key], (list, tuple)) else ([a[key]], [b[key]])
            for x, y in zip(xs, ys):
                if isinstance(x, (list, tuple)):
                    assert all(np.array_equal(p, r) for p, r in zip(x, y)), key
                else:
                    assert np.array_equal(x, y), key

    ref = A.AirCache(config_for(w, 0.10, seqs=seqs, max_decode_steps=1), dev)
    ref.air_set_tuning(budget_in_score=1)
    ref.air_score(0, L, q, k, v, seqs)
    want = state(ref)
    ref.close()

    ac = A.AirCache(config_for(w, 0.10, seqs=seqs, max_decode_steps=1), dev)
    ac.air_score(0, L, q, k, v, seqs)  # all layers in one call
    same(want, state(ac))
    ac.air_reset()
    for l0, l1 in ((3, 5), (0, 1), (1, 3)):  # in pieces, out of order
        ac.air_score(l0, l1, q[l0:l1], k[l0:l1], v[l0:l1], seqs)
    same(want, state(ac))
    ac.air_reset()
    ac.air_score(0, L, q, k, v, seqs)
    ac.air_score(2, 3, q[2:3], k[2:3], v[2:3], seqs)  # a layer scored twice: the arrival count is off, the kernel takes over
    same(want, state(ac))
    ac.air_reset()
    ac.air_score(0, 2, q[:2], k[:2], v[:2], seqs)  # a prompt dropped after two layers
    ac.air_reset()
    ac.air_score(0, L, q, k, v, seqs)
    same(want, state(ac))
    ac.air_reset()
    ac.air_score(0, L, q, k, v, seqs)  # and the counters are back at zero after a complete pass
    same(want, state(ac))
    for _ in range(12):  # prompts back to back with no host wait in between: every pass finds its counters at zero
        ac.air_reset()
        ac.air_score(0, 2, q[:2], k[:2], v[:2], seqs)
        ac.air_score(2, L, q[2:], k[2:], v[2:], seqs)
        ac.air_budget()
        ac.air_select_compact(0, L, k, v)
    ac.air_reset()
    ac.air_score(0, L, q, k, v, seqs)
    same(want, state(ac))
    ac.close()


# ---------------------------------------------------------------------------------------
# Eq.10 on importance rows of little or no spread
# ---------------------------------------------------------------------------------------
def _low_spread_layers(w, seqs, kinds):
    """Layer inputs whose visual keys are, per layer kind:
         "normal"    the generator's
         "equal"     copies of one key                         -> importance exactly uniform, zero spread
         "sub"       copies + k 2^-21 in one element, k = 0..3 -> spread of a few 1e-8 of the mean (below what fp32 scores resolve)
         "small"     copies + k 2^-6 in that element           -> spread of about 1e-3 of the mean
    (bf16 and fp32 both hold these values exactly)."""
    out = []
    for l, kind in enumerate(kinds):
        li = synth.layer_inputs(w, l, seqs)
        if kind != "normal":
            k = synth.storage_to_f64(li.k)
            rng = np.random.default_rng([77, l])
            for b, s in enumerate(seqs):
                vis = slice(s.vis_start, s.vis_start + s.vis_len)
                k[b, :, vis] = k[b, :, s.vis_start:s.vis_start + 1]
                k[b, :, vis, 5] = 0.0
                if kind != "equal":
                    step = 2.0 ** -21 if kind == "sub" else 2.0 ** -6
                    k[b, :, vis, 5] = step * rng.integers(0, 4, size=(k.shape[1], s.vis_len))
            kk = synth.f32_to_bf16_bits(k.astype(np.float32)) if w.dtype == "bf16" else k.astype(np.float32)
            assert np.array_equal(synth.storage_to_f64(kk)[~np.isnan(k)], k[~np.isnan(k)])  # exactly representable
            li = type(li)(li.q_text, kk, li.v)
        out.append(li)
    return out


@pytest.mark.parametrize("base,n_vis,batch", [(2, 3000, 1), (3, 2500, 3), (1, 900, 1)])
def test_skewness_of_rows_with_little_or_no_spread(base, n_vis, batch):
    """Eq.10 where its sums cancel: layers whose visual keys are all equal, equal up to differences the fp32 scores
    cannot resolve, and equal up to a relative 1e-3, next to ordinary layers (skewness 15-40).  Checked: the
    skewness the library reports against (i) Eq.10 evaluated by the oracle on the library's own fp32 scores, to
    fp64 rounding, (ii) the oracle's own value within what the score tolerance allows, and the budgets that follow
    (a skewness off by orders of magnitude would hand one layer the whole skewness share of Eq.11)."""
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device

    dev = torch.device("cuda:0")
    kinds = ["normal", "equal", "sub", "small", "normal", "equal"]
    w = synth.get_workload(base).scaled(cfg_id=800 + base, batch=batch, n_layers=len(kinds), n_vis=n_vis, n_text=40,
                                        window=0, decode_steps=1, jitter=0.1 if batch > 1 else 0.0)
    seqs = w.seqs()
    L, B, Hkv = w.n_layers, w.batch, w.n_kv_heads
    layers = _low_spread_layers(w, seqs, kinds)
    ac = A.AirCache(config_for(w, 0.10, seqs=seqs, max_decode_steps=1), dev)
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    ac.air_score(0, L, q, k, v, seqs)
    ac.air_budget()
    g_st, g_sk = ac.air_get_stats()
    o_st, o_sk, own_sk = np.zeros((B, L)), np.zeros((B, L)), np.zeros((B, L))
    bound = np.zeros((B, L))
    for l in range(L):
        sc, _, a, c = P.oracle_score_layer(w, layers[l], seqs, w.alpha)
        o_st[:, l], o_sk[:, l] = a, c
        g = ac.air_get_scores(l)
        eps = P.check_scores(g, sc, seqs, f"layer {l} ({kinds[l]})")  # worst relative score error, <= 1e-5
        for b, s in enumerate(seqs):
            rows = g[b][:, : s.vis_len].astype(np.float64)
            own_sk[b, l] = np.mean([O.skewness(r) for r in rows])
            # a relative score error eps moves z = (x - mu) / sigma by eps mu / sigma, and Eq.10 by 3 times that
            # per unit of mean z^2 (and of the skewness itself through sigma)
            rel_spread = min(max(r.std() / r.mean(), 1e-300) for r in synth.storage_to_f64(np.asarray(sc[b])))
            bound[b, l] = 3.0 * eps / rel_spread * (1.0 + abs(c[b])) + P.STAT_RTOL * abs(c[b]) + 1e-9
    np.testing.assert_allclose(g_st, o_st, rtol=P.STAT_RTOL)
    # (i) Eq.10 itself, on equal inputs: only the order of the fp64 sums differs
    np.testing.assert_allclose(g_sk, own_sk, rtol=1e-7, atol=1e-7)
    for l, kind in enumerate(kinds):
        if kind in ("equal", "sub"):  # zero spread on both sides, exactly
            assert np.all(g_sk[:, l] == 0.0) and np.all(o_sk[:, l] == 0.0), (kind, g_sk[:, l], o_sk[:, l])
        else:
            assert np.all(np.abs(g_sk[:, l] - o_sk[:, l]) <= bound[:, l]), (kind, g_sk[:, l], o_sk[:, l], bound[:, l])
        if kind == "small":  # a real, small spread: the value is the definition's, not noise
            assert np.all(np.abs(g_sk[:, l] - o_sk[:, l]) <= 0.05 * (1.0 + np.abs(o_sk[:, l]))), (g_sk[:, l], o_sk[:, l])
    g_bud = ac.air_get_budgets()
    assert np.array_equal(g_bud, P.oracle_budgets(g_st, g_sk, seqs, 0.10))
    o_bud = P.oracle_budgets(o_st, o_sk, seqs, 0.10)
    assert np.array_equal(g_bud.sum(axis=1), o_bud.sum(axis=1)) and np.abs(g_bud - o_bud).max() <= 1, (g_bud, o_bud)
    print(f"[low spread base={base}] s_k gpu {np.round(g_sk[0], 6).tolist()} oracle {np.round(o_sk[0], 6).tolist()} "
          f"budgets {g_bud[0].tolist()}", flush=True)
    ac.close()
