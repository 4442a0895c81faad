#!/usr/bin/env python3
"""Benchmark of the AirCache hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic prompt batch:
air_score + air_budget + air_select_compact over all layers (one-shot compression after
prefill), then `decode_steps` calls of air_decode_attn, each over all layers.  Inputs are
resident in HBM before the timed region starts.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--retention r] [--per-layer]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
METRIC = "compress \u00b5s/layer + compacted decode attn tokens/s; achieved HBM GB/s vs peak"


def _esize(w):
    return 2 if w.dtype == "bf16" else 4


def algorithmic_bytes(w, seqs, budgets, decode_steps):
    """Bytes the method itself has to move (per step of the benchmark), by stage.

    score   : K_v once + importance written        N_v*H_kv*d*e + 4*H_kv*N_v      per (layer, seq)
    select  : importance read + indices written    4*H_kv*N_v + 4*H_kv*k_l
    compact : kept rows of K and V read + written  4*(N_s+k_l+N_t)*H_kv*d*e
    decode  : K' and V' read once per step         2*T_l*H_kv*d*e, T_l growing by one per step
    """
    e, d, hkv = _esize(w), w.head_dim, w.n_kv_heads
    score = select = compact = 0
    decode_first = decode_last = decode_total = 0
    for b, s in enumerate(seqs):
        nonvis = s.seq_len - s.vis_len
        for l in range(w.n_layers):
            k = int(budgets[b][l])
            score += s.vis_len * hkv * d * e + 4 * hkv * s.vis_len
            select += 4 * hkv * s.vis_len + 4 * hkv * k
            compact += 4 * (nonvis + k) * hkv * d * e
            t0 = nonvis + k + 1
            decode_first += 2 * t0 * hkv * d * e
            decode_last += 2 * (t0 + decode_steps - 1) * hkv * d * e
            decode_total += sum(2 * (t0 + i) * hkv * d * e for i in range(decode_steps))
    return dict(score=score, select=select, compact=compact, compress=score + select + compact,
                decode_first=decode_first, decode_last=decode_last, decode_total=decode_total)


def cpu_baseline(w, seqs, retention, host_layers, dec_inputs, decode_steps):
    """The oracle, as it stands, on the host cores: full compression pass, then a sample of decode steps."""
    import numpy as np

    import synth
    from oracle import aircache_oracle as O

    try:
        from threadpoolctl import threadpool_info

        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    segs = [O.Segments(s.seq_len, s.vis_start, s.vis_len, s.win_start, s.win_len) for s in seqs]
    q64 = [[synth.storage_to_f64(li.q_text[b][:, : s.n_text]) for li in host_layers] for b, s in enumerate(seqs)]
    k64 = [[synth.storage_to_f64(li.k[b][:, : s.seq_len]) for li in host_layers] for b, s in enumerate(seqs)]
    v64 = [[synth.storage_to_f64(li.v[b][:, : s.seq_len]) for li in host_layers] for b, s in enumerate(seqs)]
    t0 = time.perf_counter()
    caches = []
    for b, seg in enumerate(segs):
        res = O.compress_sequence(q64[b], k64[b], seg, w.alpha, retention)
        per_layer = []
        for l in range(w.n_layers):
            per_layer.append([O.compact(k64[b][l][h], v64[b][l][h], seg, res.indices[l][h])
                              for h in range(w.n_kv_heads)])
        caches.append(per_layer)
    t_compress = time.perf_counter() - t0

    def one_decode_step(step):
        qn, kn, vn = dec_inputs[step]
        q, k, v = synth.storage_to_f64(qn), synth.storage_to_f64(kn), synth.storage_to_f64(vn)
        t1 = time.perf_counter()
        for b in range(w.batch):
            for l in range(w.n_layers):
                kcs, vcs = [], []
                for h in range(w.n_kv_heads):
                    kc, vc = caches[b][l][h]
                    # cache length of this step: pad with the new token repeated
                    kcs.append(np.concatenate([kc, np.repeat(k[l, b, h][None], step + 1, axis=0)]))
                    vcs.append(np.concatenate([vc, np.repeat(v[l, b, h][None], step + 1, axis=0)]))
                O.decode_layer(q[l, b], kcs, vcs)
        return time.perf_counter() - t1

    # every decode step when that stays within about 20 s of host time, else 8 steps spread over the run
    probe = one_decode_step(decode_steps // 2)
    n_sample = decode_steps if probe * decode_steps <= 20.0 else min(decode_steps, 8)
    sample = sorted(set(int(round(i * (decode_steps - 1) / max(n_sample - 1, 1))) for i in range(n_sample)))
    t_dec = 0.0
    for step in sample:
        t_dec += one_decode_step(step)
    t_step = t_dec / len(sample)
    total = t_compress + t_step * decode_steps
    # the same compression pass on ONE host thread (BLAS limited to one thread), for the per-core figure
    single = None
    try:
        from threadpoolctl import threadpool_limits

        with threadpool_limits(limits=1):
            t1 = time.perf_counter()
            for b, seg in enumerate(segs):
                O.compress_sequence(q64[b], k64[b], seg, w.alpha, retention)
            single = (time.perf_counter() - t1) * 1e6 / w.n_layers
    except Exception:
        pass
    return dict(value=w.batch * decode_steps / total, unit="tokens/s", cores=int(cores), kind="oracle",
                cores_note=f"threads of the BLAS pool inside numpy's matmul (the oracle's only parallel part; its own "
                           f"loops run on one thread); the host shows {os.cpu_count()} cores",
                sample=f"full compression pass of all {w.n_layers} layers ({t_compress:.2f} s) + {len(sample)} of "
                       f"{decode_steps} decode steps at their true cache lengths ({t_step * 1e3:.1f} ms/step), "
                       f"numpy fp64",
                compress_us_per_layer=t_compress * 1e6 / w.n_layers, decode_tokens_per_s=w.batch / t_step,
                compress_us_per_layer_one_thread=single)


def device_copy_reference(result, dev, dec_gbs):
    """Adds the rate of a plain device-to-device copy of 512 MiB and the rooflines as fractions of it."""
    import torch

    src = torch.ones(512 << 18, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    e0, e1 = (torch.cuda.Event(enable_timing=True) for _ in range(2))
    for _ in range(2):
        dst.copy_(src)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * src.numel() * 4 * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    result["device_copy"] = {"gbs_read_plus_write": copy_gbs, "bytes": src.numel() * 4}
    result["roofline"]["frac_of_device_copy"] = dec_gbs / copy_gbs
    result["roofline_compress"]["frac_of_device_copy"] = result["roofline_compress"]["achieved"] / copy_gbs


def cold_decode(A, w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, dev):
    """Decode steps rotating over `n_ctx` separately compressed copies of the prompt: between two visits of one
    copy's cache the other copies' caches pass through, more than the memory-side cache holds."""
    import numpy as np
    import torch

    from paper_2503_23956_amd.device_inputs import config_for

    L = w.n_layers
    probe = A.AirCache(config_for(w, retention, max_decode_steps=n_dec, seqs=seqs), dev)
    probe.air_score(0, L, prepared=probe.prepare(q, k, v, seqs))
    probe.air_budget()
    budgets = probe.air_get_budgets()
    del probe
    per_ctx = algorithmic_bytes(w, seqs, budgets, 1)["decode_first"]
    n_ctx = max(3, int(np.ceil(2.5 * 256e6 / per_ctx)))  # 2.5 x the memory-side cache between two visits
    n_ctx = min(n_ctx, 24)
    ctxs = []
    for _ in range(n_ctx):
        ac = A.AirCache(config_for(w, retention, max_decode_steps=n_dec, seqs=seqs), dev)
        ac.air_score(0, L, prepared=ac.prepare(q, k, v, seqs))
        ac.air_budget()
        ac.air_select_compact(0, L, prepared=ac.prepare(None, k, v))
        ctxs.append(ac)
    esz = dq.element_size()
    step_q, step_kv = dq[0].numel() * esz, dk[0].numel() * esz
    pq, pk, pv, po = dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr()
    per_visit = n_dec // n_ctx  # steps every copy takes per timed pass (each copy has room for n_dec appends)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    nonvis = [s.seq_len - s.vis_len for s in seqs]
    base_rows = sum((nonvis[b] + int(budgets[b][l])) for b in range(w.batch) for l in range(L))
    row_bytes = 2 * w.n_kv_heads * w.head_dim * (2 if w.dtype == "bf16" else 4)
    times, byts = [], 0
    torch.cuda.synchronize()
    for rep in range(3):  # the first pass warms the code path, not the caches
        total = 0
        e0.record()
        for t in range(per_visit):
            for ac in ctxs:
                i = rep * per_visit + t
                ac.air_decode_attn(0, L, pq + i * step_q, pk + i * step_kv, pv + i * step_kv, po)
                total += (base_rows + (i + 1) * w.batch * L) * row_bytes
        e1.record()
        torch.cuda.synchronize()
        if rep:
            times.append(e0.elapsed_time(e1))
            byts = total
        if (rep + 2) * per_visit > n_dec:
            break
    n_calls = per_visit * n_ctx
    us = float(np.mean(times)) * 1e3 / n_calls
    gbs = byts / (float(np.mean(times)) * 1e-3) / 1e9
    for ac in ctxs:
        ac.close()
    return {"us_per_step": us, "achieved": gbs, "frac": gbs / HBM_PEAK_GBS, "contexts": n_ctx,
            "bytes_between_two_visits_of_a_cache": int(per_ctx * (n_ctx - 1)),
            "note": "each step reads a cache that was last read n_ctx - 1 steps ago; the warm figure (roofline) re-reads one cache every step"}


def in_place_figures(A, w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, dev, pool_workspace_bytes):
    """The same workload with cache_in_place: the compaction runs inside (copies of) the prompt's K / V tensors.
    Reports the workspace without the cache pool and what the one-workgroup-per-unit walk costs."""
    import numpy as np
    import torch

    from paper_2503_23956_amd.device_inputs import config_for

    L = w.n_layers
    extra = n_dec + 31
    def roomy(t):
        B, H, T, d = t.shape
        big = torch.empty((B, H, T + extra, d), dtype=t.dtype, device=dev)
        big[:, :, :T] = t
        return big
    k2, v2 = [roomy(t) for t in k], [roomy(t) for t in v]
    ac = A.AirCache(config_for(w, retention, max_decode_steps=n_dec, seqs=seqs, cache_in_place=1), dev)
    prep_score, prep_compact = ac.prepare(q, k2, v2, seqs), ac.prepare(None, k2, v2)
    esz = dq.element_size()
    step_q, step_kv = dq[0].numel() * esz, dk[0].numel() * esz
    pq, pk, pv, po = dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    comp, dec = [], []
    for it in range(4):
        for big, t in zip(k2 + v2, k + v):  # the pass before compacted these tensors: restore the prompt (not timed)
            big[:, :, : t.shape[2]] = t
        ac.air_reset()
        ac.air_score(0, L, prepared=prep_score)
        ac.air_budget()
        ev[0].record()
        ac.air_select_compact(0, L, prepared=prep_compact)
        ev[1].record()
        for t in range(n_dec):
            ac.air_decode_attn(0, L, pq + t * step_q, pk + t * step_kv, pv + t * step_kv, po)
        ev[2].record()
        torch.cuda.synchronize()
        if it:
            comp.append(ev[0].elapsed_time(ev[1]))
            dec.append(ev[1].elapsed_time(ev[2]))
    res = {"workspace_bytes": int(ac.workspace_bytes), "workspace_bytes_with_cache_pool": int(pool_workspace_bytes),
           "select_compact_us": float(np.mean(comp)) * 1e3, "decode_us_per_step": float(np.mean(dec)) * 1e3 / n_dec,
           "note": "K' / V' written over the prompt's own K / V rows by one workgroup per (layer, sequence, KV head)"}
    ac.close()
    return res


def measure_config(A, cfg_id, dev, timed_passes):
    """Compression and decode timings of another workload at its 10 % retention, inputs drawn on the device."""
    import numpy as np
    import torch

    import synth
    from paper_2503_23956_amd.device_inputs import device_layer_inputs

    w = synth.get_workload(cfg_id)
    seqs = w.seqs()
    L, n_dec, retention = w.n_layers, w.decode_steps, 0.10
    q, k, v = [], [], []
    for l in range(L):
        a, b, c = device_layer_inputs(w, l, seqs, dev)
        q.append(a), k.append(b), v.append(c)
    gen = torch.Generator(device=dev)
    gen.manual_seed(77 + cfg_id)
    dt = q[0].dtype
    dq = torch.randn((n_dec, L, w.batch, w.n_q_heads, w.head_dim), generator=gen, device=dev, dtype=torch.float32).to(dt)
    dk = torch.randn((n_dec, L, w.batch, w.n_kv_heads, w.head_dim), generator=gen, device=dev, dtype=torch.float32).to(dt)
    dv = torch.randn((n_dec, L, w.batch, w.n_kv_heads, w.head_dim), generator=gen, device=dev, dtype=torch.float32).to(dt)
    out = torch.empty((L, w.batch, w.n_q_heads, w.head_dim), dtype=dt, device=dev)
    stage, wall, budgets, _, ws_bytes = timed_passes(w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, 3, 1)
    sc, bu, se, de, comp_ms = stage.mean(axis=0)
    ab = algorithmic_bytes(w, seqs, budgets, n_dec)
    res = {
        "workload": f"config{w.cfg_id}:{w.name}", "retention": retention, "batch": w.batch, "layers": L,
        "tokens": f"{w.n_sys}+{w.n_vis}+{w.n_text}", "decode_steps": n_dec, "data": "synthetic, drawn on the device",
        "units_per_decode_launch": L * w.batch * w.n_kv_heads,
        "compress_us_per_layer": comp_ms * 1e3 / L, "compress_frac": ab["compress"] / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "score_frac": ab["score"] / (sc * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "stage_us": {"score": sc * 1e3, "budget": bu * 1e3, "select_compact": se * 1e3, "decode_per_step": de * 1e3 / n_dec},
        "decode_us_per_step": de * 1e3 / n_dec, "decode_tokens_per_s": w.batch * n_dec / (de * 1e-3),
        "decode_frac": ab["decode_total"] / (de * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "decode_bytes_per_step_first_last": [ab["decode_first"], ab["decode_last"]],
        "compress_bytes": ab["compress"], "workspace_bytes": int(ws_bytes),
        "budgets_min_mean_max": [int(np.min(budgets)), float(np.mean(budgets)), int(np.max(budgets))],
    }
    del q, k, v, dq, dk, dv, out
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--retention", type=float, default=None)
    ap.add_argument("--decode-steps", type=int, default=None)
    ap.add_argument("--per-layer", action="store_true", help="one air_decode_attn call per layer instead of one per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tuning", default="", metavar="K=V,...",
                    help="launch-shape overrides passed to air_set_tuning for every context of the run (A/B measurements)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the one-launch-per-layer passes and the device-copy reference (profiling runs)")
    ap.add_argument("--score-per-layer", action="store_true",
                    help="also time air_score called one layer at a time, as a caller that scores each layer "
                         "right after its prefill would")
    ap.add_argument("--budget-divergence", action="store_true",
                    help="also report the Jensen-Shannon divergence between the layer budgets of the allocation "
                         "strategies (uniform, strength only, skewness only, both), as the paper's Tab.14 does")
    ap.add_argument("--retention-sweep", action="store_true",
                    help="also time the same workload with the full cache and at 50 % / 10 % / 1 % retention "
                         "(the quantity the paper's efficiency table reports for attention alone)")
    ap.add_argument("--graph-decode", action="store_true",
                    help="also time the decode loop replayed from a HIP graph (device-counted steps): one recorded "
                         "step of one launch per layer, as a model that calls the attention layer by layer would hold it")
    ap.add_argument("--window-sweep", action="store_true",
                    help="also time air_score with the observation windows of the paper's ablation table: elite, "
                         "continuous last 16 / 32 text tokens, all text tokens, visual window of 32")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MB",
                    help="only run a plain device copy of this many MB (reference for the rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.copy_probe:
        src = torch.ones(args.copy_probe << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": args.copy_probe << 20, "launches": 5}))
        return

    import paper_2503_23956_amd as A
    import synth
    from paper_2503_23956_amd import binding
    from paper_2503_23956_amd.device_inputs import config_for, device_layer_inputs, to_device

    if not os.path.exists(binding.LIB_PATH):
        from paper_2503_23956_amd.build import build

        build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = synth.get_workload(args.config)
    retention = args.retention if args.retention is not None else (0.10 if 0.10 in w.retention else w.retention[0])
    n_dec = args.decode_steps if args.decode_steps is not None else w.decode_steps
    seqs = w.seqs()
    L = w.n_layers

    host_layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q = [to_device(li.q_text, dev) for li in host_layers]
    k = [to_device(li.k, dev) for li in host_layers]
    v = [to_device(li.v, dev) for li in host_layers]
    dec_inputs = []
    for step in range(n_dec):
        qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
        dec_inputs.append((np.stack(qs), np.stack(ks), np.stack(vs)))
    dq = to_device(np.stack([d[0] for d in dec_inputs]), dev)  # [steps][L][B][Hq][d]
    dk = to_device(np.stack([d[1] for d in dec_inputs]), dev)
    dv = to_device(np.stack([d[2] for d in dec_inputs]), dev)
    out = torch.empty((L, w.batch, w.n_q_heads, w.head_dim), dtype=q[0].dtype, device=dev)

    tuning = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in args.tuning.split(",") if kv}

    def timed_passes(w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, steps, warmup, per_layer=False,
                     want_stats=False):
        """One context at this retention: `warmup` untimed passes of the whole hot path, then `steps` timed ones with
        three events each (in front of air_score, behind air_select_compact, behind the last decode step), then a few
        more passes with an event at every stage boundary for the breakdown.  An event costs the stream a few
        microseconds, so the stage times carry that overhead and the compression figure is the region timed as a whole.
        Returns times in ms [steps][score, budget, select_compact (means of the breakdown passes), decode, compression
        (of the timed pass)], wall seconds, budgets, stats."""
        L = w.n_layers
        ac = A.AirCache(config_for(w, retention, max_decode_steps=n_dec, seqs=seqs), dev)
        if tuning:
            ac.air_set_tuning(**tuning)
        ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
        # host-side marshalling is done once, outside the timed region: descriptor arrays and raw addresses
        prep_score = ac.prepare(q, k, v, seqs)
        prep_compact = ac.prepare(None, k, v)
        esz = dq.element_size()
        step_q = dq[0].numel() * esz
        step_kv = dk[0].numel() * esz
        lay_q = dq[0, 0].numel() * esz
        lay_kv = dk[0, 0].numel() * esz
        pq, pk, pv, po = dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr()

        hs = int(torch.cuda.current_stream(dev).cuda_stream)  # the launch stream's handle, taken once

        def one_step(events=None, boundaries=False):
            ac.air_reset()
            if events is not None:
                events[0].record()
            ac.air_score(0, L, prepared=prep_score, stream=hs)
            if boundaries:
                events[1].record()
            ac.air_budget(stream=hs)
            if boundaries:
                events[2].record()
            ac.air_select_compact(0, L, prepared=prep_compact, stream=hs)
            if events is not None:
                events[3].record()
            for t in range(n_dec):
                if per_layer:
                    for l in range(L):
                        ac.air_decode_attn(l, l + 1, pq + t * step_q + l * lay_q, pk + t * step_kv + l * lay_kv,
                                           pv + t * step_kv + l * lay_kv, po + l * lay_q, stream=hs)
                else:
                    ac.air_decode_attn(0, L, pq + t * step_q, pk + t * step_kv, pv + t * step_kv, po, stream=hs)
            if events is not None:
                events[4].record()

        for _ in range(warmup):
            one_step()
        torch.cuda.synchronize()
        budgets = ac.air_get_budgets()
        stats = ac.air_get_stats() if want_stats else None
        all_events = [[ev() for _ in range(5)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            one_step(all_events[i])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

        timed = np.array([[e[3].elapsed_time(e[4]), e[0].elapsed_time(e[3])] for e in all_events])  # ms: decode, compression
        bd_events = [[ev() for _ in range(5)] for _ in range(min(steps, 5))]
        for e in bd_events:
            one_step(e, boundaries=True)
        torch.cuda.synchronize()
        bd = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in bd_events]).mean(axis=0)
        stage = np.concatenate([np.tile(bd, (steps, 1)), timed], axis=1)
        ws_bytes = ac.workspace_bytes
        del ac
        return stage, wall, budgets, stats, ws_bytes

    def run(retention, steps, warmup, per_layer=args.per_layer, want_stats=False):
        return timed_passes(w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, steps, warmup, per_layer, want_stats)[:4]

    stage, wall, budgets, stats, ws_bytes_main = timed_passes(w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, args.steps,
                                                              args.warmup, args.per_layer, True)
    score_ms, budget_ms, select_ms, decode_ms, compress_ms = stage.mean(axis=0)
    ms_per_step = wall * 1e3 / args.steps
    ab = algorithmic_bytes(w, seqs, budgets, n_dec)
    n_launch = n_dec * (L if args.per_layer else 1)
    dec_launch_us = decode_ms * 1e3 / n_launch
    dec_gbs = ab["decode_total"] / (decode_ms * 1e-3) / 1e9
    result = {
        "metric": METRIC,
        "value": w.batch * n_dec / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"config{w.cfg_id}:{w.name}", "batch": w.batch, "layers": L,
                   "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "tokens": f"{w.n_sys}+{w.n_vis}+{w.n_text}", "retention": retention, "alpha": w.alpha,
                   "decode_steps": n_dec, "decode_launch": "per-layer" if args.per_layer else "all-layers"},
        "compress_us_per_layer": compress_ms * 1e3 / L,
        "decode_tokens_per_s": w.batch * n_dec / (decode_ms * 1e-3),
        "budgets_min_mean_max": [int(np.min(budgets)), float(np.mean(budgets)), int(np.max(budgets))],
        "stage_us": {"score": score_ms * 1e3, "budget": budget_ms * 1e3, "select_compact": select_ms * 1e3,
                     "decode_per_step": decode_ms * 1e3 / n_dec,
                     "note": "score / budget / select_compact from separate passes with an event at every stage boundary "
                             "(an event costs the stream a few us: their sum exceeds the compression pass timed as a "
                             "whole; up to 64 layers air_score's last kernel does the allocation and air_budget launches nothing)"},
        "roofline": {"kernel": "air_decode_attn", "bound": "hbm", "achieved": dec_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dec_gbs / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_launch": ab["decode_total"] / n_launch, "launch_us": dec_launch_us},
        "roofline_compress": {"kernel": "air_score+air_budget+air_select_compact", "bound": "hbm",
                              "achieved": ab["compress"] / (compress_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                              "unit": "GB/s", "frac": ab["compress"] / (compress_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "score_frac": ab["score"] / (score_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "bytes": ab["compress"]},
    }
    # median and minimum over the timed passes
    comp_iter = stage[:, 4]
    result["compress_us_per_layer_median_min"] = [float(np.median(comp_iter)) * 1e3 / L, float(comp_iter.min()) * 1e3 / L]
    result["workspace_bytes"] = int(ws_bytes_main)
    result["decode_us_per_step_median_min"] = [float(np.median(stage[:, 3])) * 1e3 / n_dec, float(stage[:, 3].min()) * 1e3 / n_dec]
    # Eq.9-10 per layer of sequence 0 (mean over the KV heads): the spread the budgets follow
    if stats is not None:
        result["layer_stats_seq0"] = {"s_t": [round(float(x), 6) for x in stats[0][0]],
                                      "s_k": [round(float(x), 4) for x in stats[1][0]]}
    # the same decode steps as one launch per layer on the one stream (a few passes)
    if not args.per_layer and not args.no_extras:
        pl = run(retention, 3, 1, per_layer=True)[0].mean(axis=0)
        result["decode_per_layer_launches"] = {"us_per_step": float(pl[3]) * 1e3 / n_dec,
                                               "tokens_per_s": w.batch * n_dec / (float(pl[3]) * 1e-3)}
    # what a plain kernel reaches on this machine: a device-to-device copy of 512 MiB
    if not args.no_extras:
        device_copy_reference(result, dev, dec_gbs)
    # HBM traffic of the dominant kernel: NOT measured in this run.  It is the per-launch sum of the rocprofv3
    # FETCH_SIZE / WRITE_SIZE counters of this kernel from the committed summary named below, which is remade
    # whenever the kernel changes (the summary states its command and the counter scaling).
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_per_kernel_config2_config5.txt")) as f:
            tr = json.load(f).get(result["config"]["workload"], {}).get("air_decode_attn")
        if tr and not args.per_layer:
            result["roofline"]["traffic"] = tr["fetch_bytes"] + tr["write_bytes"]
            result["roofline"]["traffic_source"] = ("profiles/hbm_traffic_per_kernel_config2_config5.txt: rocprofv3 --pmc byte counters of "
                                                    "this kernel, a committed summary, not measured in this run")
    except (OSError, ValueError):
        pass
    # ---- decode with a cold memory-side cache: the steps rotate over several compressed copies of the prompt, so
    # that more than the 256 MB of the memory-side cache is read between two visits of one copy
    # (an extra section that fails leaves its error text in its place: the line and its headline figures still print)
    def extra(name, fn):
        try:
            result[name] = fn()
        except Exception as e:  # noqa: BLE001
            result[name] = {"error": f"{type(e).__name__}: {e}"}
            torch.cuda.synchronize()

    if not args.no_extras and not args.per_layer:
        extra("decode_cold_cache", lambda: cold_decode(A, w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, dev))
    # ---- compaction inside the prompt's own tensors: the workspace without the cache pool
    if not args.no_extras and not args.per_layer and w.dtype == "bf16" and w.head_dim == 128:
        extra("cache_in_place", lambda: in_place_figures(A, w, seqs, q, k, v, dq, dk, dv, out, n_dec, retention, dev, ws_bytes_main))
    # ---- the quantity of the paper's efficiency table (Tab.3), for attention alone: the same workload with the
    # full cache and at 50 % / 10 % / 1 % retention
    if args.retention_sweep or not args.no_extras:
        sweep = []
        for r in (1.0, 0.5, 0.1, 0.01):
            sc, bu, se, de, comp = run(r, 3, 1)[0].mean(axis=0)
            sweep.append({"retention": r, "compress_us_per_layer": comp * 1e3 / L,
                          "decode_us_per_step": de * 1e3 / n_dec})
        for e in sweep:
            e["decode_speedup_vs_full_cache"] = sweep[0]["decode_us_per_step"] / e["decode_us_per_step"]
        result["retention_sweep"] = sweep
    if args.score_per_layer:
        ac = A.AirCache(config_for(w, retention, max_decode_steps=n_dec, seqs=seqs), dev)
        preps = [ac.prepare(q[l:l + 1], k[l:l + 1], v[l:l + 1], seqs) for l in range(L)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        times = []
        for it in range(4):
            ac.air_reset()
            e0.record()
            for l in range(L):
                ac.air_score(l, l + 1, prepared=preps[l])
            e1.record()
            torch.cuda.synchronize()
            if it:
                times.append(e0.elapsed_time(e1))
        result["score_one_layer_per_call"] = {"us_per_layer": float(np.mean(times)) * 1e3 / L,
                                              "all_layers_in_one_call_us_per_layer": score_ms * 1e3 / L}
        del ac
    if args.budget_divergence:
        from paper_2503_23956_amd.diagnostics import js_divergence

        names = {0: "strength+skew", 1: "uniform", 2: "strength", 3: "skew"}
        alloc = {}
        for mode, name in names.items():
            ac = A.AirCache(config_for(w, retention, budget_mode=mode, max_decode_steps=n_dec, seqs=seqs), dev)
            ac.air_score(0, L, prepared=ac.prepare(q, k, v, seqs))
            ac.air_budget()
            alloc[name] = ac.air_get_budgets()
            del ac
        pairs = [("uniform", "strength"), ("uniform", "skew"), ("strength", "skew"), ("uniform", "strength+skew")]
        result["budget_js_divergence"] = {
            f"{a} & {b}": float(np.mean([js_divergence(alloc[a][i], alloc[b][i]) for i in range(w.batch)]))
            for a, b in pairs}
    if args.graph_decode:
        res = {}
        for name, per_layer in (("one_launch_per_layer", True), ("all_layers_in_one_launch", False)):
            ac = A.AirCache(config_for(w, retention, max_decode_steps=n_dec, seqs=seqs, device_steps=1), dev)
            prep_score, prep_compact = ac.prepare(q, k, v, seqs), ac.prepare(None, k, v)
            sq, sk, sv = torch.empty_like(dq[0]), torch.empty_like(dk[0]), torch.empty_like(dv[0])
            g = torch.cuda.CUDAGraph()
            ac.air_score(0, L, prepared=prep_score)
            ac.air_budget()
            ac.air_select_compact(0, L, prepared=prep_compact)
            with torch.cuda.graph(g):
                if per_layer:
                    for l in range(L):
                        ac.air_decode_attn(l, l + 1, sq[l:l + 1], sk[l:l + 1], sv[l:l + 1], out[l:l + 1])
                else:
                    ac.air_decode_attn(0, L, sq, sk, sv, out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            times = []
            for it in range(4):
                ac.air_reset()
                ac.air_score(0, L, prepared=prep_score)
                ac.air_budget()
                ac.air_select_compact(0, L, prepared=prep_compact)
                sq.copy_(dq[0]), sk.copy_(dk[0]), sv.copy_(dv[0])
                e0.record()
                for _ in range(n_dec):
                    g.replay()
                e1.record()
                torch.cuda.synchronize()
                if it:
                    times.append(e0.elapsed_time(e1))
            s0 = seqs[0]
            want_len = (s0.seq_len - s0.vis_len) + int(budgets[0, 0]) + n_dec
            assert int(ac.air_get_lengths()[0, 0]) == want_len, "replayed steps did not advance the cache"
            res[name] = float(np.mean(times)) * 1e3 / n_dec
            del ac, g
        result["decode_graph_replay_us_per_step"] = res
    if args.window_sweep:
        import dataclasses

        def text_tail(n):
            return [dataclasses.replace(s, win_start=s.seq_len - min(n, s.n_text), win_len=min(n, s.n_text)) for s in seqs]

        variants = [("elite", A.AIR_WINDOW_TEXT, w.alpha, seqs),
                    ("continuous_16", A.AIR_WINDOW_TEXT, 0.0, text_tail(16)),
                    ("continuous_32", A.AIR_WINDOW_TEXT, 0.0, text_tail(32)),
                    ("all_text", A.AIR_WINDOW_TEXT, 0.0, text_tail(1 << 30)),
                    # the generator has no queries for visual tokens: the first 32 text queries stand in for them
                    ("visual_32", A.AIR_WINDOW_VISUAL, 0.0,
                     [dataclasses.replace(s, win_start=s.text_start - 32, win_len=32) for s in seqs])]
        result["window_sweep_score_us_per_layer"] = {}
        for name, kind, alpha, sq in variants:
            ac = A.AirCache(config_for(w, retention, alpha=alpha, max_decode_steps=n_dec, seqs=sq, window_kind=kind), dev)
            prep = ac.prepare(q, k, v, sq)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            times = []
            for it in range(4):
                ac.air_reset()
                e0.record()
                ac.air_score(0, L, prepared=prep)
                e1.record()
                torch.cuda.synchronize()
                if it:
                    times.append(e0.elapsed_time(e1))
            result["window_sweep_score_us_per_layer"][name] = float(np.mean(times)) * 1e3 / L
            del ac
    # ---- the other workloads the target names (GPU timing only; inputs drawn on the device)
    if not args.no_extras and not args.per_layer and args.config == 2:
        del q, k, v, dq, dk, dv, out
        torch.cuda.empty_cache()
        result["per_config"] = {}
        for cfg_id in (3, 4, 5):
            try:
                result["per_config"][f"config{cfg_id}"] = measure_config(A, cfg_id, dev, timed_passes)
            except Exception as e:  # noqa: BLE001
                result["per_config"][f"config{cfg_id}"] = {"error": f"{type(e).__name__}: {e}"}
                torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, seqs, retention, host_layers, dec_inputs, n_dec)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
