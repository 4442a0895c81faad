"""Glue between the seeded input generator and the library: configuration and device upload."""
from __future__ import annotations

from typing import List

import numpy as np

from .binding import AIR_BF16, AIR_F32, make_config


def config_for(w, retention: float, *, alpha=None, budget_mode=0, min_keep=1, max_decode_steps=None, seqs=None,
               window_kind=0, device_steps=0, cache_in_place=0, causal_text=0):
    seqs = w.seqs() if seqs is None else seqs
    return make_config(
        n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, batch=w.batch,
        max_vis_len=max(s.vis_len for s in seqs),
        max_nonvis_len=max(s.seq_len - s.vis_len for s in seqs),
        max_window=max(s.win_len for s in seqs),
        max_decode_steps=w.decode_steps if max_decode_steps is None else max_decode_steps,
        dtype=AIR_BF16 if w.dtype == "bf16" else AIR_F32,
        alpha=w.alpha if alpha is None else alpha, retention=retention, budget_mode=budget_mode, min_keep=min_keep,
        window_kind=window_kind, device_steps=device_steps, cache_in_place=cache_in_place, causal_text=causal_text)


def to_device(x: np.ndarray, device):
    """Storage-dtype numpy array (fp32, or bf16 bit patterns as uint16) -> torch tensor on `device`."""
    import torch

    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(x).to(device)


def to_host(t) -> np.ndarray:
    """torch tensor -> storage-dtype numpy array (bf16 comes back as uint16 bit patterns)."""
    import torch

    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def upload_layers(w, layers: List[int], device, gen):
    """Generate and upload the given layers; returns (q_text, k, v) lists of device tensors."""
    q, k, v = [], [], []
    for l in layers:
        li = gen(w, l)
        q.append(to_device(li.q_text, device))
        k.append(to_device(li.k, device))
        v.append(to_device(li.v, device))
    return q, k, v


def device_layer_inputs(w, layer: int, seqs, device):
    """One layer of a workload drawn ON THE DEVICE with the generator's recipe: the salient sets, directions and
    per-layer text shift are the seeded generator's own (small, made on the host), only the N(0, 1) base tensors
    come from the device's random generator (seeded per workload, layer and sequence), because drawing the 11 GB
    of the largest workload on the host takes minutes.  Same shapes, padding (NaN) and value distribution as
    synth.layer_inputs, not the same values: for timing runs, not for comparisons with the oracle.
    Returns (q_text, k, v) device tensors in the storage dtype."""
    import torch

    import synth
    from synth import generate as G

    B, Hq, Hkv, d, grp = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.group
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    max_seq = max(s.seq_len for s in seqs)
    max_text = max(s.n_text for s in seqs)
    q_text = torch.full((B, Hq, max_text, d), float("nan"), dtype=dt, device=device)
    k = torch.full((B, Hkv, max_seq, d), float("nan"), dtype=dt, device=device)
    v = torch.full((B, Hkv, max_seq, d), float("nan"), dtype=dt, device=device)
    tau = float(np.random.default_rng([w.cfg_id, G._STREAM_TAU, layer]).uniform(0.0, 6.0))
    gamma_q = 1.5 * float(np.sqrt(d))
    gen = torch.Generator(device=device)
    for b, s in enumerate(seqs):
        gen.manual_seed((w.cfg_id * 1_000_003 + layer) * 1_000_003 + b)
        kb = torch.randn((Hkv, s.seq_len, d), generator=gen, device=device, dtype=torch.float32)
        vb = torch.randn((Hkv, s.seq_len, d), generator=gen, device=device, dtype=torch.float32)
        qb = torch.randn((Hq, s.n_text, d), generator=gen, device=device, dtype=torch.float32)
        u = np.random.default_rng([w.cfg_id, G._STREAM_DIR, layer, b]).standard_normal((Hkv, d)).astype(np.float32)
        u /= np.linalg.norm(u, axis=1, keepdims=True)
        ud = torch.from_numpy(u).to(device)
        sal = torch.from_numpy(synth.salient_mask(w, layer, b, s)).to(device)
        vis = kb[:, s.vis_start:s.vis_start + s.vis_len]
        vis += 2.0 * sal[None, :, None].to(torch.float32) * ud[:, None, :]
        kb[:, s.text_start:] += tau * ud[:, None, :]
        qb += gamma_q * ud.repeat_interleave(grp, dim=0)[:, None, :]
        k[b, :, : s.seq_len] = kb.to(dt)
        v[b, :, : s.seq_len] = vb.to(dt)
        q_text[b, :, : s.n_text] = qb.to(dt)
    return q_text, k, v
