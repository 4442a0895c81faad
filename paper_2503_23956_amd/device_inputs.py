"""Glue between the seeded input generator and the library: configuration and device upload."""
from __future__ import annotations

from typing import List

import numpy as np

from .binding import AIR_BF16, AIR_F32, make_config


def config_for(w, retention: float, *, alpha=None, budget_mode=0, min_keep=1, max_decode_steps=None, seqs=None,
               window_kind=0, device_steps=0):
    seqs = w.seqs() if seqs is None else seqs
    return make_config(
        n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, batch=w.batch,
        max_vis_len=max(s.vis_len for s in seqs),
        max_nonvis_len=max(s.seq_len - s.vis_len for s in seqs),
        max_window=max(s.win_len for s in seqs),
        max_decode_steps=w.decode_steps if max_decode_steps is None else max_decode_steps,
        dtype=AIR_BF16 if w.dtype == "bf16" else AIR_F32,
        alpha=w.alpha if alpha is None else alpha, retention=retention, budget_mode=budget_mode, min_keep=min_keep,
        window_kind=window_kind, device_steps=device_steps)


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
