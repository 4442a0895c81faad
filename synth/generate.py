"""Seeded tensors for one layer of a workload.

Recipe (stands in for LLaVA-OV / Qwen2-VL activations on the paper's VQA and
video benchmarks, none of which is available here):

* base Q, K, V ~ N(0, 1) i.i.d., drawn per (workload, layer, sequence);
* a seeded subset of the visual tokens is "salient": their keys are shifted by
  +2 along a unit direction u drawn per (layer, sequence, KV head);
* every text-span query of the heads that share that KV head is shifted by
  1.5*sqrt(head_dim) along the same u, so salient keys gain about +3 in the
  scaled logit and the importance distribution gets a head effect;
* every text key is shifted by tau_l * u, tau_l seeded per layer in [0, 6], so
  the share of attention that goes to visual tokens differs between layers;
* the salient fraction and its placement depend on the workload (uniform,
  varying per layer, clustered in a few video frames, log-uniform per layer);
* values are rounded once to the storage dtype (fp32 or bf16); padding rows of
  ragged batches hold NaN so that any read outside a sequence shows up.

bf16 tensors are carried as uint16 bit patterns in numpy.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from .configs import Seq, Workload

_STREAM_BASE, _STREAM_SALIENT, _STREAM_DIR, _STREAM_TAU, _STREAM_FRAC, _STREAM_DECODE, _STREAM_FRAMES = range(7)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, 0x7FC0, r)
    return r.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def storage_to_f64(x: np.ndarray) -> np.ndarray:
    """Exact fp64 value of a stored tensor (fp32 array or bf16 bit patterns)."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f64(x)
    return x.astype(np.float64)


def _to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32)


def _pad_value(dtype: str):
    return np.uint16(0x7FC0) if dtype == "bf16" else np.float32(np.nan)


def salient_fraction(w: Workload, layer: int) -> float:
    if w.salient == "uniform5":
        return 0.05
    if w.salient == "layer_linear_1_20":
        fr = np.linspace(0.01, 0.20, w.n_layers)
        perm = np.random.default_rng([w.cfg_id, _STREAM_FRAC]).permutation(w.n_layers)
        return float(fr[perm[layer]])
    if w.salient == "frames3":
        return 0.03
    if w.salient == "loguniform":
        u = np.random.default_rng([w.cfg_id, _STREAM_FRAC]).uniform(np.log(0.005), np.log(0.30), w.n_layers)
        return float(np.exp(u[layer]))
    raise ValueError(w.salient)


def salient_mask(w: Workload, layer: int, b: int, seq: Seq) -> np.ndarray:
    """Boolean [vis_len]: which visual tokens carry the salient shift."""
    n = seq.vis_len
    f = salient_fraction(w, layer)
    rng = np.random.default_rng([w.cfg_id, _STREAM_SALIENT, layer, b])
    mask = np.zeros(n, dtype=bool)
    if w.salient == "frames3":
        n_frames = 32
        per = max(n // n_frames, 1)
        frames = np.random.default_rng([w.cfg_id, _STREAM_FRAMES, b]).choice(n_frames, size=3, replace=False)
        pool = np.concatenate([np.arange(fr * per, min((fr + 1) * per, n)) for fr in sorted(frames)])
        cnt = min(max(int(round(f * n)), 1), pool.size)
        mask[rng.choice(pool, size=cnt, replace=False)] = True
        return mask
    cnt = min(max(int(round(f * n)), 1), n)
    mask[rng.choice(n, size=cnt, replace=False)] = True
    return mask


@dataclass
class LayerInputs:
    """Storage-dtype tensors of one layer, head-major and padded to the batch maximum.

    q_text: [B][H_q ][max_text][d]  queries of the text span only (row j = text token j)
    k, v  : [B][H_kv][max_seq ][d]
    """

    q_text: np.ndarray
    k: np.ndarray
    v: np.ndarray


def layer_inputs(w: Workload, layer: int, seqs: List[Seq] | None = None) -> LayerInputs:
    seqs = w.seqs() if seqs is None else seqs
    B, Hq, Hkv, d, G = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.group
    max_seq = max(s.seq_len for s in seqs)
    max_text = max(s.n_text for s in seqs)
    st = np.uint16 if w.dtype == "bf16" else np.float32
    q_text = np.full((B, Hq, max_text, d), _pad_value(w.dtype), dtype=st)
    k = np.full((B, Hkv, max_seq, d), _pad_value(w.dtype), dtype=st)
    v = np.full((B, Hkv, max_seq, d), _pad_value(w.dtype), dtype=st)
    tau = float(np.random.default_rng([w.cfg_id, _STREAM_TAU, layer]).uniform(0.0, 6.0))
    gamma_q = 1.5 * np.sqrt(d)
    for b, s in enumerate(seqs):
        rng = np.random.default_rng([w.cfg_id, _STREAM_BASE, layer, b])
        kb = rng.standard_normal((Hkv, s.seq_len, d), dtype=np.float32)
        vb = rng.standard_normal((Hkv, s.seq_len, d), dtype=np.float32)
        qb = rng.standard_normal((Hq, s.n_text, d), dtype=np.float32)
        u = np.random.default_rng([w.cfg_id, _STREAM_DIR, layer, b]).standard_normal((Hkv, d)).astype(np.float32)
        u /= np.linalg.norm(u, axis=1, keepdims=True)
        sal = salient_mask(w, layer, b, s)
        vis = slice(s.vis_start, s.vis_start + s.vis_len)
        for h in range(Hkv):
            kv = kb[h, vis]
            kv[sal] += 2.0 * u[h]
            kb[h, s.text_start:] += tau * u[h]
            qb[h * G:(h + 1) * G] += np.float32(gamma_q) * u[h]
        k[b, :, : s.seq_len] = _to_storage(kb, w.dtype)
        v[b, :, : s.seq_len] = _to_storage(vb, w.dtype)
        q_text[b, :, : s.n_text] = _to_storage(qb, w.dtype)
    return LayerInputs(q_text, k, v)


def decode_inputs(w: Workload, layer: int, step: int):
    """New-token tensors of one decode step of one layer, storage dtype.

    Returns q_new [B][H_q][d], k_new [B][H_kv][d], v_new [B][H_kv][d].
    """
    rng = np.random.default_rng([w.cfg_id, _STREAM_DECODE, layer, step])
    q = rng.standard_normal((w.batch, w.n_q_heads, w.head_dim), dtype=np.float32)
    k = rng.standard_normal((w.batch, w.n_kv_heads, w.head_dim), dtype=np.float32)
    v = rng.standard_normal((w.batch, w.n_kv_heads, w.head_dim), dtype=np.float32)
    return _to_storage(q, w.dtype), _to_storage(k, w.dtype), _to_storage(v, w.dtype)
