"""Workload shapes.

The five workloads follow the shapes the paper evaluates on: LLaVA-OV-7B /
Qwen2-7B attention geometry (28 layers, 28 query heads over 4 KV heads,
head_dim 128) with visual-token counts in the range of Tab.8 and the latency
set-up of Tab.3 (short text instruction, long visual prefix), plus a tiny fp32
case a CPU finishes in seconds and a 72B-shaped stress case.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class Seq:
    """Token segmentation of one prompt: [system | visual | text].

    The candidate span for the elite window (Eq.5) is [win_start,
    win_start+win_len), inside the text span; its last token is the reference
    row of the text-only attention.
    """

    seq_len: int
    vis_start: int
    vis_len: int
    win_start: int
    win_len: int

    @property
    def n_sys(self) -> int:
        return self.vis_start

    @property
    def text_start(self) -> int:
        return self.vis_start + self.vis_len

    @property
    def n_text(self) -> int:
        return self.seq_len - self.text_start


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    batch: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str  # "f32" | "bf16"
    n_sys: int
    n_vis: int  # nominal; jitter makes it per-sequence
    n_text: int
    jitter: float  # +-fraction applied to n_vis and n_text per sequence
    window: int  # candidate span = last `window` text tokens; 0 = all text tokens
    alpha: float
    retention: Tuple[float, ...]
    decode_steps: int
    salient: str  # recipe name, see generate.salient_fraction / salient_mask

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def seqs(self) -> List[Seq]:
        out = []
        for b in range(self.batch):
            n_vis, n_text = self.n_vis, self.n_text
            if self.jitter > 0.0:
                rng = np.random.default_rng([self.cfg_id, 7_000_003, b])
                u, u2 = rng.uniform(-self.jitter, self.jitter, size=2)
                n_vis = int(round(self.n_vis * (1.0 + u)))
                n_text = int(round(self.n_text * (1.0 + u2)))
            seq_len = self.n_sys + n_vis + n_text
            win = n_text if self.window <= 0 else min(self.window, n_text)
            out.append(Seq(seq_len, self.n_sys, n_vis, seq_len - win, win))
        return out

    @property
    def max_seq_len(self) -> int:
        return max(s.seq_len for s in self.seqs())

    @property
    def max_text(self) -> int:
        return max(s.n_text for s in self.seqs())

    def scaled(self, **kw) -> "Workload":
        """Same structure at another size (used for CPU-sized and mid-sized cases)."""
        return dataclasses.replace(self, **kw)


CONFIGS = {
    # Tiny CPU-checkable case; fp32; continuous last-16 window (the paper's
    # "continuous text tokens" ablation, Tab.5) is exercised with alpha = 0 and
    # the elite window with alpha = 0.9 on the same span.
    1: Workload("tiny-f32", 1, 1, 2, 4, 2, 64, "f32", 16, 576, 64, 0.0, 16, 0.9,
                (0.10,), 1, "uniform5"),
    # LLaVA-OV-7B-shaped, one anyres image.
    2: Workload("llava-ov-7b-anyres", 2, 1, 28, 28, 4, 128, "bf16", 14, 7290, 128, 0.0, 0, 0.9,
                (0.10,), 128, "layer_linear_1_20"),
    # Batched mid-length, ragged.
    3: Workload("batched-ragged", 3, 16, 28, 28, 4, 128, "bf16", 14, 2304, 256, 0.10, 0, 0.9,
                (0.05, 0.10, 0.25), 256, "layer_linear_1_20"),
    # Video-like: 32 frames x 196 tokens, salient tokens clustered in 3 frames.
    4: Workload("video-32f", 4, 4, 28, 28, 4, 128, "bf16", 14, 32 * 196, 512, 0.0, 0, 0.9,
                (0.10,), 512, "frames3"),
    # 72B-shaped single-GPU stress.
    5: Workload("72b-stress", 5, 2, 80, 64, 8, 128, "bf16", 14, 16384, 512, 0.0, 0, 0.9,
                (0.01, 0.02, 0.05, 0.10, 0.25, 0.50), 256, "loguniform"),
}


def get_workload(cfg_id: int) -> Workload:
    return CONFIGS[cfg_id]
