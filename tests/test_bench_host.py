"""Host-side checks of bench.py that need no GPU: the one-GPU contract and the algorithmic-byte counts."""
import subprocess
import sys
from pathlib import Path

import numpy as np
import pytest

ROOT = Path(__file__).resolve().parent.parent
sys.path.insert(0, str(ROOT))

import bench  # noqa: E402
import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and not p.stdout.strip()


def test_algorithmic_bytes_match_the_per_unit_formulas():
    # config 2 with the uniform budget: figures that can be written down by hand
    w = synth.get_workload(2)
    seqs = w.seqs()
    budgets = np.full((1, w.n_layers), 729, dtype=np.int32)
    ab = bench.algorithmic_bytes(w, seqs, budgets, decode_steps=128)
    L, hkv, d, e = 28, 4, 128, 2
    n_v, nonvis = 7290, 14 + 128
    assert ab["score"] == L * (n_v * hkv * d * e + 4 * hkv * n_v)
    assert ab["select"] == L * (4 * hkv * n_v + 4 * hkv * 729)
    assert ab["compact"] == L * 4 * (nonvis + 729) * hkv * d * e
    t0 = nonvis + 729 + 1  # keys the first decode step reads, the appended one included
    assert ab["decode_first"] == L * 2 * t0 * hkv * d * e
    assert ab["decode_last"] == L * 2 * (t0 + 127) * hkv * d * e
    assert ab["decode_total"] == sum(L * 2 * (t0 + i) * hkv * d * e for i in range(128))
    assert ab["compress"] == ab["score"] + ab["select"] + ab["compact"]
    # the figures quoted for this workload: 49.9 -> 57.3 MB per decode step, ~316 MB per compression pass
    assert abs(ab["decode_first"] / 1e6 - 50.0) < 0.3 and abs(ab["decode_last"] / 1e6 - 57.3) < 0.3
    assert abs(ab["compress"] / 1e6 - 316) < 2


def test_metric_string_is_the_one_the_baseline_file_names():
    import json
    import os

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    path = os.path.join(root, "BASELINE.json")
    if not os.path.exists(path):
        pytest.skip("no BASELINE.json beside the repository")
    assert bench.METRIC == json.load(open(path))["metric"]
