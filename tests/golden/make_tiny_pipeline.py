"""Writes tests/golden/tiny_pipeline.txt: what the CPU oracle gives for the tiny fp32 workload (config 1).

The paper prints no worked example, so this file is not a pin of the oracle against the paper (the pins
are the closed forms and library cross-checks of tests/test_oracle_pins.py).  It records the oracle's own
answer so that an unintended change of its arithmetic shows up as a diff; a deliberate change reruns
this script and says why in its commit.  Calls nothing but the oracle and the seeded input generator:

    python tests/golden/make_tiny_pipeline.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import synth  # noqa: E402
from oracle import aircache_oracle as O  # noqa: E402


def tiny_pipeline_lines():
    w = synth.get_workload(1)
    s = w.seqs()[0]
    seg = O.Segments(s.seq_len, s.vis_start, s.vis_len, s.win_start, s.win_len)
    layers = [synth.layer_inputs(w, l) for l in range(w.n_layers)]
    res = O.compress_sequence([li.q_text[0].astype(np.float64) for li in layers],
                              [li.k[0].astype(np.float64) for li in layers], seg, w.alpha, 0.10)
    out = [f"# config 1 ({w.name}): {w.n_layers} layers, {w.n_q_heads}/{w.n_kv_heads} heads, d={w.head_dim}, "
           f"tokens {w.n_sys}+{w.n_vis}+{w.n_text}, window {s.win_len}, alpha {w.alpha}, retention 0.10",
           "budgets " + " ".join(str(k) for k in res.budgets)]
    for l in range(w.n_layers):
        out.append(f"layer {l} s_t {res.s_t[l]:.12e} s_k {res.s_k[l]:.12e}")
        for h, e in enumerate(res.elites[l]):
            out.append(f"layer {l} head {h} elite " + " ".join(str(int(x)) for x in e))
        for h in range(w.n_kv_heads):
            out.append(f"layer {l} kv {h} kept " + " ".join(str(int(x)) for x in res.indices[l][h]))
            top = np.argsort(-res.scores[l][h], kind="stable")[:3]
            out.append(f"layer {l} kv {h} top3 " + " ".join(f"{int(i)}:{res.scores[l][h][i]:.12e}" for i in top))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_pipeline.txt")
    with open(path, "w") as f:
        f.write("\n".join(tiny_pipeline_lines()) + "\n")
    print("wrote", path)
