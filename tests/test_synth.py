"""The seeded input generator: shapes, determinism, structure."""
import numpy as np

import synth


def test_bf16_rounding_is_nearest_even_and_exact_on_round_trip():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40, 0.0], dtype=np.float32)
    b = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f64(b)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to the even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1 + 2^-7 and 1 + 2^-6: goes to 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert np.array_equal(synth.f32_to_bf16_bits(back.astype(np.float32)), b)


def test_segments_and_ragged_batch():
    w = synth.get_workload(3)
    seqs = w.seqs()
    assert len(seqs) == 16
    assert len({s.vis_len for s in seqs}) > 4
    for s in seqs:
        assert abs(s.vis_len - 2304) <= 231 and abs(s.n_text - 256) <= 26
        assert s.win_start + s.win_len == s.seq_len and s.win_start >= s.text_start
    s1 = synth.get_workload(1).seqs()[0]
    assert (s1.seq_len, s1.vis_start, s1.vis_len, s1.win_start, s1.win_len) == (656, 16, 576, 640, 16)


def test_layer_inputs_deterministic_and_padded_with_nan():
    w = synth.get_workload(3).scaled(batch=3, n_layers=2, n_vis=60, n_text=20)
    a = synth.layer_inputs(w, 1)
    b = synth.layer_inputs(w, 1)
    assert np.array_equal(a.k, b.k) and np.array_equal(a.q_text, b.q_text) and np.array_equal(a.v, b.v)
    seqs = w.seqs()
    assert a.k.shape == (3, 4, max(s.seq_len for s in seqs), 128) and a.k.dtype == np.uint16
    short = min(range(3), key=lambda i: seqs[i].seq_len)
    if seqs[short].seq_len < a.k.shape[2]:
        assert np.all(np.isnan(synth.storage_to_f64(a.k[short, :, seqs[short].seq_len:])))
    assert not np.any(np.isnan(synth.storage_to_f64(a.k[short, :, : seqs[short].seq_len])))


def test_salient_recipes():
    w2 = synth.get_workload(2)
    fr = sorted(synth.salient_fraction(w2, l) for l in range(28))
    assert abs(fr[0] - 0.01) < 1e-12 and abs(fr[-1] - 0.20) < 1e-12
    w4 = synth.get_workload(4)
    s = w4.seqs()[0]
    m = synth.salient_mask(w4, 0, 0, s)
    frames = np.unique(np.nonzero(m)[0] // 196)
    assert len(frames) <= 3 and abs(m.mean() - 0.03) < 0.002
    w5 = synth.get_workload(5)
    f5 = [synth.salient_fraction(w5, l) for l in range(80)]
    assert 0.005 <= min(f5) and max(f5) <= 0.30
