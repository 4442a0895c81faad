"""Error behaviour of the boundary with a live context: every misuse is caught on the host, returns a
status, and leaves the context usable (no kernel is launched for a rejected call)."""
import dataclasses

import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _setup():
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device

    dev = torch.device("cuda:0")
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=300, n_text=24, decode_steps=2)
    seqs = w.seqs()
    ac = A.AirCache(config_for(w, 0.1, max_decode_steps=2, seqs=seqs), dev)
    layers = [synth.layer_inputs(w, l, seqs) for l in range(w.n_layers)]
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    return A, ac, w, seqs, q, k, v, dev


def test_stage_order_shapes_and_capacity_are_enforced():
    import torch

    A, ac, w, seqs, q, k, v, dev = _setup()
    B = A.binding
    L = w.n_layers

    def status(fn, *a, **kw):
        with pytest.raises(B.AirError) as e:
            fn(*a, **kw)
        return e.value.status

    # stages out of order
    assert status(ac.air_budget) == B.AIR_ERR_STATE                      # nothing scored yet
    assert status(ac.air_select_compact, 0, L, k=k, v=v) == B.AIR_ERR_STATE  # no budgets yet
    # an empty visual span, a span past the configured maximum, no text token
    s0 = seqs[0]
    for bad in (dataclasses.replace(s0, vis_len=0), dataclasses.replace(s0, vis_len=s0.vis_len + 1),
                dataclasses.replace(s0, seq_len=s0.vis_start + s0.vis_len)):
        assert status(ac.air_score, 0, L, q, k, v, [bad]) == B.AIR_ERR_SHAPE
    assert status(ac.air_score, L, L + 1, q[:1], k[:1], v[:1], seqs) == B.AIR_ERR_INVALID_ARG  # layer range past the end
    # the context is still usable: the regular sequence of calls goes through
    ac.air_score(0, 1, q[:1], k[:1], v[:1], seqs)
    assert status(ac.air_budget) == B.AIR_ERR_STATE                      # one layer still unscored
    ac.air_score(1, 2, q[1:], k[1:], v[1:], seqs)
    ac.air_budget()
    budgets = ac.air_get_budgets()
    assert budgets.sum() == round(0.1 * 300 * L)
    too_big = budgets.copy()
    too_big[0, 0] = 301
    assert status(ac.air_set_budgets, too_big) == B.AIR_ERR_SHAPE
    qn = torch.zeros((L, 1, w.n_q_heads, w.head_dim), dtype=q[0].dtype, device=dev)
    kn = torch.zeros((L, 1, w.n_kv_heads, w.head_dim), dtype=q[0].dtype, device=dev)
    out = torch.empty_like(qn)
    assert status(ac.air_decode_attn, 0, L, qn, kn, kn, out) == B.AIR_ERR_STATE  # not compacted yet
    ac.air_select_compact(0, L, k=k, v=v)
    assert status(ac.air_score, 0, L, q, k, v, seqs) == B.AIR_ERR_STATE   # already compacted
    ac.air_decode_attn(0, L, qn, kn, kn, out)
    ac.air_decode_attn(0, L, qn, kn, kn, out)
    assert status(ac.air_decode_attn, 0, L, qn, kn, kn, out) == B.AIR_ERR_STATE  # max_decode_steps used up
    torch.cuda.synchronize()
    assert np.array_equal(ac.air_get_lengths()[0], ac.air_get_budgets()[0] + (s0.seq_len - s0.vis_len) + 2)
    # and after a reset the next prompt goes through again
    ac.air_reset()
    ac.air_score(0, L, q, k, v, seqs)
    ac.air_budget()
    assert np.array_equal(ac.air_get_budgets(), budgets)
    # budgets handed in by the caller do not need every layer scored, but selecting a layer does: an unscored
    # layer is refused (its score rows would be the previous prompt's), a scored one and one with fixed indices go through
    ac.air_reset()
    ac.air_score(0, 1, q[:1], k[:1], v[:1], seqs)
    ac.air_set_budgets(budgets)
    assert status(ac.air_select_compact, 0, L, k=k, v=v) == B.AIR_ERR_STATE
    assert status(ac.air_select_compact, 1, 2, k=k[1:], v=v[1:]) == B.AIR_ERR_STATE
    idx = np.zeros((1, w.n_kv_heads, ac.cfg.max_vis_len), dtype=np.int32)
    idx[:, :, :] = np.arange(ac.cfg.max_vis_len)
    ac.air_set_indices(1, idx)
    ac.air_select_compact(0, L, k=k, v=v)
    assert np.array_equal(ac.air_get_indices(1)[0, 0, : budgets[0, 1]], np.arange(budgets[0, 1]))
    # launch-shape overrides outside their lists are refused and change nothing
    assert status(ac.air_set_tuning, decode_splits=3) == B.AIR_ERR_INVALID_ARG
    assert status(ac.air_set_tuning, select_threads=128) == B.AIR_ERR_INVALID_ARG
    ac.air_set_tuning(decode_splits=2, decode_waves=4)
    ac.close()


def test_device_side_generator_follows_the_recipe():
    """The benchmark draws the larger workloads on the device (device_layer_inputs): same shapes, padding and
    structure as the seeded host generator (the salient sets, directions and text shift ARE the host generator's),
    only the N(0, 1) base tensors differ."""
    import torch

    from paper_2503_23956_amd.device_inputs import device_layer_inputs, to_host

    dev = torch.device("cuda:0")
    w = synth.get_workload(3).scaled(batch=3, n_layers=2, n_vis=900, n_text=40)
    seqs = w.seqs()
    host = synth.layer_inputs(w, 1, seqs)
    q, k, v = device_layer_inputs(w, 1, seqs, dev)
    for a, b in ((q, host.q_text), (k, host.k), (v, host.v)):
        assert tuple(a.shape) == b.shape and a.dtype == torch.bfloat16
        ah = synth.storage_to_f64(to_host(a))
        assert np.array_equal(np.isnan(ah), np.isnan(synth.storage_to_f64(b)))  # the same padding rows hold NaN
    kd = synth.storage_to_f64(to_host(k))
    kh = synth.storage_to_f64(host.k)
    for b, s in enumerate(seqs):
        sal = synth.salient_mask(w, 1, b, s)
        vis = slice(s.vis_start, s.vis_start + s.vis_len)
        for h in range(w.n_kv_heads):
            # the salient keys are shifted by 2 along the same unit direction on both sides: project on the host's shift
            shift = kh[b, h, vis][sal].mean(axis=0) - kh[b, h, vis][~sal].mean(axis=0)
            u = shift / np.linalg.norm(shift)
            proj = (kd[b, h, vis][sal] @ u).mean() - (kd[b, h, vis][~sal] @ u).mean()
            assert abs(proj - 2.0) < 0.6, proj
        assert abs(kd[b, :, vis].std() - 1.0) < 0.1
