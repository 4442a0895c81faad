"""air_decode_attn_static, the decode entry point that allocates nothing (its split-K exchange area is a fixed
array inside the library), against air_decode_attn through the C ABI: bitwise-equal outputs and caches on two
calls in a row, the second on a smaller input; sizes beyond the fixed area are refused before any launch."""
import ctypes as C

import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _compressed_pair(w, dev, tuning):
    """Two contexts over the same prompt, compressed alike: one for each entry point."""
    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device

    seqs = w.seqs()
    L = w.n_layers
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    pair = []
    tuning = dict(tuning)
    device_steps = 1 if tuning.pop("device_steps", False) else 0  # the tokens appended so far counted on the device
    for _ in range(2):
        ac = A.AirCache(config_for(w, 0.25, max_decode_steps=w.decode_steps, seqs=seqs, device_steps=device_steps), dev)
        ac.air_set_tuning(**tuning)
        ac.air_score(0, L, q, k, v, seqs)
        ac.air_budget()
        ac.air_select_compact(0, L, k, v)
        pair.append(ac)
    return pair


def _raw_decode(ac, fn_name, L, qn, kn, vn, out):
    """The call through the raw C ABI (no binding method in between)."""
    import torch

    fn = getattr(ac.lib, fn_name)
    st = fn(ac.handle, C.c_void_p(int(torch.cuda.current_stream().cuda_stream)), 0, L, C.c_void_p(qn.data_ptr()),
            C.c_void_p(kn.data_ptr()), C.c_void_p(vn.data_ptr()), C.c_void_p(out.data_ptr()))
    assert st == 0, (fn_name, st, ac.lib.air_last_error(ac.handle))


@pytest.mark.parametrize("base,tuning", [(2, dict(decode_splits=4, decode_waves=4, decode_tiles=4)),
                                         (2, dict(decode_splits=16, decode_waves=1, decode_tiles=2)),
                                         (2, dict(decode_splits=1, decode_waves=4, decode_tiles=4, decode_halves=2)),
                                         # two workgroups per unit that meet at an arrival counter of the static area
                                         (2, dict(decode_splits=1, decode_waves=4, decode_tiles=4, decode_halves=2, device_steps=True)),
                                         (1, dict(decode_splits=4))])
def test_static_entry_point_matches_the_workspace_one(base, tuning):
    import torch

    from paper_2503_23956_amd.device_inputs import to_device

    dev = torch.device("cuda:0")
    # first the larger input, then a smaller one: the fixed area still holds the first call's partials and counters
    shapes = [dict(n_layers=3, n_vis=900, n_text=37), dict(n_layers=2, n_vis=260, n_text=12)]
    for sh in shapes:
        w = synth.get_workload(base).scaled(decode_steps=3, window=0, **sh)
        ref, stat = _compressed_pair(w, dev, tuning)
        L = w.n_layers
        dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        out_r = torch.zeros((L, w.batch, w.n_q_heads, w.head_dim), dtype=dt, device=dev)
        out_s = torch.ones_like(out_r)
        for step in range(3):
            qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
            qn, kn, vn = (to_device(np.stack(x), dev) for x in (qs, ks, vs))
            _raw_decode(ref, "air_decode_attn", L, qn, kn, vn, out_r)
            _raw_decode(stat, "air_decode_attn_static", L, qn, kn, vn, out_s)
            torch.cuda.synchronize()
            assert not torch.isnan(out_s.float()).any()
            assert torch.equal(out_r, out_s), f"{sh} step {step}: outputs differ"
        lens = ref.air_get_lengths()
        assert np.array_equal(lens, stat.air_get_lengths())
        for (l, b, h) in [(0, 0, 0), (L - 1, w.batch - 1, w.n_kv_heads - 1)]:
            kr, vr = ref.air_get_cache(l, b, h, int(lens[b, l]))
            ks_, vs_ = stat.air_get_cache(l, b, h, int(lens[b, l]))
            assert np.array_equal(kr, ks_) and np.array_equal(vr, vs_)
        ref.close()
        stat.close()


def test_static_entry_point_refuses_what_its_fixed_area_cannot_hold():
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import to_device

    dev = torch.device("cuda:0")
    # 9 layers x 8 sequences x 4 KV heads = 288 units; 4 splits each need 1152 slots, the area holds 1024
    w = synth.get_workload(3).scaled(batch=8, n_layers=9, n_vis=200, n_text=12, decode_steps=2, jitter=0.0)
    ref, stat = _compressed_pair(w, dev, dict(decode_splits=4))
    L = w.n_layers
    qs, ks, vs = zip(*[synth.decode_inputs(w, l, 0) for l in range(L)])
    qn, kn, vn = (to_device(np.stack(x), dev) for x in (qs, ks, vs))
    out_s = torch.full((L, w.batch, w.n_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=dev)
    with pytest.raises(A.AirError) as e:
        stat.air_decode_attn_static(0, L, qn, kn, vn, out_s)
    assert e.value.status == A.binding.AIR_ERR_SHAPE and "1152" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(out_s == 7.0)  # refused before anything was launched
    assert np.array_equal(stat.air_get_lengths(), ref.air_get_lengths())  # and nothing was appended
    # the same step in two calls of fewer layers fits, and equals the workspace entry point's result
    out_r = torch.empty_like(out_s)
    ref.air_decode_attn(0, L, qn, kn, vn, out_r)
    stat.air_decode_attn_static(0, 5, qn[:5], kn[:5], vn[:5], out_s[:5])
    stat.air_decode_attn_static(5, L, qn[5:], kn[5:], vn[5:], out_s[5:])
    torch.cuda.synchronize()
    assert torch.equal(out_r, out_s)
    # one workgroup per unit exchanges nothing: any size goes through
    ref.air_set_tuning(decode_splits=1)
    stat.air_set_tuning(decode_splits=1)
    qs, ks, vs = zip(*[synth.decode_inputs(w, l, 1) for l in range(L)])
    qn, kn, vn = (to_device(np.stack(x), dev) for x in (qs, ks, vs))
    ref.air_decode_attn(0, L, qn, kn, vn, out_r)
    stat.air_decode_attn_static(0, L, qn, kn, vn, out_s)
    torch.cuda.synchronize()
    assert torch.equal(out_r, out_s)
    ref.close()
    stat.close()
