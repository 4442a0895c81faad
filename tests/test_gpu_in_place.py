"""Compaction inside the prompt's own K / V tensors (cache_in_place) against the workspace-pool path: same kept
indices, same cache rows, bitwise the same decode outputs; no cache pool in the workspace; refusals on the host."""
import numpy as np
import pytest

import synth
from oracle import aircache_oracle as O
from tests import parity_util as P

pytestmark = pytest.mark.gpu


def _roomy(x_host, extra_rows, dev):
    """[B][H][T][d] host tensor -> device tensor with `extra_rows` more (NaN) rows per head, contiguous."""
    import torch

    from paper_2503_23956_amd.device_inputs import to_device

    t = to_device(x_host, dev)
    B, H, T, d = t.shape
    big = torch.full((B, H, T + extra_rows, d), float("nan"), dtype=t.dtype, device=dev)
    big[:, :, :T] = t
    return big


@pytest.mark.parametrize("base,batch,n_vis,retention,steps,tuning",
                         [(2, 1, 1500, 0.10, 40, None), (2, 1, 700, 1.00, 35, None), (2, 1, 3000, 0.01, 3, None),
                          (3, 3, 900, 0.25, 34, None),
                          # the split-K instance of the in-place decode kernel, and through the entry point with the static exchange area
                          (2, 1, 1500, 0.10, 36, dict(decode_splits=4, decode_waves=4, decode_tiles=4)),
                          (2, 1, 1500, 0.10, 36, dict(decode_splits=2, decode_waves=8, decode_tiles=2, static=True)),
                          # two workgroups per unit, one half of the columns of V' each
                          (2, 1, 1500, 0.10, 36, dict(decode_splits=1, decode_waves=4, decode_tiles=4, decode_halves=2))])
def test_in_place_compaction_equals_the_pool_path(base, batch, n_vis, retention, steps, tuning):
    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device, to_host

    dev = torch.device("cuda:0")
    w = synth.get_workload(base).scaled(cfg_id=900 + base, batch=batch, n_layers=3, n_vis=n_vis, n_text=37, window=0,
                                        decode_steps=steps, jitter=0.1 if batch > 1 else 0.0)
    seqs = w.seqs()
    L, B, Hkv, G = w.n_layers, w.batch, w.n_kv_heads, w.group
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    extra = steps + 31
    k2 = [_roomy(li.k, extra, dev) for li in layers]
    v2 = [_roomy(li.v, extra, dev) for li in layers]
    pool = A.AirCache(config_for(w, retention, seqs=seqs, max_decode_steps=steps), dev)
    inpl = A.AirCache(config_for(w, retention, seqs=seqs, max_decode_steps=steps, cache_in_place=1), dev)
    use_static = bool(tuning and tuning.get("static"))
    if tuning:
        for ac in (pool, inpl):
            ac.air_set_tuning(**{k_: v_ for k_, v_ in tuning.items() if k_ != "static"})
    # the workspace of the in-place context holds no cache pool
    max_nonvis = max(s.seq_len - s.vis_len for s in seqs)
    kept = int(np.floor(retention * max(s.vis_len for s in seqs) * L + 0.5))
    pool_bytes = 2 * B * Hkv * (L * (max_nonvis + steps + 31) + kept) * w.head_dim * 2
    assert pool.workspace_bytes - inpl.workspace_bytes >= pool_bytes - 4096
    for ac, kk, vv in ((pool, k, v), (inpl, k2, v2)):
        ac.air_score(0, L, q, kk, vv, seqs)
        ac.air_budget()
    assert np.array_equal(pool.air_get_budgets(), inpl.air_get_budgets())
    pool.air_select_compact(0, L, k, v)
    inpl.air_select_compact(0, 2, k2[:2], v2[:2])  # in two calls: layer ranges work as on the pool path
    inpl.air_select_compact(2, L, k2[2:], v2[2:])
    bud = pool.air_get_budgets()
    lens = pool.air_get_lengths()
    assert np.array_equal(lens, inpl.air_get_lengths())
    for l in range(L):
        ia, ib = pool.air_get_indices(l), inpl.air_get_indices(l)
        for b, s in enumerate(seqs):
            assert np.array_equal(ia[b, :, : bud[b, l]], ib[b, :, : bud[b, l]])
            for h in range(Hkv):
                rows = O.compact_rows(P.seg_of(s), ia[b, h, : bud[b, l]])
                ka, va = pool.air_get_cache(l, b, h, len(rows))
                kb, vb = inpl.air_get_cache(l, b, h, len(rows))
                assert np.array_equal(ka, kb) and np.array_equal(va, vb), (l, b, h)
                assert np.array_equal(kb, layers[l].k[b, h][rows]) and np.array_equal(vb, layers[l].v[b, h][rows])
    out_a = torch.empty((L, B, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    out_b = torch.empty_like(out_a)
    for step in range(steps):
        qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
        qn, kn, vn = (to_device(np.stack(x), dev) for x in (qs, ks, vs))
        pool.air_decode_attn(0, L, qn, kn, vn, out_a)
        (inpl.air_decode_attn_static if use_static else inpl.air_decode_attn)(0, L, qn, kn, vn, out_b)
        torch.cuda.synchronize()
        assert not torch.isnan(out_b.float()).any()
        assert torch.equal(out_a, out_b), f"decode step {step}"
    lens = pool.air_get_lengths()
    assert np.array_equal(lens, inpl.air_get_lengths())
    for (l, b, h) in [(0, 0, 0), (L - 1, B - 1, Hkv - 1)]:
        ka, va = pool.air_get_cache(l, b, h, int(lens[b, l]))
        kb, vb = inpl.air_get_cache(l, b, h, int(lens[b, l]))
        assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    # and the last step agrees with the oracle's attention over those rows
    got = synth.storage_to_f64(to_host(out_b))
    q64 = synth.storage_to_f64(np.stack(qs))
    for (l, b, h) in [(0, 0, 0), (L - 1, B - 1, Hkv - 1)]:
        kb, vb = inpl.air_get_cache(l, b, h, int(lens[b, l]))
        want = O.decode_attn(q64[l, b, h * G:(h + 1) * G], synth.storage_to_f64(kb), synth.storage_to_f64(vb))
        assert np.abs(got[l, b, h * G:(h + 1) * G] - want).max() <= P.DECODE_ATOL["bf16"]
    pool.close()
    inpl.close()


def test_in_place_compaction_refusals():
    import ctypes as C

    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device

    dev = torch.device("cuda:0")
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=300, n_text=24, decode_steps=8)
    seqs = w.seqs()
    L = w.n_layers
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    ac = A.AirCache(config_for(w, 0.1, seqs=seqs, max_decode_steps=8, cache_in_place=1), dev)
    ac.air_score(0, L, q, k, v, seqs)
    ac.air_budget()
    before = [t.clone() for t in k]
    with pytest.raises(A.AirError) as e:  # no room for the appended tokens behind the prompt
        ac.air_select_compact(0, L, k, v)
    assert e.value.status == A.binding.AIR_ERR_SHAPE
    km = [t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in k]  # token-major: a head's rows are not contiguous
    with pytest.raises(A.AirError) as e:
        ac.air_select_compact(0, L, km, km)
    assert e.value.status == A.binding.AIR_ERR_SHAPE
    torch.cuda.synchronize()
    assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(before, k))  # nothing was written
    ac.close()
    # the in-place cache exists for the bf16 / head_dim 128 kernels only
    bad = A.make_config(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, batch=1, max_vis_len=576, max_nonvis_len=80,
                        max_window=16, max_decode_steps=1, dtype=A.AIR_F32, cache_in_place=1)
    assert A.load_library().air_workspace_bytes(C.byref(bad)) == 0
