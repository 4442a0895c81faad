"""A decode step recorded into a HIP graph and replayed: with device-counted steps every replay appends
its token and attends over the longer cache, exactly as the host-counted eager calls do."""
import numpy as np
import pytest

import synth
from oracle import aircache_oracle as O
from tests import parity_util as P

pytestmark = pytest.mark.gpu


def _contexts(w, steps, dev):
    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import config_for, to_device

    seqs = w.seqs()
    L = w.n_layers
    layers = [synth.layer_inputs(w, l, seqs) for l in range(L)]
    q = [to_device(li.q_text, dev) for li in layers]
    k = [to_device(li.k, dev) for li in layers]
    v = [to_device(li.v, dev) for li in layers]
    eager = A.AirCache(config_for(w, 0.10, max_decode_steps=steps, seqs=seqs), dev)
    counted = A.AirCache(config_for(w, 0.10, max_decode_steps=steps, seqs=seqs, device_steps=1), dev)

    def compress(ac, compact=True):
        ac.air_reset()
        ac.air_score(0, L, q, k, v, seqs)
        ac.air_budget()
        if compact:
            ac.air_select_compact(0, L, k, v)

    compress(eager)
    compress(counted)
    return A, eager, counted, compress, seqs, layers


@pytest.mark.parametrize("shape", [(1, 8, 4, 0), (4, 4, 4, 0), (1, 4, 4, 2), None])
def test_replayed_decode_step_matches_eager_calls(shape):
    import torch

    from paper_2503_23956_amd.device_inputs import to_device, to_host

    dev = torch.device("cuda:0")
    steps = 37  # crosses a 32-token block of the cache
    w = synth.get_workload(2).scaled(n_layers=3, n_vis=900, n_text=40, decode_steps=steps)
    A, eager, counted, compress, seqs, layers = _contexts(w, steps, dev)
    if shape is not None:  # the same launch shape on both sides makes the outputs bitwise comparable
        for ac in (eager, counted):
            # shape[3] = 2: two workgroups per unit that meet at the unit's arrival counter to advance the device-side count
            ac.air_set_tuning(decode_splits=shape[0], decode_waves=shape[1], decode_tiles=shape[2], decode_halves=shape[3])
    L, B, Hkv, G, d = w.n_layers, w.batch, w.n_kv_heads, w.group, w.head_dim
    ins = []
    for step in range(steps):
        qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
        ins.append(tuple(to_device(np.stack(x), dev) for x in (qs, ks, vs)))
    sq, sk, sv = (torch.empty_like(x) for x in ins[0])
    sout = torch.zeros((L, B, w.n_q_heads, d), dtype=sq.dtype, device=dev)
    out_e = torch.empty_like(sout)

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):  # recording runs nothing: the cache does not move
        counted.air_decode_attn(0, L, sq, sk, sv, sout)
    assert np.array_equal(counted.air_get_lengths(), eager.air_get_lengths())

    def run_steps(n):
        for step in range(n):
            for dst, src in zip((sq, sk, sv), ins[step]):
                dst.copy_(src)
            g.replay()
            eager.air_decode_attn(0, L, *ins[step], out_e)  # eager work between the replays
            torch.cuda.synchronize()
            if shape is not None:
                assert torch.equal(sout, out_e), f"step {step}"
            else:
                diff = (sout.float() - out_e.float()).abs().max().item()
                assert diff <= 1e-2, f"step {step}: {diff}"
        assert np.array_equal(counted.air_get_lengths(), eager.air_get_lengths())

    run_steps(steps)
    # the replayed cache holds the same rows as the eager one, and the oracle's attention over it agrees
    lens = eager.air_get_lengths()
    got = synth.storage_to_f64(to_host(sout))
    q64 = synth.storage_to_f64(to_host(ins[steps - 1][0]))
    for (l, b, h) in [(0, 0, 0), (L - 1, B - 1, Hkv - 1)]:
        kc, vc = counted.air_get_cache(l, b, h, int(lens[b, l]))
        ke, ve = eager.air_get_cache(l, b, h, int(lens[b, l]))
        assert np.array_equal(kc, ke) and np.array_equal(vc, ve)
        want = O.decode_attn(q64[l, b, h * G:(h + 1) * G], synth.storage_to_f64(kc), synth.storage_to_f64(vc))
        assert np.abs(got[l, b, h * G:(h + 1) * G] - want).max() <= P.DECODE_ATOL[w.dtype]

    # one replay past the capacity: nothing is appended, the output stays, the getter reports it
    before = sout.clone()
    g.replay()
    torch.cuda.synchronize()
    assert torch.equal(sout, before)
    with pytest.raises(A.AirError) as e:
        counted.air_get_lengths()
    assert e.value.status == A.binding.AIR_ERR_STATE

    # a new prompt: before its compaction the lengths are the bare ones (the old counts and the flag are not its own)
    compress(eager, compact=False)
    compress(counted, compact=False)
    assert np.array_equal(counted.air_get_lengths(), eager.air_get_lengths())
    # compacting again starts the count at zero and lowers the flag; the same recorded step serves the new cache
    compress(eager)
    compress(counted)
    assert np.array_equal(counted.air_get_lengths(), eager.air_get_lengths())
    run_steps(3)
    eager.close()
    counted.close()


def test_device_counted_steps_without_a_graph_and_config_limits():
    import ctypes as C

    import torch

    import paper_2503_23956_amd as A
    from paper_2503_23956_amd.device_inputs import to_device

    dev = torch.device("cuda:0")
    steps = 5
    w = synth.get_workload(2).scaled(n_layers=2, n_vis=400, n_text=24, decode_steps=steps)
    A, eager, counted, compress, seqs, layers = _contexts(w, steps, dev)
    L = w.n_layers
    out_e = torch.empty((L, w.batch, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    out_c = torch.empty_like(out_e)
    for step in range(steps):  # plain calls count on the device as well; layer by layer here
        qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
        qn, kn, vn = (to_device(np.stack(x), dev) for x in (qs, ks, vs))
        eager.air_decode_attn(0, L, qn, kn, vn, out_e)
        for l in range(L):
            counted.air_decode_attn(l, l + 1, qn[l:l + 1], kn[l:l + 1], vn[l:l + 1], out_c[l:l + 1])
        torch.cuda.synchronize()
        assert (out_c.float() - out_e.float()).abs().max().item() <= 1e-2
    assert np.array_equal(counted.air_get_lengths(), eager.air_get_lengths())
    with pytest.raises(A.AirError):  # a layer that has been decoded on cannot be compacted again without a reset
        counted.air_select_compact(0, L, [to_device(li.k, dev) for li in layers], [to_device(li.v, dev) for li in layers])
    # device-counted steps exist for the bf16 / head_dim 128 kernels only
    lib = A.load_library()
    bad = A.make_config(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, batch=1, max_vis_len=576, max_nonvis_len=80,
                        max_window=16, max_decode_steps=1, dtype=A.AIR_F32, device_steps=1)
    assert lib.air_workspace_bytes(C.byref(bad)) == 0
    eager.close()
    counted.close()


def test_layers_out_of_step_in_one_call():
    """A call whose layers have appended different numbers of tokens (layer 0 was decoded on once more than the
    rest) carries the per-layer counts with the launch; it must give what layer-by-layer calls give."""
    import torch

    from paper_2503_23956_amd.device_inputs import to_device

    dev = torch.device("cuda:0")
    w = synth.get_workload(2).scaled(n_layers=3, n_vis=500, n_text=24, decode_steps=4)
    A, one, ref, compress, seqs, layers = _contexts(w, 4, dev)  # `ref` counts on the device; used layer by layer here
    L = w.n_layers
    steps = []
    for step in range(2):
        qs, ks, vs = zip(*[synth.decode_inputs(w, l, step) for l in range(L)])
        steps.append(tuple(to_device(np.stack(x), dev) for x in (qs, ks, vs)))
    shape = (L, w.batch, w.n_q_heads, w.head_dim)
    out_a = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
    out_b = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
    # layer 0 alone first, then all layers in one call: layer 0 gets its second token, the others their first
    one.air_decode_attn(0, 1, steps[0][0][:1], steps[0][1][:1], steps[0][2][:1], out_a[:1])
    mixed = tuple(torch.cat([steps[1][i][:1], steps[0][i][1:]]) for i in range(3))
    one.air_decode_attn(0, L, *mixed, out_a)
    # reference: the same tokens layer by layer
    ref.air_decode_attn(0, 1, steps[0][0][:1], steps[0][1][:1], steps[0][2][:1], out_b[:1])
    for l in range(L):
        ref.air_decode_attn(l, l + 1, mixed[0][l:l + 1], mixed[1][l:l + 1], mixed[2][l:l + 1], out_b[l:l + 1])
    torch.cuda.synchronize()
    assert (out_a.float() - out_b.float()).abs().max().item() <= 1e-2
    la, lb = one.air_get_lengths(), ref.air_get_lengths()
    s0 = seqs[0]
    appended = la[0] - (s0.seq_len - s0.vis_len) - one.air_get_budgets()[0]
    assert np.array_equal(la, lb) and appended.tolist() == [2, 1, 1]
    one.close()
    ref.close()
