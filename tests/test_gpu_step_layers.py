"""oxy_step_layers (the per-layer loop of one step below the ABI; optionally the merge of
layer l and the append of layer l+1 in one launch, or the append folded into the work items)
must give bit for bit what the per-layer calls give: outputs, LSE and pool contents."""
import numpy as np
import pytest

from paper_2603_14371_amd import synth

pytestmark = pytest.mark.gpu


def test_step_layers_equals_per_layer_calls():
    import torch
    from paper_2603_14371_amd import binding as B
    from paper_2603_14371_amd.harness import GpuWorld, bits_of, to_device_bf16
    w = synth.tiny(prefix_len=200, chunk=50, prior=77, n_layers=5)
    data = synth.DataSource(31337)
    results = {}
    flags_of = {"step_layers": 0, "step_layers_fused": B.STEP_FUSE_ACROSS_LAYERS,
                "step_layers_fold": B.STEP_FOLD_APPEND, "step_layers_graph": B.STEP_GRAPH,
                "step_layers_fused_graph": B.STEP_FUSE_ACROSS_LAYERS | B.STEP_GRAPH,
                "step_layers_fold_graph": B.STEP_FOLD_APPEND | B.STEP_GRAPH}
    for mode in ("per_layer",) + tuple(flags_of):
        gw = GpuWorld(w, data, split_tokens=64)
        gw.run(w["trace"][:-1])                     # everything but the final mixed step
        op = w["trace"][-1]
        n_tok = sum(n for _, n in op["items"])
        L = gw.n_layers
        k = torch.stack([to_device_bf16(data(op["data"], l, "k", n_tok), gw.device) for l in range(L)])
        v = torch.stack([to_device_bf16(data(op["data"], l, "v", n_tok), gw.device) for l in range(L)])
        q = torch.stack([to_device_bf16(data(op["data"], l, "q", n_tok), gw.device) for l in range(L)])
        o = torch.zeros_like(q)
        lse = torch.zeros((L, n_tok, 8), dtype=torch.float32, device=gw.device)
        stream = torch.cuda.current_stream(gw.device).cuda_stream
        batch = B.oxy_batch_build(gw.pool, op["items"], 0, stream)
        if mode == "per_layer":
            for l in range(L):
                B.oxy_stream_append(gw.pool, batch, l, k[l].data_ptr(), v[l].data_ptr(), stream)
                B.oxy_mixed_attention(gw.pool, batch, l, q[l].data_ptr(), o[l].data_ptr(),
                                      lse[l].data_ptr(), gw.scale, stream)
        else:
            B.oxy_step_layers(gw.pool, batch, 0, L, k.data_ptr(), v.data_ptr(), k.stride(0) * 2,
                              q.data_ptr(), o.data_ptr(), q.stride(0) * 2, lse.data_ptr(),
                              lse.stride(0) * 4, gw.scale,
                              flags_of[mode], None, stream)
        torch.cuda.synchronize()
        B.oxy_batch_destroy(batch)
        pools = []
        for sid in (0, 1):
            slots = gw.stream_slots(sid)
            pools.append([gw.gather(l, slots) for l in range(L)])
        results[mode] = (bits_of(o), lse.cpu().numpy(), pools)
        gw.close()
    a = results["per_layer"]
    for other in flags_of:
        b = results[other]
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), other
        assert np.all(np.isfinite(b[1])) and np.any(b[0] != 0)
        for pa, pb in zip(a[2], b[2]):
            for (ka, va), (kb, vb) in zip(pa, pb):
                assert np.array_equal(ka, kb) and np.array_equal(va, vb), other


@pytest.mark.parametrize("fold", [True, False], ids=["folded_append", "separate_append"])
def test_recorded_steps_replayed_over_a_decode_loop(fold):
    """OXY_STEP_GRAPH over a whole frame with resident buffers: 4 mixed steps, then decode-only
    steps whose own history crosses split boundaries (new work items -> a new recording) and
    block boundaries (longer tables, same recording).  Between replays the program does eager
    work of its own (refilling the resident inputs, reading the outputs back, synchronising).
    Every step's outputs, LSE and the final pool contents equal the unrecorded run's bits."""
    import torch
    from paper_2603_14371_amd import binding as B
    from paper_2603_14371_amd.harness import GpuWorld, bits_of, to_device_bf16
    w = synth.pi05_frame(n_layers=3, prefix_len=200, chunk=50, denoise_steps=4, decode_tokens=150)
    data = synth.DataSource(2718)
    steps = [op for op in w["trace"] if op["op"] == "step"]
    first = w["trace"].index(steps[0])
    base = B.STEP_FOLD_APPEND if fold else 0
    outs = {}
    for graph in (False, True):
        gw = GpuWorld(w, data, stream_split_tokens=64)
        gw.run(w["trace"][:first])
        L = gw.n_layers
        stream = torch.cuda.current_stream(gw.device).cuda_stream
        res = []
        bufs = {}
        for op in steps:
            n_tok = sum(n for _, n in op["items"])
            if n_tok not in bufs:       # resident buffers per batch shape, as a serving loop has
                mk = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16, device=gw.device)
                bufs[n_tok] = (mk(L, n_tok, 256), mk(L, n_tok, 256), mk(L, n_tok, 8, 256),
                               mk(L, n_tok, 8, 256),
                               torch.zeros((L, n_tok, 8), dtype=torch.float32, device=gw.device))
            k, v, q, o, lse = bufs[n_tok]
            for l in range(L):
                k[l].copy_(to_device_bf16(data(op["data"], l, "k", n_tok), gw.device))
                v[l].copy_(to_device_bf16(data(op["data"], l, "v", n_tok), gw.device))
                q[l].copy_(to_device_bf16(data(op["data"], l, "q", n_tok), gw.device))
            o.zero_()
            batch = B.oxy_batch_build(gw.pool, op["items"], 0, stream)
            B.oxy_step_layers(gw.pool, batch, 0, L, k.data_ptr(), v.data_ptr(), k.stride(0) * 2,
                              q.data_ptr(), o.data_ptr(), q.stride(0) * 2, lse.data_ptr(),
                              lse.stride(0) * 4, gw.scale, base | (B.STEP_GRAPH if graph else 0),
                              None, stream)
            B.oxy_batch_destroy(batch)
            torch.cuda.synchronize()
            res.append((bits_of(o), lse.cpu().numpy().copy()))
        inst, upd, rep = B.oxy_step_graph_stats(gw.pool)
        if graph:
            # one recording per batch shape (mixed, decode-only): the grid is padded to 64 work
            # items, so crossing a split boundary does not change the launch shape here
            assert rep == len(steps) and inst == 2 and upd == 0, (inst, upd, rep)
        else:
            assert (inst, upd, rep) == (0, 0, 0)
        pool = [gw.gather(l, gw.stream_slots(1)) for l in range(L)]
        outs[graph] = (res, pool)
        gw.close()
    for i, ((o0, l0), (o1, l1)) in enumerate(zip(outs[False][0], outs[True][0])):
        assert np.array_equal(o0, o1) and np.array_equal(l0, l1), "step %d" % i
        assert np.any(o0 != 0) and np.all(np.isfinite(l0))
    for (ka, va), (kb, vb) in zip(outs[False][1], outs[True][1]):
        assert np.array_equal(ka, kb) and np.array_equal(va, vb)


def test_recordings_beyond_the_cache_are_updated_in_place():
    """Eleven forms of the same step (eleven output buffers) against a cache of eight
    recordings: the ninth to eleventh re-record and update an instantiated graph in place.
    Every one of them, and a second round over all eleven, gives the unrecorded bits."""
    import torch
    from paper_2603_14371_amd import binding as B
    from paper_2603_14371_amd.harness import GpuWorld, bits_of, to_device_bf16
    w = synth.tiny(prefix_len=300, chunk=50, prior=90, n_layers=3)
    data = synth.DataSource(1618)
    gw = GpuWorld(w, data)
    try:
        gw.run(w["trace"][:-1])
        op = w["trace"][-1]
        n_tok = sum(n for _, n in op["items"])
        L = gw.n_layers
        k, v, q = (torch.stack([to_device_bf16(data(op["data"], l, what, n_tok), gw.device)
                                for l in range(L)]) for what in "kvq")
        stream = torch.cuda.current_stream(gw.device).cuda_stream
        batch = B.oxy_batch_build(gw.pool, op["items"], 0, stream)

        def run(o, flags):
            B.oxy_step_layers(gw.pool, batch, 0, L, k.data_ptr(), v.data_ptr(), k.stride(0) * 2,
                              q.data_ptr(), o.data_ptr(), q.stride(0) * 2, 0, 0, gw.scale, flags,
                              None, stream)
            torch.cuda.synchronize()
            return bits_of(o)

        ref = run(torch.zeros_like(q), B.STEP_FOLD_APPEND)
        assert np.any(ref != 0)
        outs = [torch.zeros_like(q) for _ in range(11)]
        for rnd in range(2):
            for i, o in enumerate(outs):
                o.zero_()
                got = run(o, B.STEP_FOLD_APPEND | B.STEP_GRAPH)
                assert np.array_equal(got, ref), "round %d form %d" % (rnd, i)
        inst, upd, rep = B.oxy_step_graph_stats(gw.pool)
        assert inst == 8 and upd == 3 + 11 and rep == 22, (inst, upd, rep)
        B.oxy_batch_destroy(batch)
    finally:
        gw.close()
