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
    for mode in ("per_layer", "step_layers", "step_layers_fused", "step_layers_fold"):
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
                              {"step_layers": 0, "step_layers_fused": B.STEP_FUSE_ACROSS_LAYERS,
                               "step_layers_fold": B.STEP_FOLD_APPEND}[mode], None, stream)
        torch.cuda.synchronize()
        B.oxy_batch_destroy(batch)
        pools = []
        for sid in (0, 1):
            slots = gw.stream_slots(sid)
            pools.append([gw.gather(l, slots) for l in range(L)])
        results[mode] = (bits_of(o), lse.cpu().numpy(), pools)
        gw.close()
    a = results["per_layer"]
    for other in ("step_layers", "step_layers_fused", "step_layers_fold"):
        b = results[other]
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), other
        assert np.all(np.isfinite(b[1])) and np.any(b[0] != 0)
        for pa, pb in zip(a[2], b[2]):
            for (ka, va), (kb, vb) in zip(pa, pb):
                assert np.array_equal(ka, kb) and np.array_equal(va, vb), other
