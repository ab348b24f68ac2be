"""Shared helpers of the GPU parity tests: run one trace through the HIP path and through
the oracle on the same seeded bits, then compare element by element."""
import numpy as np

from oracle import attention
from oracle.replay import OracleWorld
from paper_2603_14371_amd import synth

# tolerance of the comparison for bf16 inputs, fp32 accumulation, bf16 output
O_ATOL, O_RTOL = 2e-3, 1e-2
LSE_ATOL, LSE_RTOL = 1e-3, 1e-3


def assert_o_close(gpu_bits, ref, what=""):
    got = attention.widen_bf16(gpu_bits)
    assert got.shape == ref.shape, what
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    err = np.abs(got - ref)
    bound = O_ATOL + O_RTOL * np.abs(ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.all(err <= bound), "%s: |err| %.3e > bound %.3e at %s (ref %.5f got %.5f)" % (
        what, err[worst], bound[worst], worst, ref[worst], got[worst])
    return float(err.max())


def assert_lse_close(gpu, ref, what=""):
    err = np.abs(gpu.astype(np.float64) - ref)
    bound = LSE_ATOL + LSE_RTOL * np.abs(ref)
    assert np.all(err <= bound), "%s: LSE |err| max %.3e" % (what, err.max())


def run_both(workload, layers=None, head_dim=None, data_fn=None, compare=True, oracle_steps=None,
             **gpu_kw):
    """Returns (gpu_world, gpu_results, oracle_world, oracle_results); the GPU world is left
    open for read-back and must be closed by the caller."""
    from paper_2603_14371_amd.harness import GpuWorld
    w = workload
    src = data_fn or synth.DataSource(w["seed"], w["sigma"])
    order = None if w["free_order"] is None else list(w["free_order"])
    ow = OracleWorld(w["num_blocks"], w["n_layers"], src, w["scale"], free_order=order,
                     layers=layers)
    gw = GpuWorld(w, src, layers=layers, **gpu_kw)
    g_res, o_res = [], []
    for i, op in enumerate(w["trace"]):
        g = gw.apply(op)
        if oracle_steps is not None and op["op"] == "step" and i not in oracle_steps:
            op_o = dict(op, attend=False)
        else:
            op_o = op
        o = ow.apply(op_o)
        g_res.append(g)
        o_res.append(o)
        if not compare:
            continue
        for key in ("pid", "sid", "slots"):
            if key in o:
                assert g[key] == o[key], "op %d (%s): %s differs" % (i, op["op"], key)
        if op["op"] == "step":
            for layer, ref in o["O"].items():
                assert_o_close(g["O"][layer], ref, "op %d layer %d" % (i, layer))
                if layer in g["LSE"]:
                    assert_lse_close(g["LSE"][layer], o["LSE"][layer], "op %d layer %d" % (i, layer))
    return gw, g_res, ow, o_res


def assert_pool_contents_equal(gw, ow):
    """Every live token of every live stream and prefix, read back through the library, has
    exactly the bits the oracle's un-paged lists hold."""
    from paper_2603_14371_amd import binding as B
    n = 0
    for sid, per_layer in ow.stream_kv.items():
        slots = gw.stream_slots(sid)
        for layer, (k, v) in per_layer.items():
            assert len(slots) == len(k)
            if len(slots) == 0:
                continue
            gk, gv = gw.gather(layer, slots)
            assert np.array_equal(gk, k) and np.array_equal(gv, v), "stream %d layer %d" % (sid, layer)
            n += len(slots)
    for pid in ow.pool.prefixes:
        slots = gw.prefix_slots(pid)
        for layer, (k, v) in ow.prefix_kv[pid].items():
            gk, gv = gw.gather(layer, slots)
            assert np.array_equal(gk, k) and np.array_equal(gv, v), "prefix %d layer %d" % (pid, layer)
            n += len(slots)
    return n
