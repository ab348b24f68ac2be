"""The library's frame scheduler driving the HIP path, frame by frame, against the scheduling
oracle driving the float64 oracle: same steps, same slots, outputs within tolerance, pool
contents bit-exact.  Arrivals: several, one or no observation per frame; random lengths."""
import numpy as np
import pytest

from oracle import schedule as S
from oracle.pool_model import ACTION, DECODE
from oracle.replay import OracleWorld
from paper_2603_14371_amd import synth
from parity_util import assert_lse_close, assert_o_close, assert_pool_contents_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode,fold", [(S.BATCHED, True), (S.BATCHED, False), (S.UNBATCHED, True),
                                       (S.UPPER_BOUND, True)])
def test_scheduled_frames_match_the_oracle(mode, fold):
    from paper_2603_14371_amd import binding as B
    from paper_2603_14371_amd.harness import GpuWorld
    rng = np.random.default_rng(7 + mode)
    arrivals = [[int(rng.integers(1, 14)) for _ in range(int(rng.integers(0, 3)))] for _ in range(7)]
    arrivals[0] = [9, 3]
    arrivals += [[], []]
    k, s_act, chunk, max_active, prefix_len, nb = 4, 2, 11, 4, 72, 512
    w = synth._workload("sched", 4242, 2, nb, [], free_order=synth._perm(99, nb))
    src = synth.DataSource(w["seed"])
    gw = GpuWorld(w, src, max_q_tokens=64, max_append_tokens=128, split_tokens=32,
                  stream_split_tokens=32, fold_append=fold, poison=True)
    ow = OracleWorld(nb, 2, src, w["scale"], free_order=list(w["free_order"]))
    sched = B.oxy_sched_create(gw.pool, k, s_act, chunk, max_active, mode)
    expect = S.simulate(arrivals, k, s_act, mode, max_active)
    tag = [0]

    def recipe(n):
        tag[0] += 1
        return {"tag": tag[0], "tok0": 0, "n_total": n}

    sid_of, n_steps = {}, 0
    try:
        for t, targets in enumerate(arrivals):
            f = expect[t]
            act_sid, pids = [], []
            for n, want in zip(targets, f["admitted"]):
                pid = gw.apply({"op": "prefix_create"})["pid"]
                assert pid == ow.apply({"op": "prefix_create"})["pid"]
                op = {"op": "prefix_append", "pid": pid, "n": prefix_len, "pos0": 0,
                      "data": recipe(prefix_len)}
                assert gw.apply(op)["slots"] == ow.apply(op)["slots"]
                assert B.oxy_sched_admit(sched, pid, n) == want
                act_sid.append(ow.apply({"op": "stream_create", "pid": pid, "kind": ACTION})["sid"])
                if want >= 0:
                    sid_of[want] = ow.apply({"op": "stream_create", "pid": pid, "kind": DECODE})["sid"]
                pids.append(pid)
            for act, dec in f["steps"]:
                items, n_action = B.oxy_sched_next_step(sched)
                assert items == [(act_sid[p], chunk) for p in act] + [(sid_of[r], 1) for r in dec]
                op = {"op": "step", "items": items, "attend": True,
                      "data": recipe(sum(n for _, n in items))}
                g, o = gw.step(op), ow.apply(op)
                assert g["slots"] == o["slots"]
                for layer, ref in o["O"].items():
                    assert_o_close(g["O"][layer], ref, "frame %d layer %d" % (t, layer))
                    assert_lse_close(g["LSE"][layer], o["LSE"][layer], "frame %d" % t)
                n_steps += 1
            assert B.oxy_sched_next_step(sched) == ([], 0)
            assert B.oxy_sched_end_frame(sched) == f["finished"]
            for sid in act_sid:
                ow.apply({"op": "stream_release", "sid": sid})
            for r in f["finished"]:
                ow.apply({"op": "stream_release", "sid": sid_of[r]})
            for pid in pids:
                ow.apply({"op": "prefix_release", "pid": pid})
            assert B.oxy_free_blocks(gw.pool) == ow.pool.free[::-1]
            if t == 4:
                assert_pool_contents_equal(gw, ow)      # requests in flight, mid-run
        assert n_steps > 10
        B.oxy_sched_destroy(sched)
        assert B.oxy_pool_stats(gw.pool)[1:] == (0, 0)
    finally:
        gw.close()
