"""Prefixes of consecutive frames that share a history segment through forked block tables:
outputs against the float64 oracle, pool contents bit-exact, and bit for bit what prefixes
holding private copies of the same tokens give."""
import numpy as np
import pytest

from paper_2603_14371_amd import synth
from paper_2603_14371_amd.synth import ACTION, DECODE
from parity_util import assert_pool_contents_equal, run_both

pytestmark = pytest.mark.gpu


def _trace(fork):
    r0 = {"tag": 100, "tok0": 0, "n_total": 208}
    r1 = {"tag": 101, "tok0": 0, "n_total": 80}
    r2 = {"tag": 102, "tok0": 0, "n_total": 50}
    tag = [200]

    def step(items):
        tag[0] += 1
        return {"op": "step", "items": items, "attend": True,
                "data": {"tag": tag[0], "tok0": 0, "n_total": sum(n for _, n in items)}}

    t = [{"op": "prefix_create", "pid": 0},
         {"op": "prefix_append", "pid": 0, "n": 208, "pos0": 0, "data": r0},
         {"op": "stream_create", "pid": 0, "kind": DECODE, "sid": 0},
         step([(0, 3)])]
    # frame 1: first 128 tokens are frame 0's, then 80 of its own
    if fork:
        t.append({"op": "prefix_fork", "parent": 0, "n": 128, "pid": 1})
    else:
        t += [{"op": "prefix_create", "pid": 1},
              {"op": "prefix_append", "pid": 1, "n": 128, "pos0": 0, "data": r0}]
    t += [{"op": "prefix_append", "pid": 1, "n": 80, "pos0": 128, "data": r1},
          {"op": "stream_create", "pid": 1, "kind": ACTION, "sid": 1},
          {"op": "stream_create", "pid": 1, "kind": DECODE, "sid": 2},
          step([(1, 13), (0, 1), (2, 1)]),
          {"op": "prefix_release", "pid": 0},
          {"op": "stream_release", "sid": 0}]     # frame 0's own tail blocks return to the stack
    # frame 2: first 160 tokens are frame 1's (128 of them came from frame 0), then 50 new
    if fork:
        t.append({"op": "prefix_fork", "parent": 1, "n": 160, "pid": 2})
    else:
        t += [{"op": "prefix_create", "pid": 2},
              {"op": "prefix_append", "pid": 2, "n": 128, "pos0": 0, "data": r0},
              {"op": "prefix_append", "pid": 2, "n": 32, "pos0": 128, "data": r1}]
    t += [{"op": "prefix_append", "pid": 2, "n": 50, "pos0": 160, "data": r2},
          {"op": "stream_create", "pid": 2, "kind": ACTION, "sid": 3},
          {"op": "stream_create", "pid": 2, "kind": DECODE, "sid": 4},
          step([(3, 13), (2, 1), (4, 2)]),
          {"op": "stream_release", "sid": 1},
          {"op": "prefix_release", "pid": 1},
          step([(3, 13), (2, 1), (4, 1)])]
    return t


def test_forked_prefixes_match_the_oracle_and_private_copies():
    outs = {}
    for fork in (True, False):
        w = synth._workload("fork", 5150, 2, 96, _trace(fork), free_order=synth._perm(5151, 96))
        gw, g, ow, o = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True,
                                fold_append=True)
        try:
            assert_pool_contents_equal(gw, ow)
            if fork:
                from paper_2603_14371_amd import binding as B
                b1, b2 = B.oxy_prefix_blocks(gw.pool, 1), B.oxy_prefix_blocks(gw.pool, 2)
                assert b1[:10] == b2[:10] and b1[10:] != b2[10:13]
                with pytest.raises(B.OxyError) as e:          # the shared range is read-only
                    B.oxy_prefix_append(gw.pool, 2, 0, gw.kv.data_ptr(), gw.kv.data_ptr(), 1, 100, 0)
                assert e.value.code == B.ERR_SEALED
        finally:
            gw.close()
        outs[fork] = [(r["O"], r["LSE"]) for r in g if "O" in r]
    for (oa, la), (ob, lb) in zip(outs[True], outs[False]):
        for layer in oa:
            assert np.array_equal(oa[layer], ob[layer]) and np.array_equal(la[layer], lb[layer])
