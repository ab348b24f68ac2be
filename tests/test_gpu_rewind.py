"""Explicit roll-back of a language request (oxy_stream_rewind) followed by re-append and
attention -- what parallel / speculative decoding needs when drafted tokens are rejected
(Sec. 3.2, compatibility with parallel decoding) -- and a prefix append below the current
length, both against the float64 oracle on a NaN-filled pool, in both append modes."""
import numpy as np
import pytest

from paper_2603_14371_amd import synth
from paper_2603_14371_amd.synth import ACTION, DECODE, _TraceBuilder, _workload
from parity_util import assert_pool_contents_equal, run_both

pytestmark = pytest.mark.gpu


def _finish(gw, ow):
    try:
        return assert_pool_contents_equal(gw, ow)
    finally:
        gw.close()


def _rewind_trace():
    b = _TraceBuilder()
    pid = b.prefix(40)
    d0, d1, a0 = b.stream(pid, DECODE), b.stream(-1, DECODE), b.stream(pid, ACTION)
    b.step([(d0, 70), (d1, 9)], attend=False)         # histories; d0 crosses the 64-token split
    b.step([(d0, 1), (d1, 1), (a0, 5)])
    b.trace.append({"op": "stream_rewind", "sid": d0, "len": 61})   # 71 -> 61: back over the split
    b.step([(d0, 2), (d1, 1)])                        # positions 61, 62 rewritten
    for _ in range(3):                                # 63, 64, 65: across the split again
        b.step([(d0, 1), (d1, 1), (a0, 5)])
    b.trace.append({"op": "stream_rewind", "sid": d1, "len": 0})    # everything rejected
    b.trace.append({"op": "stream_rewind", "sid": d0, "len": 64})   # exactly onto the boundary
    b.step([(d1, 2), (d0, 2)])
    b.step([(d0, 1), (d1, 1)])
    b.trace.append({"op": "stream_rewind", "sid": d0, "len": 67})   # a rewind to the same length
    b.step([(d0, 1)])
    return _workload("rewind", 4711, 2, 64, b.trace)


@pytest.mark.parametrize("fold", [False, True], ids=["separate_append", "folded_append"])
def test_rewind_then_reappend_and_attend(fold):
    w = _rewind_trace()
    gw, g, ow, o = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True,
                            fold_append=fold)
    assert ow.pool.streams[0].length == 68 and ow.pool.streams[1].length == 3
    n = _finish(gw, ow)
    assert n == 2 * (40 + 68 + 3 + 5)


def test_rewind_modes_agree_bitwise():
    w = _rewind_trace()
    outs = []
    for fold in (False, True):
        gw, g, ow, _ = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True,
                                fold_append=fold, compare=False)
        gw.close()
        outs.append(g)
    for ra, rb in zip(*outs):
        for layer, x in ra.get("O", {}).items():
            assert np.array_equal(x, rb["O"][layer])


def test_prefix_append_below_the_length_overwrites_in_place():
    """Tokens [pos0, pos0+n) of an unsealed prefix are rewritten where they are (a partly
    covered page row by row, whole pages as pages); everything else keeps its bits."""
    b = _TraceBuilder()
    b.trace.append({"op": "prefix_create", "pid": 0})
    b.n_prefix = 1
    b.trace.append({"op": "prefix_append", "pid": 0, "n": 50, "pos0": 0, "data": b.recipe(50)})
    b.trace.append({"op": "prefix_append", "pid": 0, "n": 4, "pos0": 12, "data": b.recipe(4)})
    b.trace.append({"op": "prefix_append", "pid": 0, "n": 30, "pos0": 27, "data": b.recipe(30)})
    b.trace.append({"op": "prefix_append", "pid": 0, "n": 40, "pos0": 45, "data": b.recipe(40)})
    d0, a0 = b.stream(0, DECODE), b.stream(0, ACTION)
    b.step([(d0, 3), (a0, 4)])
    w = _workload("overwrite", 4712, 2, 64, b.trace)
    gw, g, ow, o = run_both(w, split_tokens=32, poison=True)
    assert ow.pool.prefixes[0].length == 85
    assert _finish(gw, ow) == 2 * (85 + 3 + 4)
