"""The append folded into the attention work items (oxy_append_attention, and
OXY_STEP_FOLD_APPEND of oxy_step_layers): outputs against the float64 oracle, pool contents
bit-exact, and bit for bit what the separate append + attention calls give."""
import numpy as np
import pytest

from paper_2603_14371_amd import synth
from parity_util import assert_pool_contents_equal, run_both

pytestmark = pytest.mark.gpu


def _finish(gw, ow):
    try:
        return assert_pool_contents_equal(gw, ow)
    finally:
        gw.close()


def _same_bits(a, b):
    for ra, rb in zip(a, b):
        for layer, o in ra.get("O", {}).items():
            assert np.array_equal(o, rb["O"][layer])
            assert np.array_equal(ra["LSE"][layer], rb["LSE"][layer])


@pytest.mark.parametrize("kw", [
    dict(),
    dict(prefix_len=70, chunk=13, prior=21),
    dict(prefix_len=0, chunk=3, prior=0),
    dict(prefix_len=33, chunk=1, prior=0),        # an action chunk on the streaming path
    dict(prefix_len=832, chunk=50, prior=300, n_layers=3),
    dict(prefix_len=64, chunk=150, prior=255),    # chunk over several splits and tiles
], ids=["tiny", "ragged", "p0", "single", "pi05_shape", "long_chunk"])
def test_folded_append_matches_oracle_and_separate_calls(kw):
    w = synth.tiny(**kw)
    gw, g_fold, ow, _ = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True,
                                 fold_append=True)
    _finish(gw, ow)
    gw, g_sep, ow, _ = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True)
    _finish(gw, ow)
    _same_bits(g_sep, g_fold)


def test_folded_append_two_token_decode_across_a_split_boundary_and_fallback():
    """Two new decode tokens whose positions fall into different splits are written by
    different work items; a multi-token decode step on a non-empty history is not covered by the
    folded form and must silently take the separate append."""
    from paper_2603_14371_amd.synth import _TraceBuilder, _workload, DECODE, ACTION
    b = _TraceBuilder()
    pid = b.prefix(40)
    d0, d1, a0 = b.stream(pid, DECODE), b.stream(-1, DECODE), b.stream(pid, ACTION)
    b.step([(d0, 63), (d1, 2), (a0, 2)])          # fresh multi-token decode, tiny action chunk
    b.step([(d0, 2), (d1, 2), (a0, 9)])           # d0: positions 63 | 64 straddle the 64-split
    b.step([(d0, 1), (d1, 1)])
    b.step([(d0, 5), (d1, 2)])                    # d0: 5 new tokens on history -> fallback
    b.step([(d1, 1), (a0, 70)])
    w = _workload("fold_mix", 77, 2, 64, b.trace)
    gw, g_fold, ow, _ = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True,
                                 fold_append=True)
    _finish(gw, ow)
    gw, g_sep, ow, _ = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True)
    _finish(gw, ow)
    _same_bits(g_sep, g_fold)


@pytest.mark.parametrize("chunk", [31, 33, 50, 64, 65])
def test_chunks_around_the_single_step_rule(chunk):
    """A chunk of at most 64 tokens on an empty history is evaluated in single 32-key steps (one
    or two split results per token), a longer one in the pool's usual splits; both next to a
    decode item, with the pool's default split sizes, in both append modes."""
    from paper_2603_14371_amd.synth import _TraceBuilder, _workload, DECODE, ACTION
    b = _TraceBuilder()
    pid = b.prefix(200)
    d0, a0, a1 = b.stream(pid, DECODE), b.stream(pid, ACTION), b.stream(-1, ACTION)
    b.step([(d0, 1), (a0, chunk), (a1, chunk)])
    b.step([(d0, 2), (a0, chunk)])
    w = _workload("chunk_rule", 4100 + chunk, 2, 96, b.trace)
    gw, g_fold, ow, _ = run_both(w, poison=True, fold_append=True)
    _finish(gw, ow)
    gw, g_sep, ow, _ = run_both(w, poison=True)
    _finish(gw, ow)
    _same_bits(g_sep, g_fold)


def test_folded_append_reduced_stress_every_item():
    w = synth.stress(n_layers=2, n_streams=16, group=4, prefix_len=300, hist_hi=400,
                     num_blocks=2048, churn_ops=300, mixed_steps=2)
    gw, g, ow, o = run_both(w, layers=[1], split_tokens=96, fold_append=True)
    _finish(gw, ow)
