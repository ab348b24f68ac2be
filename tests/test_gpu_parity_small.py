"""GPU parity, small cases: the tiny configuration and its degenerate variants, element by
element against the float64 oracle through the C ABI; indexing and pool contents bit-exact."""
import os

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


def test_tiny_config():
    w = synth.tiny()
    gw, g, ow, o = run_both(w)
    assert g[-1]["O"][0].shape == (11, 8, 256)
    assert _finish(gw, ow) == 64 + 10 + 5


@pytest.mark.parametrize("kw", [
    dict(prefix_len=70),                      # partial last prefix page
    dict(prefix_len=0),                       # no prefix at all
    dict(prefix_len=33, chunk=1, prior=0),    # single-token everything
    dict(prefix_len=64, chunk=50, prior=40),  # several pages of own history, ragged tails
    dict(prefix_len=832, chunk=50, prior=300, n_layers=3),
    dict(sigma=1.0 / 16.0),                   # the other reading of "scaled by 1/sqrt(256)"
], ids=["p70", "p0", "single", "own40", "pi05_shape", "sigma16"])
def test_tiny_variants(kw):
    w = synth.tiny(**kw)
    gw, g, ow, o = run_both(w, split_tokens=64)
    _finish(gw, ow)


def test_nan_poisoned_pool():
    """Stale bits in unused slots (here: NaN everywhere) must never reach an output."""
    w = synth.tiny(prefix_len=70, chunk=13, prior=21)
    gw, g, ow, o = run_both(w, poison=True, split_tokens=32)
    _finish(gw, ow)


def test_multi_token_decode_queries_are_causal():
    """Several new decode tokens in one step: query r sees own tokens 0..p_r only."""
    from paper_2603_14371_amd.synth import _TraceBuilder, _workload, DECODE, ACTION
    b = _TraceBuilder()
    pid = b.prefix(40)
    d0, d1 = b.stream(pid, DECODE), b.stream(-1, DECODE)
    b.step([(d0, 7), (d1, 37)])
    b.step([(d1, 3), (d0, 5)])
    b.step([(d0, 70)])
    w = _workload("multi_token", 99, 2, 64, b.trace)
    gw, g, ow, o = run_both(w, split_tokens=32)
    _finish(gw, ow)


@pytest.mark.parametrize("tile,stream", [(512, 512), (1024, 1024), (32, 32), (96, 160)])
def test_split_sizes_including_block_table_fallback(tile, stream):
    """Splits longer than 16 pages take their block ids from the block table instead of the
    work record's inline copy; the shortest and odd sizes exercise ragged last splits."""
    w = synth.tiny(prefix_len=1100, chunk=37, prior=700, n_layers=2)
    gw, g, ow, o = run_both(w, split_tokens=tile, stream_split_tokens=stream, max_partials=4096)
    _finish(gw, ow)


@pytest.mark.parametrize("fold", [False, True], ids=["separate_append", "folded_append"])
def test_histories_around_page_step_and_split_boundaries(fold):
    """Decode streams whose own histories end just before, on and just after page (16), step
    (32) and split (64) boundaries, then take one and two new tokens; with and without a
    prefix whose last page is partial."""
    from paper_2603_14371_amd.synth import _TraceBuilder, _workload, DECODE, ACTION
    b = _TraceBuilder()
    pid = b.prefix(70)
    lens = [1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193]
    sids = [b.stream(pid if i % 2 == 0 else -1, DECODE) for i in range(len(lens))]
    b.step([(s, n) for s, n in zip(sids, lens)], attend=False)
    b.step([(s, 1) for s in sids])
    b.step([(s, 2) for s in sids])
    b.step([(s, 1) for s in sids[::-1]])
    w = _workload("boundaries", 515, 2, 512, b.trace)
    gw, g, ow, o = run_both(w, split_tokens=64, stream_split_tokens=64, poison=True,
                            fold_append=fold, max_partials=4096)
    _finish(gw, ow)


def test_a_query_that_sees_only_itself_returns_its_value_row():
    """No prefix, empty history, one new token: the visible set is the token itself, so O is
    its V row exactly (bf16 in, bf16 out) and LSE is its own logit."""
    from paper_2603_14371_amd.synth import _TraceBuilder, _workload, DECODE, ACTION
    b = _TraceBuilder()
    d, a = b.stream(-1, DECODE), b.stream(-1, ACTION)
    b.step([(d, 1), (a, 1)])
    w = _workload("self_only", 808, 1, 64, b.trace)
    gw, g, ow, o = run_both(w, fold_append=True)
    try:
        src = synth.DataSource(w["seed"], w["sigma"])
        v = src(w["trace"][-1]["data"], 0, "v", 2)
        for tok in range(2):
            for h in range(8):
                assert np.array_equal(g[-1]["O"][0][tok, h], v[tok])
    finally:
        gw.close()


def test_prefix_append_of_all_layers_in_one_call_equals_per_layer_calls():
    """oxy_prefix_append_layers (one launch for all layers, in two pieces with a ragged seam)
    leaves the pool exactly as the per-layer calls do."""
    import torch
    from paper_2603_14371_amd import binding as B
    from paper_2603_14371_amd.harness import GpuWorld, to_device_bf16
    w = synth._workload("prefix_layers", 909, 3, 128, [], free_order=synth._perm(910, 128))
    data = synth.DataSource(w["seed"])
    rec = {"tag": 1, "tok0": 0, "n_total": 333}
    pools = []
    for all_layers in (False, True):
        gw = GpuWorld(w, data, poison=True)
        L = gw.n_layers
        k = torch.stack([to_device_bf16(data(rec, l, "k", 333), gw.device) for l in range(L)])
        v = torch.stack([to_device_bf16(data(rec, l, "v", 333), gw.device) for l in range(L)])
        pid = B.oxy_prefix_create(gw.pool)
        stream = torch.cuda.current_stream(gw.device).cuda_stream
        for pos0, n in ((0, 200), (200, 133)):          # 200 = 12.5 pages: a ragged seam
            if all_layers:
                B.oxy_prefix_append_layers(gw.pool, pid, 0, L, k[0, pos0].data_ptr(),
                                           v[0, pos0].data_ptr(), k.stride(0) * 2, n, pos0, stream)
            else:
                for l in range(L):
                    B.oxy_prefix_append(gw.pool, pid, l, k[l, pos0].data_ptr(),
                                        v[l, pos0].data_ptr(), n, pos0, stream)
        torch.cuda.synchronize()
        slots = gw.prefix_slots(pid)
        assert len(slots) == 333
        pools.append([gw.gather(l, slots) for l in range(L)])
        for l in range(L):
            assert np.array_equal(pools[-1][l][0], data(rec, l, "k", 333))
            assert np.array_equal(pools[-1][l][1], data(rec, l, "v", 333))
        gw.close()
    for (ka, va), (kb, vb) in zip(*pools):
        assert np.array_equal(ka, kb) and np.array_equal(va, vb)
