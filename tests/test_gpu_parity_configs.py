"""GPU parity on the five workload configurations (through the C ABI, element by element
against the float64 oracle on the same seeded bits), at their real geometry: 8 q heads over
1 kv head, head_dim 256, page 16, 832- and 2048-token prefixes, 50-query chunks."""
import numpy as np
import pytest

from paper_2603_14371_amd import synth
from parity_util import assert_pool_contents_equal, run_both

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fold", [False, True], ids=["separate_append", "folded_append"])
def test_config1_pi05_frame_all_64_steps_two_layers(fold):
    w = synth.pi05_frame()
    gw, g, ow, o = run_both(w, layers=[0, 17], fold_append=fold)
    gw.close()
    steps = [r for op, r in zip(w["trace"], g) if op["op"] == "step"]
    assert len(steps) == 64 and steps[0]["O"][17].shape == (51, 8, 256)
    assert steps[-1]["O"][0].shape == (1, 8, 256)


def test_config2_cross_frame_continuous_batching():
    """Streams born in different frames keep the prefix of their birth frame and resume
    across frames; random block placement."""
    w = synth.cross_frame(n_frames=10, targets=[16, 37, 24, 55, 18, 70, 21, 33])
    steps = [i for i, op in enumerate(w["trace"]) if op["op"] == "step"]
    chosen = set(steps[::7]) | set(steps[-3:])
    gw, g, ow, o = run_both(w, layers=[5], oracle_steps=chosen)
    try:
        assert_pool_contents_equal(gw, ow)
    finally:
        gw.close()
    sizes = [len(w["trace"][i]["items"]) for i in steps]
    assert max(sizes) >= 4          # an action chunk plus several carried-over requests


def test_config3_shared_equals_isolated_bitwise_and_matches_oracle():
    """Sec. 1 / Sec. 3.2: fanning one prefill cache out to four tasks gives what four isolated
    runs with their own prefix copies give.  On the GPU the split of a query's keys depends
    only on its own lengths, so the two runs agree bit for bit."""
    kw = dict(n_steps=40)
    shared, iso = synth.cross_task(**kw), synth.cross_task(isolated=True, **kw)
    for w in (shared, iso):         # stop before the releases so that peak block use is visible
        w["trace"] = [op for op in w["trace"] if "release" not in op["op"]]
    s_steps = [i for i, op in enumerate(shared["trace"]) if op["op"] == "step"]
    gw, gs, ow, os_ = run_both(shared, layers=[2, 9], oracle_steps=set(s_steps[::6]))
    shared_blocks = gw.w["num_blocks"] - gw_free(gw)
    gw.close()
    gw, gi, _, _ = run_both(iso, layers=[2, 9], oracle_steps=set())
    iso_blocks = gw.w["num_blocks"] - gw_free(gw)
    gw.close()
    by_step = {}
    for op, r in zip(iso["trace"], gi):
        if op["op"] == "step":
            by_step.setdefault(op["shared_step"], []).append(r)
    n = 0
    for op, r in zip(shared["trace"], gs):
        if op["op"] != "step":
            continue
        for layer in (2, 9):
            cat = np.concatenate([x["O"][layer] for x in by_step[op["shared_step"]]])
            assert np.array_equal(cat, r["O"][layer]), "step %d layer %d" % (op["shared_step"], layer)
            n += 1
    assert n == 80
    assert iso_blocks - shared_blocks == 3 * 52       # three redundant copies of the prefix


def gw_free(gw):
    from paper_2603_14371_amd import binding as B
    return B.oxy_pool_stats(gw.pool)[0]


@pytest.mark.parametrize("fold", [True, False], ids=["folded_append", "separate_append"])
def test_config4_stress_full_size_every_item_against_oracle(fold):
    """Full stress geometry in the launch configuration the benchmark times (default split, the
    new rows appended by the work items; and with the separate append): 64 streams, histories
    ~U{1..2048}, 8 shared 2048-token prefixes, fragmented pool.  Every one of the 66 items of
    every mixed step is compared with the oracle, outputs and log-sum-exp, on the first and the
    last layer; indexing is compared op by op over the whole trace inside run_both."""
    w = synth.stress(n_layers=18, mixed_steps=2)
    layers = [0, 17]
    gw, g, ow, o = run_both(w, layers=layers, want_lse=True, fold_append=fold)
    try:
        mixed = [(op, r, ro) for op, r, ro in zip(w["trace"], g, o)
                 if op["op"] == "step" and op.get("attend", True)]
        assert len(mixed) == 2
        for op, r, ro in mixed:
            assert len(op["items"]) == 66
            for layer in layers:
                assert r["O"][layer].shape == (164, 8, 256) and layer in ro["O"]
        # pool contents of the longest and the shortest histories, bit-exact
        items = w["trace"][-1]["items"]
        lens = [len(ow.stream_kv[sid][0][0]) for sid, _ in items]
        for i in (int(np.argmax(lens)), int(np.argmin(lens[2:])) + 2, 2, 65):
            sid = items[i][0]
            gk, gv = gw.gather(17, gw.stream_slots(sid))
            assert np.array_equal(gk, ow.stream_kv[sid][17][0])
            assert np.array_equal(gv, ow.stream_kv[sid][17][1])
    finally:
        gw.close()


def test_config2_cross_frame_full_lengths():
    """Config 2 at its stated sizes: 40 frames, 8 request slots, targets ~U{16..512}, 10 tokens
    per frame, a fresh 832-token prefix and a 50-query chunk every frame, shuffled free order.
    Requests live for up to 39 frames on the prefix of their birth frame; their own histories
    grow past one 256-token split while that prefix is many frames old.  One layer; the oracle
    attends on every 13th step and on the last three, indexing is compared on every op."""
    w = synth.cross_frame(n_frames=40)
    steps = [i for i, op in enumerate(w["trace"]) if op["op"] == "step"]
    assert len(steps) == 400 and max(len(w["trace"][i]["items"]) for i in steps) == 9
    chosen = set(steps[::13]) | set(steps[-3:])
    gw, g, ow, o = run_both(w, layers=[5], oracle_steps=chosen, fold_append=True)
    try:
        longest = max(len(kv[5][0]) for kv in ow.stream_kv.values())
        assert longest > 256
        assert_pool_contents_equal(gw, ow)
    finally:
        gw.close()


def test_config3_full_384_steps_shared_against_oracle_and_isolated():
    """Config 3 at full length: 10 mixed steps, then decode down to the 384-token planning
    stream alone.  One layer; oracle on every 16th step and the last two; the isolated run
    (four private prefix copies, one batch per task) must give the same bits on every step."""
    shared, iso = synth.cross_task(), synth.cross_task(isolated=True)
    s_steps = [i for i, op in enumerate(shared["trace"]) if op["op"] == "step"]
    assert len(s_steps) == 384
    chosen = set(s_steps[::16]) | set(s_steps[-2:])
    gw, gs, ow, os_ = run_both(shared, layers=[9], oracle_steps=chosen, fold_append=True)
    gw.close()
    gw, gi, _, _ = run_both(iso, layers=[9], oracle_steps=set(), fold_append=True)
    gw.close()
    by_step = {}
    for op, r in zip(iso["trace"], gi):
        if op["op"] == "step":
            by_step.setdefault(op["shared_step"], []).append(r)
    n = 0
    for op, r in zip(shared["trace"], gs):
        if op["op"] == "step":
            cat = np.concatenate([x["O"][9] for x in by_step[op["shared_step"]]])
            assert np.array_equal(cat, r["O"][9]), "step %d" % op["shared_step"]
            n += 1
    assert n == 384


def test_config4_reduced_every_item_against_oracle():
    w = synth.stress(n_layers=2, n_streams=16, group=4, prefix_len=300, hist_hi=400,
                     num_blocks=2048, churn_ops=300, mixed_steps=2)
    gw, g, ow, o = run_both(w, layers=[1], split_tokens=96)
    try:
        assert_pool_contents_equal(gw, ow)
    finally:
        gw.close()
