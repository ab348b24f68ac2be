"""Invariants of the method, checked on the oracle's replay of operation traces: shared
prefix == isolated per-task copies, the action expert's view never sees language appends,
batch independence, frame-chop invariance, placement independence.  No GPU."""
import numpy as np

from oracle import attention, brute
from oracle.pool_model import ACTION, DECODE
from oracle.replay import OracleWorld
from paper_2603_14371_amd import synth


def _replay(w, layers=None, free_order="workload", head_dim=None):
    src = synth.DataSource(w["seed"], w["sigma"], head_dim=head_dim or w["head_dim"])
    order = w["free_order"] if isinstance(free_order, str) else free_order
    world = OracleWorld(w["num_blocks"], w["n_layers"], src, w["scale"],
                        free_order=None if order is None else list(order), layers=layers)
    return world, world.run(w["trace"])


def test_shared_prefix_equals_isolated_recomputation():
    """Paper Sec. 1 / Sec. 3.2: one prefill fanned out to all tasks gives what each task would
    get from its own prefill of the same observation."""
    kw = dict(n_layers=2, prefix_len=40, chunk=6, denoise_steps=3, decode_targets=(4, 7, 9))
    shared, iso = synth.cross_task(**kw), synth.cross_task(isolated=True, **kw)
    _, rs = _replay(shared, head_dim=32)
    _, ri = _replay(iso, head_dim=32)
    steps_s = [(op, r) for op, r in zip(shared["trace"], rs) if op["op"] == "step"]
    steps_i = [(op, r) for op, r in zip(iso["trace"], ri) if op["op"] == "step"]
    n_checked = 0
    for op, r in steps_s:
        mine = [(o, x) for o, x in steps_i if o["shared_step"] == op["shared_step"]]
        assert [it for o, _ in mine for it in o["items"]] == op["items"]
        for layer in (0, 1):
            cat = np.concatenate([x["O"][layer] for _, x in mine])
            assert np.array_equal(cat, r["O"][layer])       # the oracle: exactly equal
            n_checked += 1
    assert n_checked == 2 * 9
    # and the isolated pool holds four copies of the prefix
    assert sum(1 for op in iso["trace"] if op["op"] == "prefix_create") == 4


def _mini_world(data, n_layers=1):
    return OracleWorld(64, n_layers, data, 0.25, page_size=16)


def test_action_view_is_independent_of_language_appends_and_of_batch_mates():
    """Sec. 1 (heterogeneous KV semantics) and App. A.2 (pure batching): the action chunk's
    output is the same whether or not a decode stream on the same prefix has appended, and
    an item's output does not depend on what else is in the batch or on item order."""
    data = synth.DataSource(77, head_dim=32)
    chunk_recipe = {"tag": 500, "tok0": 0, "n_total": 5}

    def run(with_decode, decode_first):
        w = _mini_world(data)
        w.apply({"op": "prefix_create"})
        w.apply({"op": "prefix_append", "pid": 0, "n": 20, "pos0": 0,
                 "data": {"tag": 1, "tok0": 0, "n_total": 20}})
        a = w.apply({"op": "stream_create", "pid": 0, "kind": ACTION})["sid"]
        d = w.apply({"op": "stream_create", "pid": 0, "kind": DECODE})["sid"]
        if with_decode:
            w.apply({"op": "step", "items": [(d, 9)], "attend": False,
                     "data": {"tag": 2, "tok0": 0, "n_total": 9}})
        if not with_decode:
            return w.apply({"op": "step", "items": [(a, 5)], "data": chunk_recipe})["O"][0]
        # action rows must come from the same recipe rows: put them first or last
        if decode_first:
            rec = {"tag": 501, "tok0": 0, "n_total": 6}
            o = w.apply({"op": "step", "items": [(d, 1), (a, 5)], "data": rec})["O"][0]
            return o[1:], rec
        rec = {"tag": 501, "tok0": 0, "n_total": 6}
        o = w.apply({"op": "step", "items": [(a, 5), (d, 1)], "data": rec})["O"][0]
        return o[:5], rec

    alone = run(False, False)
    # same q bits for the chunk are needed to compare: rebuild with explicit arrays instead
    q = data(chunk_recipe, 0, "q", 5)
    kp, vp = data({"tag": 1, "tok0": 0, "n_total": 20}, 0, "k", 20), \
        data({"tag": 1, "tok0": 0, "n_total": 20}, 0, "v", 20)
    ko, vo = data(chunk_recipe, 0, "k", 5), data(chunk_recipe, 0, "v", 5)
    direct, _ = attention.attend_item(ACTION, q, kp, vp, ko, vo, 0.25)
    assert np.array_equal(alone, direct)
    # in a mixed batch (different recipe -> different bits) only the *structure* can be
    # compared: recompute directly from that batch's bits and demand equality
    for decode_first in (False, True):
        o, rec = run(True, decode_first)
        t0 = 1 if decode_first else 0
        qm = data(rec, 0, "q", 6)[t0:t0 + 5]
        km, vm = data(rec, 0, "k", 6)[t0:t0 + 5], data(rec, 0, "v", 6)[t0:t0 + 5]
        direct, _ = attention.attend_item(ACTION, qm, kp, vp, km, vm, 0.25)
        assert np.array_equal(o, direct)


def test_frame_chop_invariance_and_resume():
    """Sec. 3.2 / App. A.2: a request interrupted every k tokens and resumed next frame
    yields what uninterrupted decoding yields; its earlier blocks never move."""
    data = synth.DataSource(78, head_dim=32)
    outs = {}
    tables = {}
    for k in (1, 3, 12):
        w = _mini_world(data)
        w.apply({"op": "prefix_create"})
        w.apply({"op": "prefix_append", "pid": 0, "n": 18, "pos0": 0,
                 "data": {"tag": 1, "tok0": 0, "n_total": 18}})
        d = w.apply({"op": "stream_create", "pid": 0, "kind": DECODE})["sid"]
        got = []
        seen_blocks = []
        for j in range(12):
            if j % k == 0 and j > 0:
                # frame boundary: other traffic allocates and frees blocks in between
                other = w.apply({"op": "stream_create", "pid": -1, "kind": DECODE})["sid"]
                w.apply({"op": "step", "items": [(other, 20)], "attend": False,
                         "data": {"tag": 900 + j, "tok0": 0, "n_total": 20}})
                w.apply({"op": "stream_release", "sid": other})
            r = w.apply({"op": "step", "items": [(d, 1)],
                         "data": {"tag": 100 + j, "tok0": 0, "n_total": 1}})
            got.append(r["O"][0][0])
            blocks = list(w.pool.streams[d].blocks)
            assert blocks[:len(seen_blocks)] == seen_blocks
            seen_blocks = blocks
        outs[k] = np.stack(got)
        tables[k] = seen_blocks
    assert np.array_equal(outs[1], outs[3]) and np.array_equal(outs[1], outs[12])


def test_outputs_do_not_depend_on_block_placement_but_tables_do():
    w = synth.tiny()
    w1, r1 = _replay(w, head_dim=32)
    w2, r2 = _replay(w, free_order=list(range(w["num_blocks"]))[::-1], head_dim=32)
    assert np.array_equal(r1[-1]["O"][0], r2[-1]["O"][0])
    assert r1[-1]["slots"] != r2[-1]["slots"]
    assert r1[-1]["O"][0].shape == (11, 8, 32)


def test_forked_prefix_reads_like_an_unforked_copy():
    """A child prefix that shares its first 32 tokens with its parent and continues with 20
    tokens of its own gives every query exactly what a prefix holding the same 52 tokens in
    blocks of its own gives; only the block tables differ."""
    from oracle.pool_model import ACTION, DECODE
    src = synth.DataSource(777)
    hist = {"tag": 1, "tok0": 0, "n_total": 48}
    tail = {"tag": 2, "tok0": 0, "n_total": 20}
    step = {"op": "step", "items": [(0, 6), (1, 1)], "attend": True,
            "data": {"tag": 3, "tok0": 0, "n_total": 7}}
    forked = [{"op": "prefix_create", "pid": 0},
              {"op": "prefix_append", "pid": 0, "n": 48, "pos0": 0, "data": hist},
              {"op": "prefix_fork", "parent": 0, "n": 32, "pid": 1},
              {"op": "prefix_append", "pid": 1, "n": 20, "pos0": 32, "data": tail},
              {"op": "stream_create", "pid": 1, "kind": ACTION, "sid": 0},
              {"op": "stream_create", "pid": 1, "kind": DECODE, "sid": 1}, step]
    plain = [{"op": "prefix_create", "pid": 0},
             {"op": "prefix_append", "pid": 0, "n": 32, "pos0": 0, "data": hist},
             {"op": "prefix_append", "pid": 0, "n": 20, "pos0": 32, "data": tail},
             {"op": "stream_create", "pid": 0, "kind": ACTION, "sid": 0},
             {"op": "stream_create", "pid": 0, "kind": DECODE, "sid": 1}, step]
    outs = []
    for trace in (forked, plain):
        ow = OracleWorld(32, 1, src, 0.0625)
        res = [ow.apply(op) for op in trace]
        outs.append(res[-1])
        if trace is forked:
            assert ow.pool.prefixes[1].blocks[:2] == ow.pool.prefixes[0].blocks[:2]
            assert ow.pool.ref[ow.pool.prefixes[0].blocks[0]] == 4   # two handles, two streams
    assert np.array_equal(outs[0]["O"][0], outs[1]["O"][0])
    assert np.array_equal(outs[0]["LSE"][0], outs[1]["LSE"][0])


# ---- pins of the replay's bookkeeping against hand-built key/value lists ----------------
# Expected values come from the pure-Python loops in oracle.brute on lists assembled here
# by hand, never from the replay itself, so a slip in the replay's handling of an operation
# (a chunk that accumulates, a rewind that keeps its tail, an overwrite that truncates or
# misplaces) shows up as a disagreement.
def _loops(kind, q, kp, vp, ko, vo, scale):
    o, lse = brute.attend_item_loops(kind, q.tolist(), kp.tolist(), vp.tolist(), ko.tolist(),
                                     vo.tolist(), scale)
    return np.array(o), np.array(lse)


def _tiny_source():
    return synth.DataSource(4242, n_heads=2, head_dim=16)


def test_action_chunk_kv_is_transient_per_denoise_step():
    """App. A.1 Eq. 6 and Sec. 1 (heterogeneous KV semantics): the action expert reads the
    prefill cache as read-only context over its S denoising steps and generates the chunk
    jointly, so at every step the chunk queries see the prefix plus THAT step's chunk
    tokens only; nothing of an earlier denoising step remains visible."""
    data = _tiny_source()
    w = OracleWorld(32, 1, data, 0.3)
    pre = {"tag": 1, "tok0": 0, "n_total": 9}
    w.apply({"op": "prefix_create"})
    w.apply({"op": "prefix_append", "pid": 0, "n": 9, "pos0": 0, "data": pre})
    a = w.apply({"op": "stream_create", "pid": 0, "kind": ACTION})["sid"]
    kp, vp = data(pre, 0, "k", 9), data(pre, 0, "v", 9)
    blocks = None
    for s in range(4):
        rec = {"tag": 10 + s, "tok0": 0, "n_total": 5}
        got = w.apply({"op": "step", "items": [(a, 5)], "data": rec})
        exp_o, exp_lse = _loops(ACTION, data(rec, 0, "q", 5), kp, vp, data(rec, 0, "k", 5),
                                data(rec, 0, "v", 5), 0.3)
        np.testing.assert_allclose(got["O"][0], exp_o, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(got["LSE"][0], exp_lse, rtol=1e-12, atol=1e-13)
        # the un-paged truth holds exactly this step's five rows, in the same blocks
        assert np.array_equal(w.stream_kv[a][0][0], data(rec, 0, "k", 5))
        assert w.pool.streams[a].length == 5
        assert blocks in (None, list(w.pool.streams[a].blocks))
        blocks = list(w.pool.streams[a].blocks)


def test_rewind_drops_the_tail_and_later_tokens_take_its_place():
    """Sec. 3.2 (compatibility with parallel decoding: rejected draft tokens are rolled
    back): decode 6 tokens, rewind to 3, append 2 new ones -> the new queries see the
    prefix, the first three original tokens and the two new ones, nothing of the dropped
    three."""
    data = _tiny_source()
    w = OracleWorld(32, 1, data, 0.3)
    pre = {"tag": 1, "tok0": 0, "n_total": 7}
    first = {"tag": 2, "tok0": 0, "n_total": 6}
    second = {"tag": 3, "tok0": 0, "n_total": 2}
    w.apply({"op": "prefix_create"})
    w.apply({"op": "prefix_append", "pid": 0, "n": 7, "pos0": 0, "data": pre})
    d = w.apply({"op": "stream_create", "pid": 0, "kind": DECODE})["sid"]
    w.apply({"op": "step", "items": [(d, 6)], "data": first, "attend": False})
    slots_before = list(w.pool.streams[d].blocks)
    w.apply({"op": "stream_rewind", "sid": d, "len": 3})
    got = w.apply({"op": "step", "items": [(d, 2)], "data": second})
    ko = np.concatenate([data(first, 0, "k", 6)[:3], data(second, 0, "k", 2)])
    vo = np.concatenate([data(first, 0, "v", 6)[:3], data(second, 0, "v", 2)])
    exp_o, exp_lse = _loops(DECODE, data(second, 0, "q", 2), data(pre, 0, "k", 7),
                            data(pre, 0, "v", 7), ko, vo, 0.3)
    np.testing.assert_allclose(got["O"][0], exp_o, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got["LSE"][0], exp_lse, rtol=1e-12, atol=1e-13)
    # positions 3 and 4 of the same block are written again; no block moved or was freed
    blk = slots_before[0]
    assert got["slots"] == [blk * 16 + 3, blk * 16 + 4]
    assert w.pool.streams[d].length == 5 and w.pool.streams[d].blocks == slots_before


def test_prefix_append_below_the_length_overwrites_in_place():
    """An append at pos0 < len on a prefix that nobody has attached to yet rewrites tokens
    [pos0, pos0+n) and leaves every other token alone; the length only grows."""
    data = _tiny_source()
    w = OracleWorld(32, 1, data, 0.3)
    a_rec = {"tag": 1, "tok0": 0, "n_total": 20}
    b_rec = {"tag": 2, "tok0": 0, "n_total": 4}
    c_rec = {"tag": 3, "tok0": 0, "n_total": 8}
    w.apply({"op": "prefix_create"})
    s_a = w.apply({"op": "prefix_append", "pid": 0, "n": 20, "pos0": 0, "data": a_rec})["slots"]
    s_b = w.apply({"op": "prefix_append", "pid": 0, "n": 4, "pos0": 12, "data": b_rec})["slots"]
    assert s_b == s_a[12:16] and w.pool.prefixes[0].length == 20      # in the middle
    s_c = w.apply({"op": "prefix_append", "pid": 0, "n": 8, "pos0": 18, "data": c_rec})["slots"]
    assert s_c[:2] == s_a[18:20] and w.pool.prefixes[0].length == 26  # across the old end
    d = w.apply({"op": "stream_create", "pid": 0, "kind": DECODE})["sid"]
    q_rec = {"tag": 4, "tok0": 0, "n_total": 1}
    got = w.apply({"op": "step", "items": [(d, 1)], "data": q_rec})
    parts = lambda what: np.concatenate([data(a_rec, 0, what, 20)[:12], data(b_rec, 0, what, 4),
                                         data(a_rec, 0, what, 20)[16:18],
                                         data(c_rec, 0, what, 8)])
    kp, vp = parts("k"), parts("v")
    assert len(kp) == 26
    exp_o, exp_lse = _loops(DECODE, data(q_rec, 0, "q", 1), kp, vp, data(q_rec, 0, "k", 1),
                            data(q_rec, 0, "v", 1), 0.3)
    np.testing.assert_allclose(got["O"][0], exp_o, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got["LSE"][0], exp_lse, rtol=1e-12, atol=1e-13)
    assert np.array_equal(w.prefix_kv[0][0][0], kp)
