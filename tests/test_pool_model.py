"""Pins the indexing oracle: a hand-worked allocation example, conservation laws under
random operation sequences, atomic failure, and the paper's worked schedule.  No GPU."""
import os

import numpy as np
import pytest

from oracle.pool_model import (ACTION, DECODE, ERR_BAD_ID, ERR_INVALID_ARG, ERR_NO_BLOCKS,
                               ERR_SEALED, PoolError, PoolModel)
from paper_2603_14371_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_tables_refcounts_and_free_order():
    """Worked by hand from the stated policy (LIFO stack, first element of free_order on top,
    release pushes in ascending logical order, own table before prefix table)."""
    m = PoolModel(8, page_size=4, free_order=[5, 2, 7, 0, 1, 3, 4, 6])
    p = m.prefix_create()
    assert p == 0
    assert m.prefix_append(p, 0, 6, 0) == [5 * 4 + 0, 21, 22, 23, 2 * 4 + 0, 9]   # blocks 5, 2
    a = m.stream_create(p, ACTION)
    d = m.stream_create(p, DECODE)
    assert (a, d) == (0, 1)
    assert [m.ref[b] for b in (5, 2)] == [3, 3]
    # batch: action takes 5 tokens -> blocks 7, 0 ; decode takes 1 token -> block 1
    slots = m.batch_build([(a, 5), (d, 1)])
    assert slots == [28, 29, 30, 31, 0, 4]
    # next step: action rewinds and rewrites the same slots; decode moves on inside block 1
    assert m.batch_build([(a, 5), (d, 1)]) == [28, 29, 30, 31, 0, 5]
    with pytest.raises(PoolError) as e:
        m.prefix_append(p, 0, 1, 6)
    assert e.value.code == ERR_SEALED
    m.stream_release(a)                    # pushes 7 then 0; prefix blocks stay (ref 2)
    assert m.free[-2:] == [7, 0] and [m.ref[b] for b in (5, 2)] == [2, 2]
    m.prefix_release(p)                    # creator's handle gone, decode stream keeps it alive
    assert [m.ref[b] for b in (5, 2)] == [1, 1] and m.stats() == (5, 1, 1)
    m.stream_release(d)                    # own block 1, then prefix blocks 5, 2
    assert m.free[-3:] == [1, 5, 2] and m.stats() == (8, 0, 0)
    assert m.stream_create(-1, DECODE) == 2          # ids are never reused
    assert m.batch_build([(2, 1)]) == [2 * 4]         # top of the stack is block 2


def test_failure_is_atomic():
    m = PoolModel(4, page_size=4)
    s0, s1 = m.stream_create(-1, DECODE), m.stream_create(-1, DECODE)
    m.batch_build([(s0, 8)])
    before = (list(m.free), list(m.ref), m.streams[s0].length, m.streams[s1].length)
    with pytest.raises(PoolError) as e:
        m.batch_build([(s0, 4), (s1, 5)])           # needs 1 + 2 blocks, 2 are free
    assert e.value.code == ERR_NO_BLOCKS
    assert before == (list(m.free), list(m.ref), m.streams[s0].length, m.streams[s1].length)
    for bad, code in (([(s0, 0)], ERR_INVALID_ARG), ([(s0, 1), (s0, 1)], ERR_INVALID_ARG),
                      ([(9, 1)], ERR_BAD_ID), ([], ERR_INVALID_ARG)):
        with pytest.raises(PoolError) as e:
            m.batch_build(bad)
        assert e.value.code == code
    p = m.prefix_create()
    with pytest.raises(PoolError) as e:
        m.prefix_append(p, 0, 4, 1)                 # hole before pos0
    assert e.value.code == ERR_INVALID_ARG
    with pytest.raises(PoolError) as e:
        m.prefix_append(p, 0, 12, 0)
    assert e.value.code == ERR_NO_BLOCKS and m.prefixes[p].blocks == []


def test_hand_worked_fork():
    """Fork worked by hand: the child lists the parent's first blocks, both freeze the shared
    range, the child grows into blocks of its own, and blocks return when the last table that
    lists them goes."""
    m = PoolModel(8, page_size=4)                     # free stack pops 0, 1, 2, ...
    p = m.prefix_create()
    m.prefix_append(p, 0, 10, 0)                      # blocks 0, 1, 2
    for bad in (3, 12, -4):                           # not a page multiple / beyond the parent
        with pytest.raises(PoolError) as e:
            m.prefix_fork(p, bad)
        assert e.value.code == ERR_INVALID_ARG
    with pytest.raises(PoolError) as e:
        m.prefix_fork(7, 4)
    assert e.value.code == ERR_BAD_ID
    c = m.prefix_fork(p, 8)
    assert c == 1 and m.prefixes[c].blocks == [0, 1] and m.prefixes[c].length == 8
    assert m.ref[:3] == [2, 2, 1]
    assert m.prefix_append(c, 0, 5, 8) == [12, 13, 14, 15, 16]    # own blocks 3, 4
    for pid, pos in ((c, 4), (p, 7)):                 # the shared range is read-only in both
        with pytest.raises(PoolError) as e:
            m.prefix_append(pid, 0, 1, pos)
        assert e.value.code == ERR_SEALED
    assert m.prefix_append(p, 0, 2, 8) == [8, 9]      # the parent's unshared tail is still its own
    d = m.stream_create(c, DECODE)
    assert m.ref[:5] == [3, 3, 1, 2, 2]
    m.prefix_release(p)                               # block 2 returns, 0 and 1 live on in the child
    assert m.free[-1] == 2 and m.ref[:3] == [2, 2, 0] and p not in m.prefixes
    m.prefix_release(c)
    m.stream_release(d)
    assert m.free[-4:] == [0, 1, 3, 4] and m.stats() == (8, 0, 0)
    e0 = m.prefix_create()
    z = m.prefix_fork(e0, 0)                          # an empty fork is an empty prefix
    assert m.prefixes[z].blocks == [] and m.prefix_append(z, 0, 1, 0) == [16]


def _check_conservation(m):
    """free + distinct live blocks = all; ref[b] = number of tables holding b (+ handle)."""
    count = [0] * m.num_blocks
    for p in m.prefixes.values():
        for b in p.blocks:
            count[b] += (1 if p.handle else 0) + p.n_streams
    for s in m.streams.values():
        for b in s.blocks:
            count[b] += 1
    assert count == m.ref
    live = {b for b in range(m.num_blocks) if m.ref[b] > 0}
    assert live.isdisjoint(m.free) and len(m.free) == len(set(m.free))
    assert len(live) + len(m.free) == m.num_blocks


@pytest.mark.parametrize("seed", range(4))
def test_conservation_under_random_operations(seed):
    rng = np.random.default_rng(seed)
    m = PoolModel(96, page_size=4, n_layers=2, free_order=rng.permutation(96).tolist())
    open_prefixes = []
    for _ in range(600):
        r = rng.random()
        try:
            if r < 0.12:
                pid = m.prefix_create()
                open_prefixes.append(pid)
                m.prefix_append(pid, 0, int(rng.integers(1, 20)), 0)
            elif r < 0.16 and m.prefixes:
                parent = int(rng.choice(list(m.prefixes)))
                n = 4 * int(rng.integers(0, m.prefixes[parent].length // 4 + 1))
                pid = m.prefix_fork(parent, n)
                open_prefixes.append(pid)
                if rng.random() < 0.7:
                    m.prefix_append(pid, 0, int(rng.integers(1, 12)), n)
            elif r < 0.3:
                pid = int(rng.choice(open_prefixes)) if open_prefixes and rng.random() < 0.8 else -1
                m.stream_create(pid, int(rng.integers(0, 2)))
            elif r < 0.7 and m.streams:
                sids = rng.permutation(list(m.streams))[:int(rng.integers(1, 5))]
                m.batch_build([(int(s), int(rng.integers(1, 9))) for s in sids])
            elif r < 0.85 and m.streams:
                m.stream_release(int(rng.choice(list(m.streams))))
            elif r < 0.92 and open_prefixes:
                m.prefix_release(open_prefixes.pop(int(rng.integers(len(open_prefixes)))))
            elif m.streams:
                sid = int(rng.choice(list(m.streams)))
                m.stream_rewind(sid, int(rng.integers(0, m.streams[sid].length + 1)))
        except PoolError as e:
            assert e.code == ERR_NO_BLOCKS
        _check_conservation(m)
    for sid in list(m.streams):
        m.stream_release(sid)
    for pid in open_prefixes:
        m.prefix_release(pid)
    assert sorted(m.free) == list(range(96)) and m.stats() == (96, 0, 0)


def _read_schedule():
    vals = {}
    for line in open(os.path.join(GOLDEN, "schedule_fig3.txt")):
        if not line.startswith("#") and line.strip():
            k, v = line.split()
            vals[k] = int(v)
    return vals


def test_worked_schedule_of_the_paper():
    """N = 12 tokens per request at k = 4 per frame, one request per frame -> the active
    decode batch settles at B = N / k = 3 and request ids equal frame indices."""
    g = _read_schedule()
    w = synth.cross_frame(n_frames=12, n_layers=1, n_slots=8, prefix_len=16, chunk=4,
                          denoise_steps=2, k=g["k"], targets=[g["N"]], num_blocks=256)
    m = PoolModel(w["num_blocks"], free_order=w["free_order"].tolist())
    sizes = {}
    decode_ids = []
    for op in w["trace"]:
        if op["op"] == "prefix_create":
            assert m.prefix_create() == op["pid"]
        elif op["op"] == "prefix_append":
            m.prefix_append(op["pid"], 0, op["n"], op["pos0"])
        elif op["op"] == "stream_create":
            assert m.stream_create(op["pid"], op["kind"]) == op["sid"]
            if op["kind"] == DECODE:
                decode_ids.append((op["pid"], op["sid"]))
        elif op["op"] == "step":
            m.batch_build(op["items"])
            n_dec = sum(1 for sid, _ in op["items"] if m.streams[sid].kind == DECODE)
            sizes.setdefault(op["frame"], []).append(n_dec)
        elif op["op"] == "stream_release":
            m.stream_release(op["sid"])
        elif op["op"] == "prefix_release":
            m.prefix_release(op["pid"])
    for frame in range(g["N"] // g["k"] - 1, 12):
        assert sizes[frame] == [g["B"]] * g["k"]
    assert sizes[0] == [1] * g["k"] and sizes[1] == [2] * g["k"]
    # one language request per frame: the t-th request (counting language requests) was
    # created in frame t, i.e. hangs off prefix t
    assert [pid for pid, _ in decode_ids] == list(range(12))
    assert m.stats()[2] == g["B"] - 1          # the requests still in flight after frame 11
