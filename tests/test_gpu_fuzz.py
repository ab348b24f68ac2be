"""Seeded random traces through the C ABI against the float64 oracle, op by op: prefixes of random
lengths on both sides of the 1024-token boundary between the streamed and the tiled prefix phase
(some forked off others, some appended in two pieces), streams with and without a prefix, action
chunks of 1..60 tokens, decode steps of 1, 2 and several tokens, history loads that are not
attended, rewinds, releases in any order, on a shuffled free order and a pool full of NaN bit
patterns.  Every id, every slot list, every output element and every log-sum-exp is compared;
at the end every live token of the pool is read back bit for bit.

The generator keeps only what it needs to emit valid operations (lengths, kinds, who is alive);
the expected values come from the oracle's replay."""
import numpy as np
import pytest

from paper_2603_14371_amd.synth import ACTION, DECODE
from parity_util import assert_pool_contents_equal, run_both

pytestmark = pytest.mark.gpu


def random_trace(seed, n_ops=90, num_blocks=1024):
    rng = np.random.default_rng(seed)
    trace, tag = [], [0]
    prefixes = {}      # pid -> [length, sealed, alive (creator's reference), n_streams]
    streams = {}       # sid -> [pid, kind, length]
    n_prefix = n_stream = 0
    blocks_used = [0]

    def recipe(n):
        tag[0] += 1
        return {"tag": tag[0], "tok0": 0, "n_total": n}

    def room(tokens):
        return blocks_used[0] + tokens // 16 + 8 < num_blocks

    def new_prefix():
        nonlocal n_prefix
        length = int(rng.choice([rng.integers(1, 200), rng.integers(200, 1024),
                                 rng.integers(1025, 1500), 1024, 1040]))
        if not room(length):
            return
        pid = n_prefix
        n_prefix += 1
        forkable = [p for p, v in prefixes.items() if v[0] >= 16 and (v[2] or v[3] > 0)]
        if forkable and rng.random() < 0.3:
            parent = int(rng.choice(forkable))
            n = 16 * int(rng.integers(1, prefixes[parent][0] // 16 + 1))
            trace.append({"op": "prefix_fork", "parent": parent, "n": n, "pid": pid})
            extra = int(rng.integers(0, 120))
            if extra:
                trace.append({"op": "prefix_append", "pid": pid, "n": extra, "pos0": n,
                              "data": recipe(extra)})
            prefixes[pid] = [n + extra, False, True, 0]
            blocks_used[0] += extra // 16 + 1
            return
        trace.append({"op": "prefix_create", "pid": pid})
        first = length if rng.random() < 0.6 else int(rng.integers(1, length + 1))
        trace.append({"op": "prefix_append", "pid": pid, "n": first, "pos0": 0, "data": recipe(first)})
        if first < length:
            trace.append({"op": "prefix_append", "pid": pid, "n": length - first, "pos0": first,
                          "data": recipe(length - first)})
        prefixes[pid] = [length, False, True, 0]
        blocks_used[0] += length // 16 + 1

    def new_stream():
        nonlocal n_stream
        attachable = [p for p, v in prefixes.items() if v[2] and v[0] > 0]
        pid = int(rng.choice(attachable)) if attachable and rng.random() < 0.85 else -1
        kind = ACTION if rng.random() < 0.35 else DECODE
        sid = n_stream
        n_stream += 1
        trace.append({"op": "stream_create", "pid": pid, "kind": kind, "sid": sid})
        streams[sid] = [pid, kind, 0]
        if pid >= 0:
            prefixes[pid][1] = True
            prefixes[pid][3] += 1

    def step():
        while len(streams) < 2:
            new_stream()
        sids = [int(s) for s in rng.permutation(list(streams))[:int(rng.integers(1, 7))]]
        attend = rng.random() < 0.8
        items = []
        for sid in sids:
            pid, kind, length = streams[sid]
            if kind == ACTION:
                n = int(rng.integers(1, 61))
            elif not attend:
                n = int(rng.integers(1, 300))
            else:
                n = int(rng.choice([1, 1, 1, 2, 2, int(rng.integers(3, 13))]))
            if not room(n):
                continue
            items.append((sid, n))
            streams[sid][2] = n if kind == ACTION else length + n
            blocks_used[0] += n // 16 + 1
        if items:
            n_tok = sum(n for _, n in items)
            trace.append({"op": "step", "items": items, "attend": bool(attend), "data": recipe(n_tok)})

    def rewind():
        cands = [s for s, v in streams.items() if v[1] == DECODE and v[2] > 0]
        if cands:
            sid = int(rng.choice(cands))
            new_len = int(rng.integers(0, streams[sid][2] + 1))
            trace.append({"op": "stream_rewind", "sid": sid, "len": new_len})
            streams[sid][2] = new_len

    def release_stream():
        if streams:
            sid = int(rng.choice(list(streams)))
            trace.append({"op": "stream_release", "sid": sid})
            pid = streams.pop(sid)[0]
            if pid >= 0:
                prefixes[pid][3] -= 1

    def release_prefix():
        alive = [p for p, v in prefixes.items() if v[2]]
        if alive:
            pid = int(rng.choice(alive))
            trace.append({"op": "prefix_release", "pid": pid})
            prefixes[pid][2] = False

    new_prefix()
    new_stream()
    for _ in range(n_ops):
        r = rng.random()
        if r < 0.10:
            new_prefix()
        elif r < 0.25:
            new_stream()
        elif r < 0.80:
            step()
        elif r < 0.87:
            rewind()
        elif r < 0.95:
            release_stream()
        else:
            release_prefix()
    order = np.random.default_rng(seed + 7).permutation(num_blocks).astype(np.int32)
    return {"name": "fuzz", "seed": 14371900 + seed, "n_layers": 3, "num_blocks": num_blocks,
            "page_size": 16, "n_q_heads": 8, "head_dim": 256, "scale": 1.0 / 16.0, "sigma": 1.0,
            "free_order": order, "trace": trace}


@pytest.mark.parametrize("seed,fold", [(s, bool((s + s // 4) % 2)) for s in range(12)])
def test_random_traces_match_the_oracle(seed, fold):
    w = random_trace(seed)
    n_steps = sum(1 for op in w["trace"] if op["op"] == "step" and op["attend"])
    assert n_steps >= 15
    gw, g, ow, o = run_both(w, layers=[0, 2], poison=True, fold_append=fold,
                            max_q_tokens=1024, max_append_tokens=4096)
    try:
        assert_pool_contents_equal(gw, ow)
    finally:
        gw.close()
