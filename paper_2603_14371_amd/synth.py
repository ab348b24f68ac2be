"""Seeded synthetic inputs and operation traces.  Holds none of the method's arithmetic.

This module is the only thing the HIP path and the CPU oracle have in common:
it draws bf16 bit patterns and writes down *which* operations a workload
performs (create a prefix, append, fan out, batch, release), never how any of
them is computed.  Shapes follow pi0.5's attention geometry: 8 query heads over
1 KV head, head_dim 256, an 832-token observation prefix (3 cameras x 256 image
tokens + 64 prompt tokens), 50-query action chunks denoised for S = 10 steps,
page size 16.  The frame schedules follow the paper's per-frame flow (Alg. 1):
prefill cache -> action denoise + fan-out -> batched decode of every active
request -> evict finished requests.

A trace is a list of dicts; see `trace ops` in the functions below.  A data
recipe is a dict {"tag", "tok0", "n_total"}: the rows [tok0, tok0+n) of an
array of n_total tokens drawn from a generator seeded by (seed, tag, layer,
what).  Two traces that name the same recipe therefore see the same bits, which
is how the shared and the isolated variant of a workload get identical inputs.
"""
import numpy as np

ACTION = 0
DECODE = 1

N_Q_HEADS = 8
HEAD_DIM = 256
PAGE = 16
_WHAT = {"k": 0, "v": 1, "q": 2}


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


class DataSource:
    """data_fn(recipe, layer, what, n) -> uint16 bit patterns, reproducible from the seed."""

    def __init__(self, seed, sigma=1.0, n_heads=N_Q_HEADS, head_dim=HEAD_DIM):
        self.seed = int(seed)
        self.sigma = float(sigma)
        self.n_heads = n_heads
        self.head_dim = head_dim

    def __call__(self, recipe, layer, what, n):
        tag, tok0, n_total = recipe["tag"], recipe["tok0"], recipe["n_total"]
        if tok0 + n > n_total:
            raise ValueError("recipe too short")
        rng = np.random.Generator(np.random.PCG64(
            np.random.SeedSequence([self.seed, int(tag), int(layer), _WHAT[what]])))
        width = self.head_dim * (self.n_heads if what == "q" else 1)
        x = rng.standard_normal((n_total, width), dtype=np.float32)
        if self.sigma != 1.0:
            x *= np.float32(self.sigma)
        bits = f32_to_bf16_bits(x[tok0:tok0 + n])
        if what == "q":
            return bits.reshape(n, self.n_heads, self.head_dim)
        return bits


class _TraceBuilder:
    def __init__(self):
        self.trace = []
        self.n_prefix = 0
        self.n_stream = 0
        self.tag = 0

    def recipe(self, n_total, tag=None, tok0=0):
        if tag is None:
            tag = self.tag
            self.tag += 1
        return {"tag": tag, "tok0": tok0, "n_total": n_total}

    def prefix(self, n_tokens, recipe=None):
        pid = self.n_prefix
        self.n_prefix += 1
        self.trace.append({"op": "prefix_create", "pid": pid})
        self.trace.append({"op": "prefix_append", "pid": pid, "n": n_tokens, "pos0": 0,
                           "data": recipe or self.recipe(n_tokens)})
        return pid

    def stream(self, pid, kind):
        sid = self.n_stream
        self.n_stream += 1
        self.trace.append({"op": "stream_create", "pid": pid, "kind": kind, "sid": sid})
        return sid

    def step(self, items, attend=True, recipe=None, **extra):
        n_tok = sum(n for _, n in items)
        op = {"op": "step", "items": [tuple(i) for i in items], "attend": attend,
              "data": recipe or self.recipe(n_tok)}
        op.update(extra)
        self.trace.append(op)
        return op

    def release_stream(self, sid):
        self.trace.append({"op": "stream_release", "sid": sid})

    def release_prefix(self, pid):
        self.trace.append({"op": "prefix_release", "pid": pid})


def _workload(name, seed, n_layers, num_blocks, trace, free_order=None, sigma=1.0, **meta):
    w = {"name": name, "seed": seed, "n_layers": n_layers, "num_blocks": num_blocks,
         "page_size": PAGE, "n_q_heads": N_Q_HEADS, "head_dim": HEAD_DIM,
         "scale": 1.0 / np.sqrt(float(HEAD_DIM)), "sigma": sigma,
         "free_order": free_order, "trace": trace}
    w.update(meta)
    return w


def _seed(cfg):
    return 14371000 + 100 * cfg


def _perm(seed, n):
    return np.random.Generator(np.random.PCG64(seed)).permutation(n).astype(np.int32)


# ---------------------------------------------------------------------------
# config 0: tiny single-layer case
# ---------------------------------------------------------------------------
def tiny(prefix_len=64, chunk=10, prior=4, n_layers=1, sigma=1.0, seed=None):
    b = _TraceBuilder()
    pid = b.prefix(prefix_len) if prefix_len > 0 else -1
    act = b.stream(pid, ACTION)
    dec = b.stream(pid, DECODE)
    if prior > 0:
        b.step([(dec, prior)], attend=False)
    b.step([(act, chunk), (dec, 1)])
    need = -(-prefix_len // PAGE) + -(-chunk // PAGE) + -(-(prior + 1) // PAGE)
    return _workload("tiny", _seed(0) if seed is None else seed, n_layers, max(64, 2 * need),
                     b.trace, sigma=sigma)


# ---------------------------------------------------------------------------
# config 1: one pi0.5-shaped frame
# ---------------------------------------------------------------------------
def pi05_frame(n_layers=18, prefix_len=832, chunk=50, denoise_steps=10, decode_tokens=64,
               sigma=1.0, seed=None):
    b = _TraceBuilder()
    pid = b.prefix(prefix_len)
    act = b.stream(pid, ACTION)
    dec = b.stream(pid, DECODE)
    for s in range(max(denoise_steps, decode_tokens)):
        items = []
        if s < denoise_steps:
            items.append((act, chunk))
        if s < decode_tokens:
            items.append((dec, 1))
        b.step(items, mixed=s < denoise_steps)
    b.release_stream(act)
    b.release_stream(dec)
    b.release_prefix(pid)
    return _workload("pi05_frame", _seed(1) if seed is None else seed, n_layers, 256, b.trace,
                     sigma=sigma)


# ---------------------------------------------------------------------------
# config 2: cross-frame continuous batching (Alg. 1 over many frames)
# ---------------------------------------------------------------------------
def cross_frame(n_frames=40, n_layers=18, n_slots=8, prefix_len=832, chunk=50,
                denoise_steps=10, k=10, target_lo=16, target_hi=512, targets=None,
                num_blocks=2048, shuffle=True, with_action=True, seed=None):
    """Each frame: a fresh prefix, one action chunk, and at most one new language
    request in the lowest free slot (bound to that frame's prefix).  Every active
    request advances one token per step for at most k steps per frame; a request
    that reaches its target stops being listed at once and is evicted at frame
    end (finished action stream first, then finished requests in id order, then
    the creator's prefix reference)."""
    seed = _seed(2) if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed + 900))
    b = _TraceBuilder()
    slots = [None] * n_slots            # each: [sid, done, target]
    frames = []
    n_created = 0
    for t in range(n_frames):
        first_op = len(b.trace)
        pid = b.prefix(prefix_len)
        act = b.stream(pid, ACTION) if with_action else None
        free = [i for i, s in enumerate(slots) if s is None]
        if free:
            if targets is not None:
                target = int(targets[n_created % len(targets)])
            else:
                target = int(rng.integers(target_lo, target_hi + 1))
            slots[free[0]] = [b.stream(pid, DECODE), 0, target]
            n_created += 1
        for s in range(max(denoise_steps if with_action else 0, k)):
            items = []
            if with_action and s < denoise_steps:
                items.append((act, chunk))
            if s < k:
                for slot in slots:
                    if slot is not None and slot[1] < slot[2]:
                        items.append((slot[0], 1))
                        slot[1] += 1
            if items:
                b.step(items, frame=t, mixed=with_action and s < denoise_steps)
        if with_action:
            b.release_stream(act)
        finished = sorted((slot[0], i) for i, slot in enumerate(slots)
                          if slot is not None and slot[1] >= slot[2])
        for sid, i in finished:
            b.release_stream(sid)
            slots[i] = None
        b.release_prefix(pid)
        frames.append((first_op, len(b.trace)))
    order = _perm(seed + 901, num_blocks) if shuffle else None
    return _workload("cross_frame", seed, n_layers, num_blocks, b.trace, free_order=order,
                     frames=frames)


# ---------------------------------------------------------------------------
# config 3: cross-task sharing vs isolated execution
# ---------------------------------------------------------------------------
def cross_task(isolated=False, n_layers=18, prefix_len=832, chunk=50, denoise_steps=10,
               decode_targets=(128, 256, 384), n_steps=None, seed=None):
    """Four tasks on one observation.  Shared: one prefix, one batch per step.
    Isolated: every task owns a copy of the prefix (same recipe, hence same bits)
    and runs in a batch of its own -- the paper's "isolated execution" baseline."""
    b = _TraceBuilder()
    prefix_recipe = b.recipe(prefix_len)
    n_tasks = 1 + len(decode_targets)
    if isolated:
        pids = [b.prefix(prefix_len, dict(prefix_recipe)) for _ in range(n_tasks)]
    else:
        pids = [b.prefix(prefix_len, dict(prefix_recipe))] * n_tasks
    act = b.stream(pids[0], ACTION)
    decs = [b.stream(pids[1 + i], DECODE) for i in range(len(decode_targets))]
    total = max(denoise_steps, max(decode_targets)) if n_steps is None else n_steps
    for s in range(total):
        items = []
        if s < denoise_steps:
            items.append((act, chunk))
        for sid, tgt in zip(decs, decode_targets):
            if s < tgt:
                items.append((sid, 1))
        n_tok = sum(n for _, n in items)
        tag = b.recipe(n_tok)["tag"]
        if isolated:
            tok0 = 0
            for it in items:
                b.step([it], recipe={"tag": tag, "tok0": tok0, "n_total": n_tok},
                       shared_step=s, mixed=s < denoise_steps)
                tok0 += it[1]
        else:
            b.step(items, recipe={"tag": tag, "tok0": 0, "n_total": n_tok},
                   shared_step=s, mixed=s < denoise_steps)
    b.release_stream(act)
    for sid in decs:
        b.release_stream(sid)
    for pid in sorted(set(pids)):
        b.release_prefix(pid)
    return _workload("cross_task_isolated" if isolated else "cross_task",
                     _seed(3) if seed is None else seed, n_layers, 512, b.trace)


# ---------------------------------------------------------------------------
# config 4: stress
# ---------------------------------------------------------------------------
def stress(n_layers=18, n_streams=64, group=8, prefix_len=2048, hist_lo=1, hist_hi=2048,
           n_action=2, chunk=50, mixed_steps=10, num_blocks=8192, churn_ops=2000, seed=None):
    """64 decode streams with own histories ~U{1..2048}; prefixes of 2048 tokens shared
    by groups of 8; action chunk i hangs off prefix group i.  The pool is first
    fragmented by a seeded churn of scratch streams created, grown and released
    through the same public operations, on top of a shuffled free order."""
    seed = _seed(4) if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed + 900))
    b = _TraceBuilder()
    # churn: scratch streams without a prefix, never attended
    live = []                           # [sid, own length]
    budget = num_blocks // 4

    def held():
        return sum((n + PAGE - 1) // PAGE for _, n in live)

    for _ in range(churn_ops):
        r = rng.random()
        if live and (r < 0.35 or held() > budget):
            sid, _ = live.pop(int(rng.integers(len(live))))
            b.release_stream(sid)
        elif live and r < 0.65:
            i = int(rng.integers(len(live)))
            grow = int(rng.integers(1, 5 * PAGE))
            b.step([(live[i][0], grow)], attend=False, churn=True)
            live[i][1] += grow
        else:
            sid = b.stream(-1, DECODE)
            grow = int(rng.integers(1, 8 * PAGE))
            b.step([(sid, grow)], attend=False, churn=True)
            live.append([sid, grow])
    for sid, _ in live:
        b.release_stream(sid)
    n_groups = n_streams // group
    pids = [b.prefix(prefix_len) for _ in range(n_groups)]
    acts = [b.stream(pids[i % n_groups], ACTION) for i in range(n_action)]
    decs = [b.stream(pids[i // group], DECODE) for i in range(n_streams)]
    hist = [int(h) for h in rng.integers(hist_lo, hist_hi + 1, size=n_streams)]
    b.step(list(zip(decs, hist)), attend=False, history=True)
    first_mixed = len(b.trace)
    for s in range(mixed_steps):
        b.step([(a, chunk) for a in acts] + [(d, 1) for d in decs], mixed=True)
    return _workload("stress", seed, n_layers, num_blocks, b.trace,
                     free_order=_perm(seed + 901, num_blocks), first_mixed=first_mixed,
                     hist=hist)


def by_index(i, **kw):
    return [tiny, pi05_frame, cross_frame, cross_task, stress][i](**kw)
