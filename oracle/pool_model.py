"""Indexing oracle: a small Python model of the paged, refcounted KV block pool.

Test infrastructure only; shares no code with the C++ library it checks.

The paper's manager (Sec. 3.2; App. A.2) keeps one resumable state per request
and exposes Store / Retrieve / Update / Remove plus Batch / UnBatch.  The KV
part of that state is modelled here as (prefix reference, own block table, own
length).  The paper has no allocator, so the policy below is this build's
specification and the library must follow it exactly (block tables, slots and
refcounts are compared bit for bit):

* LIFO free stack.  It starts as `free_order` with its first element on top.
* Blocks are popped one at a time in logical order; inside one batch build all
  blocks of item 0 come before those of item 1.
* A prefix allocates blocks when an append first reaches a token range, in
  ascending logical order; each starts with refcount 1 (the creator's handle).
* Attaching a stream seals the prefix (the action expert's view of the prefill
  cache is read-only, Sec. 1) and adds 1 to every prefix block's refcount.
* Own tokens of a stream always start at offset 0 of the stream's own first
  block; the tail of a partial last prefix page stays dead.
* Release subtracts 1 per table entry and pushes, in ascending logical order,
  the blocks that reach 0: a stream's own table first, then its prefix's table.
* Request ids are sequential and never reused: the id is the number of requests
  created before it (App. A.2, "r_t is the total number of requests created so
  far"); prefix ids and stream ids are separate counters.
* An ACTION item is rewound to length 0 at every batch build (its chunk K/V is
  transient per denoising step and reuses the same blocks); a DECODE item grows.
* A failing call changes nothing (NO_BLOCKS is detected before any pop).
* Fork (an extension beyond the paper, for prefixes of consecutive frames that begin with
  the same history segment): the child prefix starts with the parent's first n tokens, n a
  multiple of the page size, by listing the parent's blocks (refcount + 1 each); the shared
  range becomes read-only in both (an append below it fails with SEALED); the child appends
  behind it into blocks of its own.  Release treats shared blocks like any other entry.
"""

ACTION = 0
DECODE = 1

OK = 0
ERR_INVALID_ARG = -1
ERR_NO_BLOCKS = -2
ERR_BAD_ID = -3
ERR_SEALED = -4


class PoolError(Exception):
    def __init__(self, code, what=""):
        super().__init__("%d %s" % (code, what))
        self.code = code


class _Prefix:
    def __init__(self):
        self.blocks = []
        self.length = 0
        self.sealed = False
        self.handle = True      # creator's reference still held
        self.n_streams = 0
        self.frozen = 0         # tokens below this position are shared with a fork


class _Stream:
    def __init__(self, prefix_id, kind):
        self.prefix_id = prefix_id
        self.kind = kind
        self.blocks = []
        self.length = 0


class PoolModel:
    def __init__(self, num_blocks, page_size=16, n_layers=1, free_order=None):
        order = list(range(num_blocks)) if free_order is None else list(free_order)
        if sorted(order) != list(range(num_blocks)):
            raise PoolError(ERR_INVALID_ARG, "free_order is not a permutation")
        self.num_blocks = num_blocks
        self.page = page_size
        self.n_layers = n_layers
        self.free = order[::-1]                 # top of stack = end of list
        self.ref = [0] * num_blocks
        self.prefixes = {}
        self.streams = {}
        self.next_prefix_id = 0
        self.next_stream_id = 0

    # -- helpers -----------------------------------------------------------
    def _blocks_for(self, n_tokens):
        return (n_tokens + self.page - 1) // self.page

    def _pop(self):
        b = self.free.pop()
        self.ref[b] = 1
        return b

    def _unref_table(self, table):
        for b in table:                         # ascending logical order
            self.ref[b] -= 1
            if self.ref[b] == 0:
                self.free.append(b)

    def _maybe_drop_prefix(self, pid):
        p = self.prefixes[pid]
        if not p.handle and p.n_streams == 0:
            del self.prefixes[pid]

    # -- prefixes ----------------------------------------------------------
    def prefix_create(self):
        pid = self.next_prefix_id
        self.next_prefix_id += 1
        self.prefixes[pid] = _Prefix()
        return pid

    def prefix_append(self, pid, layer, n_tokens, pos0):
        """Returns the slots (block*page + offset) of tokens pos0 .. pos0+n_tokens-1."""
        p = self.prefixes.get(pid)
        if p is None or not p.handle:
            raise PoolError(ERR_BAD_ID)
        if not (0 <= layer < self.n_layers) or n_tokens < 1 or pos0 < 0 or pos0 > p.length:
            raise PoolError(ERR_INVALID_ARG)
        if p.sealed or pos0 < p.frozen:
            raise PoolError(ERR_SEALED)
        need = self._blocks_for(pos0 + n_tokens) - len(p.blocks)
        if need > len(self.free):
            raise PoolError(ERR_NO_BLOCKS)
        for _ in range(max(need, 0)):
            p.blocks.append(self._pop())
        p.length = max(p.length, pos0 + n_tokens)
        return [p.blocks[t // self.page] * self.page + t % self.page
                for t in range(pos0, pos0 + n_tokens)]

    def prefix_fork(self, parent_id, n_tokens):
        """New prefix whose tokens 0 .. n_tokens-1 are the parent's (same blocks)."""
        p = self.prefixes.get(parent_id)
        if p is None:
            raise PoolError(ERR_BAD_ID)
        if n_tokens < 0 or n_tokens % self.page != 0 or n_tokens > p.length:
            raise PoolError(ERR_INVALID_ARG)
        pid = self.next_prefix_id
        self.next_prefix_id += 1
        c = _Prefix()
        c.blocks = p.blocks[:n_tokens // self.page]
        for b in c.blocks:
            self.ref[b] += 1
        c.length = c.frozen = n_tokens
        p.frozen = max(p.frozen, n_tokens)
        self.prefixes[pid] = c
        return pid

    def prefix_release(self, pid):
        p = self.prefixes.get(pid)
        if p is None or not p.handle:
            raise PoolError(ERR_BAD_ID)
        p.handle = False
        self._unref_table(p.blocks)
        self._maybe_drop_prefix(pid)

    # -- streams -----------------------------------------------------------
    def stream_create(self, pid, kind):
        if kind not in (ACTION, DECODE):
            raise PoolError(ERR_INVALID_ARG)
        if pid != -1:
            p = self.prefixes.get(pid)
            if p is None or not p.handle:
                raise PoolError(ERR_BAD_ID)
            p.sealed = True
            p.n_streams += 1
            for b in p.blocks:
                self.ref[b] += 1
        sid = self.next_stream_id
        self.next_stream_id += 1
        self.streams[sid] = _Stream(pid, kind)
        return sid

    def stream_rewind(self, sid, new_len):
        s = self.streams.get(sid)
        if s is None:
            raise PoolError(ERR_BAD_ID)
        if not (0 <= new_len <= s.length):
            raise PoolError(ERR_INVALID_ARG)
        s.length = new_len

    def stream_release(self, sid):
        s = self.streams.get(sid)
        if s is None:
            raise PoolError(ERR_BAD_ID)
        del self.streams[sid]
        self._unref_table(s.blocks)
        if s.prefix_id != -1:
            p = self.prefixes[s.prefix_id]
            self._unref_table(p.blocks)
            p.n_streams -= 1
            self._maybe_drop_prefix(s.prefix_id)

    # -- Batch (Alg. 1, "Batch" + the length part of "Update") -------------
    def batch_build(self, items):
        """items: list of (stream_id, n_new).  Returns the slot of every new token,
        items in order, tokens in order."""
        if len(items) < 1:
            raise PoolError(ERR_INVALID_ARG)
        seen = set()
        plan = []
        need_total = 0
        for sid, n_new in items:
            s = self.streams.get(sid)
            if s is None:
                raise PoolError(ERR_BAD_ID)
            if n_new < 1 or sid in seen:
                raise PoolError(ERR_INVALID_ARG)
            seen.add(sid)
            old_len = 0 if s.kind == ACTION else s.length
            new_len = old_len + n_new
            need = max(0, self._blocks_for(new_len) - len(s.blocks))
            need_total += need
            plan.append((s, old_len, new_len, need))
        if need_total > len(self.free):
            raise PoolError(ERR_NO_BLOCKS)
        slots = []
        for s, old_len, new_len, need in plan:
            for _ in range(need):
                s.blocks.append(self._pop())
            s.length = new_len
            slots.extend(s.blocks[t // self.page] * self.page + t % self.page
                         for t in range(old_len, new_len))
        return slots

    # -- introspection -----------------------------------------------------
    def stats(self):
        return len(self.free), len(self.prefixes), len(self.streams)
