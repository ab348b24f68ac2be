"""Replays an operation trace on the un-paged truth: pool_model for indexing,
attention for values.  Test infrastructure only.

A trace is a list of plain dicts (no code of either implementation inside):

  {"op": "prefix_create", "pid": expected id}
  {"op": "prefix_append", "pid", "n", "pos0", "data": recipe}       every layer gets its own data
  {"op": "prefix_fork", "parent", "n", "pid": expected id}          child starts as parent[:n]
  {"op": "stream_create", "pid" (-1 = none), "kind", "sid": expected id}
  {"op": "stream_rewind", "sid", "len"}
  {"op": "step", "items": [(sid, n_new), ...], "data": recipe, "attend": bool}
  {"op": "stream_release", "sid"} / {"op": "prefix_release", "pid"}

`data_fn(recipe, layer, what, n)` supplies bf16 bit patterns: what in {"k","v"}
gives [n, d] uint16, what == "q" gives [n, H, d] uint16.  It is handed in by the
caller; the oracle generates no inputs itself.

The order of operations is the paper's Alg. 1: prefill cache of the new frame,
fan-out to the action expert and a fresh language request, batched decoding of
all active requests, eviction of finished ones.  The truth kept per stream is
the logical (un-paged, un-shared) token list per layer, so a shared prefix is
read here exactly as an isolated per-task copy would be.
"""
import numpy as np

from . import attention
from .pool_model import PoolModel, ACTION


class OracleWorld:
    def __init__(self, num_blocks, n_layers, data_fn, scale, page_size=16,
                 free_order=None, layers=None):
        self.pool = PoolModel(num_blocks, page_size, n_layers, free_order)
        self.n_layers = n_layers
        self.layers = list(range(n_layers)) if layers is None else list(layers)
        self.data_fn = data_fn
        self.scale = scale
        self.prefix_kv = {}     # pid -> {layer: (k_bits [P,d], v_bits [P,d])}
        self.stream_kv = {}     # sid -> {layer: [k_bits [n,d], v_bits [n,d]]}
        self.stream_meta = {}   # sid -> (pid, kind)

    # each handler returns what the GPU side can be compared with
    def apply(self, op):
        kind = op["op"]
        if kind == "prefix_create":
            pid = self.pool.prefix_create()
            self.prefix_kv[pid] = {}
            return {"pid": pid}
        if kind == "prefix_append":
            pid, n, pos0 = op["pid"], op["n"], op["pos0"]
            slots = None
            for layer in range(self.n_layers):
                slots = self.pool.prefix_append(pid, layer, n, pos0)
            for layer in self.layers:
                k = self.data_fn(op["data"], layer, "k", n)
                v = self.data_fn(op["data"], layer, "v", n)
                old = self.prefix_kv[pid].get(layer)
                if old is None:
                    old = (np.zeros((0, k.shape[1]), np.uint16),) * 2
                # tokens [pos0, pos0+n) are (over)written, everything else stays: the
                # logical length is max(old length, pos0+n), as in the pool model
                self.prefix_kv[pid][layer] = tuple(
                    np.concatenate([o[:pos0], new, o[pos0 + n:]]) for o, new in zip(old, (k, v)))
            return {"slots": slots}
        if kind == "prefix_fork":
            pid = self.pool.prefix_fork(op["parent"], op["n"])
            self.prefix_kv[pid] = {layer: (k[:op["n"]].copy(), v[:op["n"]].copy())
                                   for layer, (k, v) in self.prefix_kv[op["parent"]].items()}
            return {"pid": pid}
        if kind == "stream_create":
            sid = self.pool.stream_create(op["pid"], op["kind"])
            self.stream_kv[sid] = {}
            self.stream_meta[sid] = (op["pid"], op["kind"])
            return {"sid": sid}
        if kind == "stream_rewind":
            self.pool.stream_rewind(op["sid"], op["len"])
            for layer, kv in self.stream_kv[op["sid"]].items():
                kv[0], kv[1] = kv[0][:op["len"]], kv[1][:op["len"]]
            return {}
        if kind == "stream_release":
            self.pool.stream_release(op["sid"])
            del self.stream_kv[op["sid"]]
            del self.stream_meta[op["sid"]]
            return {}
        if kind == "prefix_release":
            self.pool.prefix_release(op["pid"])
            return {}
        if kind == "step":
            return self._step(op)
        raise ValueError("unknown op %r" % kind)

    def _step(self, op):
        items = [tuple(it) for it in op["items"]]
        slots = self.pool.batch_build(items)
        n_tok = sum(n for _, n in items)
        out = {"slots": slots, "O": {}, "LSE": {}}
        for layer in self.layers:
            k_new = self.data_fn(op["data"], layer, "k", n_tok)
            v_new = self.data_fn(op["data"], layer, "v", n_tok)
            t0 = 0
            for sid, n_new in items:
                pid, kind = self.stream_meta[sid]
                kv = self.stream_kv[sid].get(layer)
                d = k_new.shape[1]
                if kv is None or kind == ACTION:
                    kv = [np.zeros((0, d), np.uint16), np.zeros((0, d), np.uint16)]
                kv = [np.concatenate([kv[0], k_new[t0:t0 + n_new]]),
                      np.concatenate([kv[1], v_new[t0:t0 + n_new]])]
                self.stream_kv[sid][layer] = kv
                t0 += n_new
            if not op.get("attend", True):
                continue
            q = self.data_fn(op["data"], layer, "q", n_tok)
            o_all = np.empty(q.shape, np.float64)
            lse_all = np.empty(q.shape[:2], np.float64)
            t0 = 0
            for sid, n_new in items:
                pid, kind = self.stream_meta[sid]
                ko, vo = self.stream_kv[sid][layer]
                if pid == -1:
                    kp = vp = np.zeros((0, ko.shape[1]), np.uint16)
                else:
                    kp, vp = self.prefix_kv[pid][layer]
                o_all[t0:t0 + n_new], lse_all[t0:t0 + n_new] = attention.attend_item(
                    kind, q[t0:t0 + n_new], kp, vp, ko, vo, self.scale)
                t0 += n_new
            out["O"][layer] = o_all
            out["LSE"][layer] = lse_all
        return out

    def run(self, trace):
        return [self.apply(op) for op in trace]
