"""Runs workload traces (see synth) through the C-ABI library.

This is the frame driver in the order of the paper's Alg. 1: prefix of the new
frame -> fan-out to an action stream and a fresh language stream -> per step one
batch descriptor serving all layers (append, then mixed attention) -> release of
finished requests.  torch is used for device memory and the HIP stream only;
every step of the path runs inside liboxy.so.
"""
import numpy as np
import torch

from . import binding as B


def to_device_bf16(bits, device):
    """uint16 bit patterns (numpy) -> bf16 tensor on the device, bits unchanged."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device, non_blocking=False).view(torch.bfloat16)


def bits_of(t):
    """bf16 tensor -> uint16 bit patterns (numpy)."""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def trace_limits(trace):
    max_q = max([sum(n for _, n in op["items"]) for op in trace
                 if op["op"] == "step" and op.get("attend", True)] + [1])
    max_app = max([sum(n for _, n in op["items"]) for op in trace if op["op"] == "step"] + [1])
    return max_q, max_app


class GpuWorld:
    """Owns the device buffers of one pool and applies trace operations to it."""

    def __init__(self, workload, data_fn=None, layers=None, device="cuda:0", split_tokens=0,
                 stream_split_tokens=0,
                 max_live_batches=2, max_q_tokens=None, max_append_tokens=None,
                 max_work_items=0, max_partials=0, want_lse=True, poison=False,
                 fold_append=False):
        if not torch.cuda.is_available():
            raise RuntimeError("GpuWorld needs a GPU; there is no CPU fallback")
        w = workload
        self.w = w
        self.device = torch.device(device)
        self.n_layers = w["n_layers"]
        self.layers = list(range(self.n_layers)) if layers is None else list(layers)
        self.data_fn = data_fn
        self.scale = float(w["scale"])
        self.want_lse = want_lse
        self.fold_append = fold_append     # one call per layer: append inside the attention
        mq, ma = trace_limits(w["trace"])
        cfg = B.make_config(self.n_layers, w["num_blocks"], free_order=w.get("free_order"),
                            max_live_batches=max_live_batches,
                            max_q_tokens=max_q_tokens or mq, max_append_tokens=max_append_tokens or ma,
                            max_work_items=max_work_items, max_partials=max_partials,
                            split_tokens=split_tokens,
                            stream_split_tokens=stream_split_tokens)
        kv_bytes = B.oxy_kv_bytes(cfg)
        ws_bytes = B.oxy_workspace_bytes(cfg)
        if kv_bytes == 0 or ws_bytes == 0:
            raise ValueError("invalid pool configuration")
        self.kv = torch.empty(kv_bytes, dtype=torch.uint8, device=self.device)
        if poison:      # every bf16 of the pool is a NaN until something is appended
            self.kv.view(torch.int16).fill_(0x7FC1)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        cfg.kv_base, cfg.kv_bytes = self.kv.data_ptr(), kv_bytes
        cfg.workspace, cfg.workspace_bytes = self.ws.data_ptr(), ws_bytes
        self.cfg = cfg
        self.pool = B.oxy_pool_create(cfg)
        self.kinds = {}

    def close(self):
        if self.pool is not None:
            torch.cuda.synchronize(self.device)
            B.oxy_pool_destroy(self.pool)
            self.pool = None

    def _stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    # -- trace operations ---------------------------------------------------
    def apply(self, op):
        kind = op["op"]
        if kind == "prefix_create":
            return {"pid": B.oxy_prefix_create(self.pool)}
        if kind == "prefix_append":
            for layer in self.layers:
                k = to_device_bf16(self.data_fn(op["data"], layer, "k", op["n"]), self.device)
                v = to_device_bf16(self.data_fn(op["data"], layer, "v", op["n"]), self.device)
                B.oxy_prefix_append(self.pool, op["pid"], layer, k.data_ptr(), v.data_ptr(),
                                    op["n"], op["pos0"], self._stream())
            torch.cuda.synchronize(self.device)     # k, v go out of scope here
            blocks = B.oxy_prefix_blocks(self.pool, op["pid"])
            return {"slots": [blocks[t // 16] * 16 + t % 16
                              for t in range(op["pos0"], op["pos0"] + op["n"])]}
        if kind == "prefix_fork":
            return {"pid": B.oxy_prefix_fork(self.pool, op["parent"], op["n"])}
        if kind == "stream_create":
            sid = B.oxy_stream_create(self.pool, op["pid"], op["kind"])
            self.kinds[sid] = op["kind"]
            return {"sid": sid}
        if kind == "stream_rewind":
            B.oxy_stream_rewind(self.pool, op["sid"], op["len"])
            return {}
        if kind == "stream_release":
            B.oxy_stream_release(self.pool, op["sid"])
            return {}
        if kind == "prefix_release":
            B.oxy_prefix_release(self.pool, op["pid"])
            return {}
        if kind == "step":
            return self.step(op)
        raise ValueError("unknown op %r" % kind)

    def step(self, op):
        items = [tuple(it) for it in op["items"]]
        attend = op.get("attend", True)
        n_tok = sum(n for _, n in items)
        batch = B.oxy_batch_build(self.pool, items, 0 if attend else B.BATCH_APPEND_ONLY,
                                  self._stream())
        out = {"slots": B.oxy_batch_slots(batch), "O": {}, "LSE": {},
               "info": B.oxy_batch_info(batch)}
        try:
            for layer in self.layers:
                k = to_device_bf16(self.data_fn(op["data"], layer, "k", n_tok), self.device)
                v = to_device_bf16(self.data_fn(op["data"], layer, "v", n_tok), self.device)
                if not (attend and self.fold_append):
                    B.oxy_stream_append(self.pool, batch, layer, k.data_ptr(), v.data_ptr(),
                                        self._stream())
                if attend:
                    q = to_device_bf16(self.data_fn(op["data"], layer, "q", n_tok), self.device)
                    o = torch.empty_like(q)
                    lse = torch.empty((n_tok, 8), dtype=torch.float32, device=self.device) \
                        if self.want_lse else None
                    lse_ptr = lse.data_ptr() if lse is not None else 0
                    if self.fold_append:
                        B.oxy_append_attention(self.pool, batch, layer, k.data_ptr(), v.data_ptr(),
                                               q.data_ptr(), o.data_ptr(), lse_ptr, self.scale,
                                               self._stream())
                    else:
                        B.oxy_mixed_attention(self.pool, batch, layer, q.data_ptr(), o.data_ptr(),
                                              lse_ptr, self.scale, self._stream())
                    torch.cuda.synchronize(self.device)
                    out["O"][layer] = bits_of(o)
                    if lse is not None:
                        out["LSE"][layer] = lse.cpu().numpy()
                torch.cuda.synchronize(self.device)
        finally:
            B.oxy_batch_destroy(batch)
        return out

    def run(self, trace):
        return [self.apply(op) for op in trace]

    # -- read-back ------------------------------------------------------------
    def gather(self, layer, slots):
        n = len(slots)
        k = torch.empty((n, 256), dtype=torch.bfloat16, device=self.device)
        v = torch.empty_like(k)
        B.oxy_gather_kv(self.pool, layer, slots, k.data_ptr(), v.data_ptr(), self._stream())
        torch.cuda.synchronize(self.device)
        return bits_of(k), bits_of(v)

    def stream_slots(self, sid):
        _, _, own_len, _ = B.oxy_stream_info(self.pool, sid)
        blocks = B.oxy_stream_blocks(self.pool, sid)
        return [blocks[t // 16] * 16 + t % 16 for t in range(own_len)]

    def prefix_slots(self, pid):
        length = B.oxy_prefix_info(self.pool, pid)[0]
        blocks = B.oxy_prefix_blocks(self.pool, pid)
        return [blocks[t // 16] * 16 + t % 16 for t in range(length)]
