"""ctypes binding of liboxy.so: same names as include/oxy.h, argument marshalling only.

Device buffers are passed as integer addresses (torch tensors' data_ptr()); the HIP
stream as torch.cuda.current_stream().cuda_stream.  Every function raises OxyError
on a negative status.  There is no fallback: if the library is missing, loading fails.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboxy.so")

OK = 0
ERR_INVALID_ARG, ERR_NO_BLOCKS, ERR_BAD_ID, ERR_SEALED = -1, -2, -3, -4
ERR_BUSY, ERR_WORKSPACE, ERR_DEVICE = -5, -6, -7
KIND_ACTION, KIND_DECODE = 0, 1
POOL_HOST_ONLY = 1
BATCH_APPEND_ONLY = 1
STEP_FUSE_ACROSS_LAYERS = 1
STEP_FOLD_APPEND = 2
STEP_GRAPH = 4
SCHED_BATCHED, SCHED_UNBATCHED, SCHED_UPPER_BOUND = 0, 1, 2

EXPORTS = [
    "oxy_version", "oxy_last_error", "oxy_kv_bytes", "oxy_workspace_bytes", "oxy_pool_create",
    "oxy_pool_destroy", "oxy_prefix_create", "oxy_prefix_append", "oxy_prefix_append_layers",
    "oxy_prefix_fork",
    "oxy_prefix_release",
    "oxy_stream_create", "oxy_stream_release", "oxy_stream_rewind", "oxy_batch_build",
    "oxy_stream_append", "oxy_mixed_attention", "oxy_mixed_attention_static", "oxy_step_layers", "oxy_step_graph_stats",
    "oxy_append_attention",
    "oxy_batch_destroy",
    "oxy_gather_kv",
    "oxy_stream_info", "oxy_stream_blocks", "oxy_prefix_info", "oxy_prefix_blocks",
    "oxy_block_refcounts", "oxy_free_blocks", "oxy_pool_stats", "oxy_batch_info",
    "oxy_batch_slots", "oxy_batch_work",
    "oxy_sched_create", "oxy_sched_destroy", "oxy_sched_admit", "oxy_sched_next_step",
    "oxy_sched_end_frame", "oxy_sched_info", "oxy_sched_request_info", "oxy_sched_calibrate",
]


class OxyError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("oxy status %d: %s" % (code, message))
        self.code = code


class PoolConfig(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32),
        ("kv_base", ctypes.c_void_p), ("kv_bytes", ctypes.c_size_t),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("free_order", ctypes.POINTER(ctypes.c_int32)),
        ("max_live_batches", ctypes.c_int32), ("max_q_tokens", ctypes.c_int32),
        ("max_append_tokens", ctypes.c_int32), ("max_work_items", ctypes.c_int32),
        ("max_partials", ctypes.c_int32), ("split_tokens", ctypes.c_int32),
        ("stream_split_tokens", ctypes.c_int32),
        ("flags", ctypes.c_int32),
    ]


class SchedConfig(ctypes.Structure):
    _fields_ = [("k", ctypes.c_int32), ("denoise_steps", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("max_active", ctypes.c_int32), ("mode", ctypes.c_int32)]


class Item(ctypes.Structure):
    _fields_ = [("stream_id", ctypes.c_int32), ("n_new", ctypes.c_int32)]


_lib = None


def lib():
    """Loads the built library (build it first with paper_2603_14371_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("liboxy.so is not built: run `python -m paper_2603_14371_amd.build` "
                          "(or __graft_entry__.build()) first")
        # torch ships a HIP runtime of its own under the same library name as the system's: the
        # one that is loaded first serves the whole process, and device buffers come from torch,
        # so torch's has to be the one (the system's, loaded first, does not find the device
        # once torch's other libraries are in)
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        L.oxy_last_error.restype = ctypes.c_char_p
        L.oxy_kv_bytes.restype = ctypes.c_size_t
        L.oxy_workspace_bytes.restype = ctypes.c_size_t
        L.oxy_kv_bytes.argtypes = [ctypes.POINTER(PoolConfig)]
        L.oxy_workspace_bytes.argtypes = [ctypes.POINTER(PoolConfig)]
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        pi32 = ctypes.POINTER(ctypes.c_int32)
        sig = {
            "oxy_pool_create": [ctypes.POINTER(PoolConfig), ctypes.POINTER(vp)],
            "oxy_pool_destroy": [vp],
            "oxy_prefix_create": [vp, pi32],
            "oxy_prefix_append": [vp, i32, i32, vp, vp, i32, i32, vp],
            "oxy_prefix_append_layers": [vp, i32, i32, i32, vp, vp, ctypes.c_size_t, i32, i32, vp],
            "oxy_prefix_fork": [vp, i32, i32, pi32],
            "oxy_prefix_release": [vp, i32],
            "oxy_stream_create": [vp, i32, i32, pi32],
            "oxy_stream_release": [vp, i32],
            "oxy_stream_rewind": [vp, i32, i32],
            "oxy_batch_build": [vp, ctypes.POINTER(Item), i32, i32, vp, ctypes.POINTER(vp)],
            "oxy_stream_append": [vp, vp, i32, vp, vp, vp],
            "oxy_mixed_attention": [vp, vp, i32, vp, vp, vp, ctypes.c_float, vp],
            "oxy_mixed_attention_static": [vp, vp, i32, vp, vp, vp, ctypes.c_float, vp],
            "oxy_step_layers": [vp, vp, i32, i32, vp, vp, ctypes.c_size_t, vp, vp, ctypes.c_size_t,
                                vp, ctypes.c_size_t, ctypes.c_float, i32, ctypes.POINTER(vp), vp],
            "oxy_step_graph_stats": [vp, pi32, pi32, pi32],
            "oxy_append_attention": [vp, vp, i32, vp, vp, vp, vp, vp, ctypes.c_float, vp],
            "oxy_batch_destroy": [vp],
            "oxy_gather_kv": [vp, i32, ctypes.POINTER(ctypes.c_int64), i32, vp, vp, vp],
            "oxy_stream_info": [vp, i32, pi32, pi32, pi32, pi32],
            "oxy_stream_blocks": [vp, i32, pi32, i32],
            "oxy_prefix_info": [vp, i32, pi32, pi32, pi32, pi32],
            "oxy_prefix_blocks": [vp, i32, pi32, i32],
            "oxy_block_refcounts": [vp, pi32, i32],
            "oxy_free_blocks": [vp, pi32, i32],
            "oxy_pool_stats": [vp, pi32, pi32, pi32],
            "oxy_batch_info": [vp, pi32, pi32, pi32, pi32],
            "oxy_batch_slots": [vp, ctypes.POINTER(ctypes.c_int64), i32],
            "oxy_batch_work": [vp, pi32, i32],
            "oxy_sched_create": [vp, ctypes.POINTER(SchedConfig), ctypes.POINTER(vp)],
            "oxy_sched_destroy": [vp],
            "oxy_sched_admit": [vp, i32, i32, pi32],
            "oxy_sched_next_step": [vp, ctypes.POINTER(Item), i32, pi32, pi32],
            "oxy_sched_end_frame": [vp, pi32, i32, pi32],
            "oxy_sched_info": [vp, pi32, pi32, pi32, pi32],
            "oxy_sched_request_info": [vp, i32, pi32, pi32, pi32, pi32],
            "oxy_sched_calibrate": [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                    i32, ctypes.c_double, i32, i32, i32, ctypes.c_double, pi32,
                                    ctypes.POINTER(ctypes.c_double)],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = ctypes.c_int32
        _lib = L
    return _lib


def _check(status):
    if status != OK:
        raise OxyError(status, lib().oxy_last_error().decode())


def _i32():
    return ctypes.c_int32(0)


def oxy_version():
    return lib().oxy_version()


def oxy_last_error():
    return lib().oxy_last_error().decode()


def make_config(n_layers, num_blocks, kv_base=0, kv_bytes=0, workspace=0, workspace_bytes=0,
                free_order=None, max_live_batches=0, max_q_tokens=0, max_append_tokens=0,
                max_work_items=0, max_partials=0, split_tokens=0, stream_split_tokens=0, flags=0,
                n_q_heads=8, n_kv_heads=1, head_dim=256, page_size=16):
    cfg = PoolConfig(n_layers, n_q_heads, n_kv_heads, head_dim, page_size, num_blocks,
                     kv_base or None, kv_bytes, workspace or None, workspace_bytes, None,
                     max_live_batches, max_q_tokens, max_append_tokens, max_work_items,
                     max_partials, split_tokens, stream_split_tokens, flags)
    if free_order is not None:
        arr = np.ascontiguousarray(free_order, dtype=np.int32)
        cfg._keep = arr
        cfg.free_order = arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    return cfg


def oxy_kv_bytes(cfg):
    return lib().oxy_kv_bytes(ctypes.byref(cfg))


def oxy_workspace_bytes(cfg):
    return lib().oxy_workspace_bytes(ctypes.byref(cfg))


def oxy_pool_create(cfg):
    out = ctypes.c_void_p()
    _check(lib().oxy_pool_create(ctypes.byref(cfg), ctypes.byref(out)))
    return out


def oxy_pool_destroy(pool):
    _check(lib().oxy_pool_destroy(pool))


def oxy_prefix_create(pool):
    out = _i32()
    _check(lib().oxy_prefix_create(pool, ctypes.byref(out)))
    return out.value


def oxy_prefix_append(pool, prefix_id, layer, k_ptr, v_ptr, n_tokens, pos0, stream):
    _check(lib().oxy_prefix_append(pool, prefix_id, layer, k_ptr or None, v_ptr or None, n_tokens,
                                   pos0, stream or None))


def oxy_prefix_append_layers(pool, prefix_id, layer_begin, layer_end, k_ptr, v_ptr, layer_stride,
                             n_tokens, pos0, stream):
    _check(lib().oxy_prefix_append_layers(pool, prefix_id, layer_begin, layer_end, k_ptr or None,
                                          v_ptr or None, layer_stride, n_tokens, pos0,
                                          stream or None))


def oxy_prefix_fork(pool, parent_prefix_id, n_tokens):
    out = _i32()
    _check(lib().oxy_prefix_fork(pool, parent_prefix_id, n_tokens, ctypes.byref(out)))
    return out.value


def oxy_prefix_release(pool, prefix_id):
    _check(lib().oxy_prefix_release(pool, prefix_id))


def oxy_stream_create(pool, prefix_id, kind):
    out = _i32()
    _check(lib().oxy_stream_create(pool, prefix_id, kind, ctypes.byref(out)))
    return out.value


def oxy_stream_release(pool, stream_id):
    _check(lib().oxy_stream_release(pool, stream_id))


def oxy_stream_rewind(pool, stream_id, new_len):
    _check(lib().oxy_stream_rewind(pool, stream_id, new_len))


def oxy_batch_build(pool, items, flags, stream):
    arr = (Item * len(items))(*[Item(int(s), int(n)) for s, n in items])
    out = ctypes.c_void_p()
    _check(lib().oxy_batch_build(pool, arr, len(items), flags, stream or None, ctypes.byref(out)))
    return out


def oxy_stream_append(pool, batch, layer, k_ptr, v_ptr, stream):
    _check(lib().oxy_stream_append(pool, batch, layer, k_ptr, v_ptr, stream or None))


def oxy_mixed_attention(pool, batch, layer, q_ptr, out_ptr, lse_ptr, scale, stream):
    _check(lib().oxy_mixed_attention(pool, batch, layer, q_ptr, out_ptr, lse_ptr or None,
                                     ctypes.c_float(scale), stream or None))


def oxy_mixed_attention_static(pool, batch, layer, q_ptr, out_ptr, lse_ptr, scale, stream):
    _check(lib().oxy_mixed_attention_static(pool, batch, layer, q_ptr, out_ptr, lse_ptr or None,
                                            ctypes.c_float(scale), stream or None))


def oxy_step_layers(pool, batch, layer_begin, layer_end, k_ptr, v_ptr, kv_layer_stride, q_ptr,
                    out_ptr, q_layer_stride, lse_ptr, lse_layer_stride, scale, flags, events, stream):
    """events: None or a ctypes array of 4*(layer_end-layer_begin) raw hipEvent_t handles."""
    _check(lib().oxy_step_layers(pool, batch, layer_begin, layer_end, k_ptr, v_ptr, kv_layer_stride,
                                 q_ptr, out_ptr, q_layer_stride, lse_ptr or None, lse_layer_stride,
                                 ctypes.c_float(scale), flags, events, stream or None))


def oxy_step_graph_stats(pool):
    """(instantiations, updates, replays) of OXY_STEP_GRAPH on this pool."""
    a, b, c = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().oxy_step_graph_stats(pool, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def oxy_append_attention(pool, batch, layer, k_ptr, v_ptr, q_ptr, out_ptr, lse_ptr, scale, stream):
    _check(lib().oxy_append_attention(pool, batch, layer, k_ptr, v_ptr, q_ptr, out_ptr,
                                      lse_ptr or None, ctypes.c_float(scale), stream or None))


def oxy_batch_destroy(batch):
    _check(lib().oxy_batch_destroy(batch))


def oxy_gather_kv(pool, layer, slots, k_out_ptr, v_out_ptr, stream):
    arr = np.ascontiguousarray(slots, dtype=np.int64)
    _check(lib().oxy_gather_kv(pool, layer, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                               len(arr), k_out_ptr, v_out_ptr, stream or None))


def oxy_stream_info(pool, stream_id):
    """-> (prefix_id, kind, own_len, n_blocks)"""
    a, b, c, d = _i32(), _i32(), _i32(), _i32()
    _check(lib().oxy_stream_info(pool, stream_id, ctypes.byref(a), ctypes.byref(b),
                                 ctypes.byref(c), ctypes.byref(d)))
    return a.value, b.value, c.value, d.value


def _int_array(n):
    return np.zeros(max(n, 1), dtype=np.int32)


def _p32(arr):
    return arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def oxy_stream_blocks(pool, stream_id):
    n = oxy_stream_info(pool, stream_id)[3]
    out = _int_array(n)
    _check(lib().oxy_stream_blocks(pool, stream_id, _p32(out), n))
    return out[:n].tolist()


def oxy_prefix_info(pool, prefix_id):
    """-> (len, n_blocks, sealed, n_streams)"""
    a, b, c, d = _i32(), _i32(), _i32(), _i32()
    _check(lib().oxy_prefix_info(pool, prefix_id, ctypes.byref(a), ctypes.byref(b),
                                 ctypes.byref(c), ctypes.byref(d)))
    return a.value, b.value, c.value, d.value


def oxy_prefix_blocks(pool, prefix_id):
    n = oxy_prefix_info(pool, prefix_id)[1]
    out = _int_array(n)
    _check(lib().oxy_prefix_blocks(pool, prefix_id, _p32(out), n))
    return out[:n].tolist()


def oxy_pool_stats(pool):
    """-> (free_blocks, live_prefixes, live_streams)"""
    a, b, c = _i32(), _i32(), _i32()
    _check(lib().oxy_pool_stats(pool, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def oxy_block_refcounts(pool, num_blocks):
    out = _int_array(num_blocks)
    _check(lib().oxy_block_refcounts(pool, _p32(out), num_blocks))
    return out.tolist()


def oxy_free_blocks(pool):
    n = oxy_pool_stats(pool)[0]
    out = _int_array(n)
    _check(lib().oxy_free_blocks(pool, _p32(out), n))
    return out[:n].tolist()


def oxy_batch_info(batch):
    """-> (n_items, n_tokens, n_work, n_partials)"""
    a, b, c, d = _i32(), _i32(), _i32(), _i32()
    _check(lib().oxy_batch_info(batch, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                ctypes.byref(d)))
    return a.value, b.value, c.value, d.value


def oxy_batch_slots(batch):
    n = oxy_batch_info(batch)[1]
    out = np.zeros(n, dtype=np.int64)
    _check(lib().oxy_batch_slots(batch, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), n))
    return out.tolist()


def oxy_batch_work(batch):
    n = oxy_batch_info(batch)[2]
    out = np.zeros((max(n, 1), 8), dtype=np.int32)
    _check(lib().oxy_batch_work(batch, _p32(out), n))
    return out[:n]


def oxy_sched_create(pool, k, denoise_steps, chunk, max_active=0, mode=SCHED_BATCHED):
    cfg = SchedConfig(k, denoise_steps, chunk, max_active, mode)
    out = ctypes.c_void_p()
    _check(lib().oxy_sched_create(pool, ctypes.byref(cfg), ctypes.byref(out)))
    return out


def oxy_sched_destroy(sched):
    _check(lib().oxy_sched_destroy(sched))


def oxy_sched_admit(sched, prefix_id, target_len):
    rid = _i32()
    _check(lib().oxy_sched_admit(sched, prefix_id, target_len, ctypes.byref(rid)))
    return rid.value


def oxy_sched_next_step(sched, cap=4096):
    """Returns (items, n_action_items); items == [] when the frame has no more steps."""
    arr = (Item * cap)()
    n, na = _i32(), _i32()
    _check(lib().oxy_sched_next_step(sched, arr, cap, ctypes.byref(n), ctypes.byref(na)))
    return [(arr[i].stream_id, arr[i].n_new) for i in range(n.value)], na.value


def oxy_sched_end_frame(sched, cap=4096):
    out = (ctypes.c_int32 * cap)()
    n = _i32()
    _check(lib().oxy_sched_end_frame(sched, out, cap, ctypes.byref(n)))
    return list(out[:n.value])


def oxy_sched_info(sched):
    a, b, c, d = _i32(), _i32(), _i32(), _i32()
    _check(lib().oxy_sched_info(sched, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                ctypes.byref(d)))
    return a.value, b.value, c.value, d.value


def oxy_sched_request_info(sched, request_id):
    a, b, c, d = _i32(), _i32(), _i32(), _i32()
    _check(lib().oxy_sched_request_info(sched, request_id, ctypes.byref(a), ctypes.byref(b),
                                        ctypes.byref(c), ctypes.byref(d)))
    return a.value, b.value, c.value, d.value


def oxy_sched_calibrate(t_mixed, t_decode, t_observation, denoise_steps, target_len,
                        arrivals_per_frame, frame_budget):
    """Returns (k, modelled frame time at k); k == 0 if no budget meets frame_budget."""
    n = len(t_mixed)
    assert len(t_decode) == n
    a = (ctypes.c_double * n)(*t_mixed)
    b = (ctypes.c_double * n)(*t_decode)
    k, t = _i32(), ctypes.c_double(0.0)
    _check(lib().oxy_sched_calibrate(a, b, n, t_observation, denoise_steps, target_len,
                                     arrivals_per_frame, frame_budget, ctypes.byref(k),
                                     ctypes.byref(t)))
    return k.value, t.value
