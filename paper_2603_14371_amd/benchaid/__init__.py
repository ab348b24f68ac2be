"""Benchmark-only measurement aids (a plain copy and a plain streaming read of known size),
in a shared object of their own so that liboxy.so holds the method only."""
import ctypes
import os

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libprobe.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("libprobe.so is not built: run `python -m paper_2603_14371_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.oxyprobe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.oxyprobe_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        L.oxyprobe_copy.restype = L.oxyprobe_read.restype = ctypes.c_int
        _lib = L
    return _lib


def copy(dst_ptr, src_ptr, n_bytes, stream):
    rc = _load().oxyprobe_copy(dst_ptr, src_ptr, n_bytes, stream or None)
    if rc:
        raise RuntimeError("oxyprobe_copy: hip error %d" % rc)


def read(src_ptr, n_bytes, sink_ptr, stream):
    rc = _load().oxyprobe_read(src_ptr, n_bytes, sink_ptr, stream or None)
    if rc:
        raise RuntimeError("oxyprobe_read: hip error %d" % rc)
