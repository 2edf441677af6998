"""ctypes binding of the measurement probes (include/distattn_probe.h, libdistattn_probe.so).  Marshalling only."""
import ctypes
import os

import torch

from . import distattn as da

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdistattn_probe.so")
EXPORTS = ["da_probe_read", "da_probe_copy", "da_probe_read_write"]

_lib = None


def lib():
    """The loaded probe library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.da_probe_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32, vp, vp]
        L.da_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.da_probe_read_write.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_size_t,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
        for name in EXPORTS:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _stream_ptr(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def probe_read(src, segment_bytes, workgroups, variant, sink, stream=None):
    """Enqueue one streaming read of the whole tensor ``src`` (da_probe_read)."""
    st = lib().da_probe_read(ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(), segment_bytes,
                             workgroups, variant, ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream))
    if st != da.DA_OK:
        raise da.DistAttnError(st, "da_probe_read")


def probe_copy(src, dst, stream=None):
    """Enqueue one plain copy of ``src`` into ``dst`` (da_probe_copy)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    st = lib().da_probe_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), nbytes, _stream_ptr(stream))
    if st != da.DA_OK:
        raise da.DistAttnError(st, "da_probe_copy")


def probe_read_write(src, dst, item_bytes, frag_bytes, workgroups, burst, staggered, sink, stream=None):
    """Enqueue one pass of da_probe_read_write over the whole tensor ``src``."""
    st = lib().da_probe_read_write(ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                                   ctypes.c_void_p(dst.data_ptr()), dst.numel() * dst.element_size(), item_bytes, frag_bytes,
                                   workgroups, burst, int(bool(staggered)), ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream))
    if st != da.DA_OK:
        raise da.DistAttnError(st, "da_probe_read_write")
