"""Binding of libbittrain_bench.so, the measurement aids that bench.py uses.

That library is the codec's source compiled once more with per-tile time stamps, plus a
dependency-free stream with the codec's traffic shape (csrc/bench_aids.h).  It is not part of
the product: nothing but the benchmark loads it.
"""
import ctypes
import os

from . import bittrain as bt

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbittrain_bench.so")

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libbittrain_bench.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        u64, vp, ci = ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int
        L.bt_stream_probe.restype = ci
        L.bt_stream_probe.argtypes = [vp, vp, u64, ci, ci, vp]
        L.bt_timeline_set.restype = ci
        L.bt_timeline_set.argtypes = [vp, u64, ctypes.c_uint32, ctypes.c_uint32]
        _lib = L
    return _lib


def bt_stream_probe(src, dst, tiles, read_rows, write_rows, stream=None):
    """A dependency-free stream of `tiles` workgroups reading read_rows and writing write_rows
    4 KiB rows each."""
    bt._dev(src, "src")
    bt._dev(dst, "dst")
    if bt._bytes(src) < tiles * read_rows * 4096 or bt._bytes(dst) < max(tiles * write_rows * 4096, 16 * tiles):
        raise ValueError("buffers too small for this many tiles")
    bt._check("bt_stream_probe", lib().bt_stream_probe(bt._ptr(src), bt._ptr(dst), tiles, read_rows, write_rows,
                                                       bt._stream(stream)))


def bt_timeline_set(buf, tiles, max_passes):
    """Switch the per-tile time stamps of THIS library's codec kernels on (buf: zeroed int64 device
    tensor) or off (buf None)."""
    if buf is None:
        bt._check("bt_timeline_set", lib().bt_timeline_set(None, 0, 0, 0))
        return
    bt._dev(buf, "buf")
    if buf.element_size() != 8:
        raise ValueError("buf must be a tensor of 64-bit integers")
    bt._check("bt_timeline_set", lib().bt_timeline_set(bt._ptr(buf), buf.numel(), tiles, max_passes))
