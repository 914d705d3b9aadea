"""TEST INFRASTRUCTURE ONLY: numpy front end of the C oracle ``bt_oracle.c``.

``build()`` compiles the C file with gcc into ``oracle/libbt_oracle.so``;
the functions below marshal numpy arrays and nothing else.  Arrays are passed
as raw bits: any dtype of item size 2, 4 or 8 works (fp16 and bf16 arrive as
``uint16`` views).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bt_oracle.c")
_LIB = os.path.join(_HERE, "libbt_oracle.so")
_lib = None


def build(force=True):
    """Compile the oracle.  Plain C, -O2, no threads, no vector pragmas."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        u64, vp, ci = ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int
        lib.bt_oracle_compressed_size.restype = u64
        lib.bt_oracle_compressed_size.argtypes = [u64, u64, ci]
        lib.bt_oracle_dense_size.restype = u64
        lib.bt_oracle_dense_size.argtypes = [u64, ci]
        lib.bt_oracle_compress.restype = u64
        lib.bt_oracle_compress.argtypes = [vp, u64, ci, vp, vp]
        lib.bt_oracle_decompress.restype = u64
        lib.bt_oracle_decompress.argtypes = [vp, vp, u64, ci, vp]
        lib.bt_oracle_relu_backward.restype = ci
        lib.bt_oracle_relu_backward.argtypes = [vp, vp, u64, ci, vp]
        lib.bt_oracle_prune.restype = u64
        lib.bt_oracle_prune.argtypes = [vp, u64, ci, ctypes.c_double, vp]
        lib.bt_oracle_coo_size.restype = u64
        lib.bt_oracle_coo_size.argtypes = [u64, ci, ci, ci]
        lib.bt_oracle_mask_apply.restype = ci
        lib.bt_oracle_mask_apply.argtypes = [vp, vp, u64, ci, vp]
        lib.bt_oracle_tile_index.restype = u64
        lib.bt_oracle_tile_index.argtypes = [vp, u64, u64, vp]
        _lib = lib
    return _lib


def _flat(a):
    a = np.ascontiguousarray(a).reshape(-1)
    if a.dtype.itemsize not in (2, 4, 8):
        raise ValueError("element width must be 2, 4 or 8 bytes")
    return a


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def compressed_size(n, nnz, width):
    return int(_load().bt_oracle_compressed_size(n, nnz, width))


def dense_size(n, width):
    return int(_load().bt_oracle_dense_size(n, width))


def compress(T):
    """Algorithm 1.  Returns (bitmap uint32[ceil(n/32)], values[nnz], nnz);
    values has T's dtype."""
    T = _flat(T)
    n = T.size
    bitmap = np.full((n + 31) // 32, 0xDEADBEEF, dtype=np.uint32)  # oracle must clear it
    values = np.empty(n, dtype=T.dtype)
    nnz = int(_load().bt_oracle_compress(_ptr(T), n, T.dtype.itemsize, _ptr(bitmap), _ptr(values)))
    assert nnz <= n
    return bitmap, values[:nnz].copy(), nnz


def decompress(bitmap, values, n):
    """Algorithm 2.  Returns the flat dense tensor of n elements (dtype of values)."""
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint32)
    values = _flat(values)
    assert bitmap.size == (n + 31) // 32
    out = np.empty(n, dtype=values.dtype)
    out.view(np.uint8)[:] = 0xA5  # every element must be overwritten
    used = int(_load().bt_oracle_decompress(_ptr(bitmap), _ptr(values), n, values.dtype.itemsize, _ptr(out)))
    assert used <= values.size, "bitmap has more set bits than there are values"
    return out


def relu_backward(bitmap, grad_out):
    """grad_in[i] = bit(i) ? grad_out[i] : +0."""
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint32)
    g = _flat(grad_out)
    n = g.size
    assert bitmap.size == (n + 31) // 32
    out = np.empty(n, dtype=g.dtype)
    out.view(np.uint8)[:] = 0xA5
    rc = _load().bt_oracle_relu_backward(_ptr(bitmap), _ptr(g), n, g.dtype.itemsize, _ptr(out))
    assert rc == 0
    return out


DTYPE_CODES = {"f32": 0, "f16": 1, "bf16": 2, "f64": 3}


def prune(T, dtype, threshold):
    """Section 4.3: keep elements whose value exceeds the threshold, +0 elsewhere.
    T holds raw bits (uint32 for "f32", uint16 for "f16" / "bf16", uint64 for "f64")."""
    T = _flat(T)
    code = DTYPE_CODES[dtype]
    assert T.dtype.itemsize == {0: 4, 1: 2, 2: 2, 3: 8}[code]
    out = np.empty_like(T)
    out.view(np.uint8)[:] = 0xA5
    kept = int(_load().bt_oracle_prune(_ptr(T), T.size, code, float(threshold), _ptr(out)))
    assert kept <= T.size
    return out


def compress_pruned(T, dtype, threshold):
    """Pruning followed by Algorithm 1: (bitmap, values, nnz)."""
    return compress(prune(T, dtype, threshold))


def coo_size(nnz, ndim, index_bytes, width):
    """M_c of Section 3.2."""
    return int(_load().bt_oracle_coo_size(nnz, ndim, index_bytes, width))


def mask_apply(bitmap, x):
    """Double mask (Section 3.1): out[i] = bit(i) ? x[i] : +0 with another tensor's bitmap."""
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint32)
    x = _flat(x)
    n = x.size
    assert bitmap.size == (n + 31) // 32
    out = np.empty(n, dtype=x.dtype)
    out.view(np.uint8)[:] = 0xA5
    rc = _load().bt_oracle_mask_apply(_ptr(bitmap), _ptr(x), n, x.dtype.itemsize, _ptr(out))
    assert rc == 0
    return out


def tile_index(bitmap, n, tile_elems):
    """Algorithm 2's counter j at elements 0, tile_elems, 2 * tile_elems, ...: uint64[ceil(n / tile_elems)]."""
    bitmap = np.ascontiguousarray(bitmap, dtype=np.uint32)
    assert bitmap.size == (n + 31) // 32 and tile_elems > 0
    tiles = (n + tile_elems - 1) // tile_elems
    index = np.full(tiles + 1, 0xA5A5A5A5A5A5A5A5, dtype=np.uint64)
    wrote = int(_load().bt_oracle_tile_index(_ptr(bitmap), n, tile_elems, _ptr(index)))
    assert wrote == tiles and index[tiles] == 0xA5A5A5A5A5A5A5A5
    return index[:tiles].copy()
