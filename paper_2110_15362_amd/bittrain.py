"""Thin binding over the C-ABI library ``libbittrain.so``.

Argument marshalling only: every step of the codec runs in the HIP kernels of
the library.  PyTorch supplies device memory and the stream, nothing else.
There is no CPU fallback: if the library is missing, or a call fails, this
module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbittrain.so")

BT_F32, BT_F16, BT_BF16, BT_F64 = 0, 1, 2, 3
# 32-bit words of a workspace that a caller may look at (BT_WS_* of the C header)
BT_WS_ERROR_WORD, BT_WS_WAIT_LIMIT_WORD, BT_WS_PATIENCE_WORD, BT_WS_WIDE_WORD = 2, 3, 4, 5
BT_STATIC_MAX_TILES = 16384
BT_OK = 0
STATUS_NAMES = {0: "BT_OK", 1: "BT_ERR_NULL", 2: "BT_ERR_DTYPE", 3: "BT_ERR_ALIGN", 4: "BT_ERR_WORKSPACE",
                5: "BT_ERR_HIP", 6: "BT_ERR_SIZE", 7: "BT_ERR_UNSUPPORTED"}
BT_MAX_ELEMENTS = 1 << 37

_DTYPES = {torch.float32: BT_F32, torch.float16: BT_F16, torch.bfloat16: BT_BF16, torch.float64: BT_F64}

_lib = None


class BitTrainError(RuntimeError):
    def __init__(self, call, status):
        self.status = status
        super().__init__("%s failed: %s (%s)" % (call, STATUS_NAMES.get(status, status), status_str(status)))


class CompressItem(ctypes.Structure):
    """bt_compress_item of the C header."""
    _fields_ = [("d_in", ctypes.c_void_p), ("n", ctypes.c_uint64), ("d_bitmap", ctypes.c_void_p),
                ("d_values", ctypes.c_void_p), ("values_cap", ctypes.c_uint64), ("d_nnz", ctypes.c_void_p),
                ("d_index", ctypes.c_void_p), ("d_dense_out", ctypes.c_void_p)]


class DecompressItem(ctypes.Structure):
    """bt_decompress_item of the C header."""
    _fields_ = [("d_bitmap", ctypes.c_void_p), ("d_values", ctypes.c_void_p), ("n", ctypes.c_uint64),
                ("d_out", ctypes.c_void_p), ("values_cap", ctypes.c_uint64), ("d_index", ctypes.c_void_p)]


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libbittrain.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        u64, sz, vp, ci = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int
        L.bt_compressed_size.restype, L.bt_compressed_size.argtypes = sz, [u64, u64, ci]
        L.bt_bitmap_bytes.restype, L.bt_bitmap_bytes.argtypes = sz, [u64]
        L.bt_workspace_bytes.restype, L.bt_workspace_bytes.argtypes = sz, [u64, ci]
        L.bt_dtype_size.restype, L.bt_dtype_size.argtypes = sz, [ci]
        L.bt_status_str.restype, L.bt_status_str.argtypes = ctypes.c_char_p, [ci]
        L.bt_workspace_init.restype, L.bt_workspace_init.argtypes = ci, [vp, sz, vp]
        L.bt_compress.restype = ci
        L.bt_compress.argtypes = [vp, u64, ci, vp, vp, u64, vp, vp, sz, vp]
        L.bt_compress_static.restype = ci
        L.bt_compress_static.argtypes = [vp, u64, ci, vp, vp, u64, vp, vp]
        L.bt_compress_pruned.restype = ci
        L.bt_compress_pruned.argtypes = [vp, u64, ci, ctypes.c_double, vp, vp, u64, vp, vp, sz, vp]
        L.bt_activation_compress.restype = ci
        L.bt_activation_compress.argtypes = [vp, u64, ci, ctypes.c_double, vp, vp, vp, u64, vp, vp, sz, vp]
        L.bt_decompress.restype = ci
        L.bt_decompress.argtypes = [vp, vp, u64, ci, vp, vp, sz, vp]
        L.bt_relu_backward_from_bitmap.restype = ci
        L.bt_relu_backward_from_bitmap.argtypes = [vp, vp, u64, ci, vp, vp]
        L.bt_dense_size.restype, L.bt_dense_size.argtypes = sz, [u64, ci]
        L.bt_coo_size.restype, L.bt_coo_size.argtypes = sz, [u64, ctypes.c_uint32, ctypes.c_uint32, ci]
        L.bt_mask_apply.restype = ci
        L.bt_mask_apply.argtypes = [vp, vp, u64, ci, vp, vp]
        L.bt_tile_elems.restype, L.bt_tile_elems.argtypes = sz, [ci]
        L.bt_index_bytes.restype, L.bt_index_bytes.argtypes = sz, [u64, ci]
        L.bt_compress_indexed.restype = ci
        L.bt_compress_indexed.argtypes = [vp, u64, ci, vp, vp, u64, vp, vp, vp, sz, vp]
        L.bt_decompress_indexed.restype = ci
        L.bt_decompress_indexed.argtypes = [vp, vp, u64, vp, u64, ci, vp, vp]
        L.bt_batch_workspace_bytes.restype = sz
        L.bt_batch_workspace_bytes.argtypes = [ctypes.POINTER(u64), sz, ci]
        L.bt_compress_batch.restype = ci
        L.bt_compress_batch.argtypes = [ctypes.POINTER(CompressItem), sz, ci, vp, sz, vp]
        L.bt_decompress_batch.restype = ci
        L.bt_decompress_batch.argtypes = [ctypes.POINTER(DecompressItem), sz, ci, vp, sz, vp]
        L.bt_compress_batch_pruned.restype = ci
        L.bt_compress_batch_pruned.argtypes = [ctypes.POINTER(CompressItem), sz, ci, ctypes.c_double, vp, sz, vp]
        L.bt_decompress_batch_indexed.restype = ci
        L.bt_decompress_batch_indexed.argtypes = [ctypes.POINTER(DecompressItem), sz, ci, vp]
        L.bt_workspace_status.restype = ci
        L.bt_workspace_status.argtypes = [vp, vp, vp]
        _lib = L
    return _lib


def status_str(status):
    return lib().bt_status_str(int(status)).decode()


def dtype_code(dtype):
    try:
        return _DTYPES[dtype]
    except KeyError:
        raise TypeError("libbittrain handles float64, float32, float16 and bfloat16, not %s" % dtype)


def bt_compressed_size(n, nnz, dtype):
    return int(lib().bt_compressed_size(n, nnz, dtype if isinstance(dtype, int) else dtype_code(dtype)))


def _code(dtype):
    return dtype if isinstance(dtype, int) else dtype_code(dtype)


def bt_dense_size(n, dtype):
    return int(lib().bt_dense_size(n, _code(dtype)))


def bt_coo_size(nnz, ndim, index_bytes, dtype):
    return int(lib().bt_coo_size(nnz, ndim, index_bytes, _code(dtype)))


def bt_bitmap_bytes(n):
    return int(lib().bt_bitmap_bytes(n))


def bt_workspace_bytes(n, dtype):
    return int(lib().bt_workspace_bytes(n, dtype if isinstance(dtype, int) else dtype_code(dtype)))


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None else 0)


def _check(call, status):
    if status != BT_OK:
        raise BitTrainError(call, status)


def _dev(t, name):
    if not t.is_cuda:
        raise ValueError("%s must live in device memory" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)


def new_workspace(n, dtype, device="cuda", stream=None):
    """Allocate and initialise a workspace for tensors of up to n elements."""
    ws = torch.empty(bt_workspace_bytes(n, dtype), dtype=torch.uint8, device=device)
    bt_workspace_init(ws, stream)
    return ws


def bt_workspace_init(workspace, stream=None):
    _dev(workspace, "workspace")
    _check("bt_workspace_init", lib().bt_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                                        _stream(stream)))


def bt_compress(x, bitmap, values, nnz, workspace, stream=None):
    """Algorithm 1 on device tensors.  x: dense tensor (any shape, contiguous);
    bitmap: int32[ceil(n/32)]; values: x.dtype[cap]; nnz: int64[1]; all on x's
    device.  Enqueues on the stream and returns; nothing is synchronised."""
    for t, name in ((x, "x"), (bitmap, "bitmap"), (values, "values"), (nnz, "nnz"), (workspace, "workspace")):
        _dev(t, name)
    if values.dtype != x.dtype:
        raise TypeError("values must have the dtype of x")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(x.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    if nnz.element_size() != 8 or nnz.numel() < 1:
        raise ValueError("nnz must be one 64-bit integer")
    _check("bt_compress", lib().bt_compress(
        _ptr(x), x.numel(), dtype_code(x.dtype), _ptr(bitmap), _ptr(values), values.numel(), _ptr(nnz),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def bt_compress_static(x, bitmap, values, nnz, stream=None):
    """bt_compress on the library's own workspace (nothing is allocated by the call); x of at
    most BT_STATIC_MAX_TILES tiles.  Calls on one GPU share that workspace: keep them ordered."""
    for t, name in ((x, "x"), (bitmap, "bitmap"), (values, "values"), (nnz, "nnz")):
        _dev(t, name)
    if values.dtype != x.dtype:
        raise TypeError("values must have the dtype of x")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(x.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    if nnz.element_size() != 8 or nnz.numel() < 1:
        raise ValueError("nnz must be one 64-bit integer")
    _check("bt_compress_static", lib().bt_compress_static(
        _ptr(x), x.numel(), dtype_code(x.dtype), _ptr(bitmap), _ptr(values), values.numel(), _ptr(nnz), _stream(stream)))


def bt_compress_pruned(x, threshold, bitmap, values, nnz, workspace, stream=None):
    """Section 4.3 fused into Algorithm 1: keep x[i] where x[i] > threshold (ReLU for
    threshold 0 on a pre-activation tensor).  Same buffers as bt_compress."""
    for t, name in ((x, "x"), (bitmap, "bitmap"), (values, "values"), (nnz, "nnz"), (workspace, "workspace")):
        _dev(t, name)
    if values.dtype != x.dtype:
        raise TypeError("values must have the dtype of x")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(x.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    if nnz.element_size() != 8 or nnz.numel() < 1:
        raise ValueError("nnz must be one 64-bit integer")
    _check("bt_compress_pruned", lib().bt_compress_pruned(
        _ptr(x), x.numel(), dtype_code(x.dtype), ctypes.c_double(threshold), _ptr(bitmap), _ptr(values), values.numel(),
        _ptr(nnz), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def bt_decompress(bitmap, values, out, workspace, stream=None):
    """Algorithm 2 on device tensors: fills `out` (n = out.numel()) from bitmap + values."""
    for t, name in ((bitmap, "bitmap"), (values, "values"), (out, "out"), (workspace, "workspace")):
        _dev(t, name)
    if values.dtype != out.dtype:
        raise TypeError("values must have the dtype of out")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(out.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    _check("bt_decompress", lib().bt_decompress(
        _ptr(bitmap), _ptr(values), out.numel(), dtype_code(out.dtype), _ptr(out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def bt_relu_backward_from_bitmap(bitmap, grad_out, grad_in, stream=None):
    """grad_in[i] = bit(i) ? grad_out[i] : +0; grad_in may be grad_out itself."""
    for t, name in ((bitmap, "bitmap"), (grad_out, "grad_out"), (grad_in, "grad_in")):
        _dev(t, name)
    if grad_in.dtype != grad_out.dtype or grad_in.numel() != grad_out.numel():
        raise TypeError("grad_in must match grad_out")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(grad_out.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    _check("bt_relu_backward_from_bitmap", lib().bt_relu_backward_from_bitmap(
        _ptr(bitmap), _ptr(grad_out), grad_out.numel(), dtype_code(grad_out.dtype), _ptr(grad_in), _stream(stream)))


def bt_batch_workspace_bytes(ns, dtype):
    ns = list(ns)
    arr = (ctypes.c_uint64 * max(len(ns), 1))(*ns)
    return int(lib().bt_batch_workspace_bytes(arr, len(ns), dtype if isinstance(dtype, int) else dtype_code(dtype)))


def new_batch_workspace(ns, dtype, device="cuda", stream=None):
    """Allocate and initialise a workspace for batched calls on tensors of these sizes."""
    ws = torch.empty(bt_batch_workspace_bytes(ns, dtype), dtype=torch.uint8, device=device)
    bt_workspace_init(ws, stream)
    return ws


def _bytes(t):
    return t.numel() * t.element_size()


def compress_items(xs, bitmaps, values, nnz, indexes=None, dense_outs=None):
    """The host item array of the batched compressions for lists of device tensors; nnz is one
    int64 tensor with an entry per tensor; indexes (optional): an int64 tensor of
    bt_index_bytes(n) / 8 entries per tensor, to receive its tile index; dense_outs (optional,
    bt_compress_batch_pruned): a tensor like x per tensor (may be x itself) for the dense pruned
    result.  Build it once and reuse it while the buffers live."""
    if not (len(xs) == len(bitmaps) == len(values)) or nnz.numel() < len(xs) or nnz.element_size() != 8:
        raise ValueError("one bitmap, one value buffer and one 64-bit nnz entry per tensor")
    for extra, name in ((indexes, "indexes"), (dense_outs, "dense_outs")):
        if extra is not None and len(extra) != len(xs):
            raise ValueError("%s: one per tensor" % name)
    _dev(nnz, "nnz")
    items = (CompressItem * max(len(xs), 1))()
    for i, (x, b, v) in enumerate(zip(xs, bitmaps, values)):
        for t, name in ((x, "x"), (b, "bitmap"), (v, "values")):
            _dev(t, name)
        if v.dtype != x.dtype or x.dtype != xs[0].dtype:
            raise TypeError("all tensors and value buffers of a batch share one dtype")
        if b.element_size() != 4 or _bytes(b) < bt_bitmap_bytes(x.numel()):
            raise ValueError("bitmap %d must hold ceil(n/32) 32-bit words" % i)
        index = dense = None
        if indexes is not None and x.numel() != 0:
            _dev(indexes[i], "index")
            if indexes[i].element_size() != 8 or _bytes(indexes[i]) < bt_index_bytes(x.numel(), x.dtype):
                raise ValueError("index %d must hold bt_index_bytes(n, dtype) bytes of 64-bit entries" % i)
            index = indexes[i].data_ptr()
        if dense_outs is not None and x.numel() != 0:
            _dev(dense_outs[i], "dense_out")
            if dense_outs[i].dtype != x.dtype or dense_outs[i].numel() != x.numel():
                raise TypeError("dense_out %d must match x" % i)
            dense = dense_outs[i].data_ptr()
        items[i] = CompressItem(x.data_ptr(), x.numel(), b.data_ptr(), v.data_ptr(), v.numel(),
                                nnz.data_ptr() + 8 * i, index, dense)
    return items


def decompress_items(bitmaps, values, outs, indexes=None):
    """The host item array of the batched restorations for lists of device tensors; indexes: the
    tile indexes, for bt_decompress_batch_indexed."""
    if not (len(outs) == len(bitmaps) == len(values)) or (indexes is not None and len(indexes) != len(outs)):
        raise ValueError("one bitmap and one value buffer (and one index) per tensor")
    items = (DecompressItem * max(len(outs), 1))()
    for i, (b, v, o) in enumerate(zip(bitmaps, values, outs)):
        for t, name in ((b, "bitmap"), (v, "values"), (o, "out")):
            _dev(t, name)
        if v.dtype != o.dtype or o.dtype != outs[0].dtype:
            raise TypeError("all tensors and value buffers of a batch share one dtype")
        if b.element_size() != 4 or _bytes(b) < bt_bitmap_bytes(o.numel()):
            raise ValueError("bitmap %d must hold ceil(n/32) 32-bit words" % i)
        index = None
        if indexes is not None and o.numel() != 0:
            _dev(indexes[i], "index")
            if indexes[i].element_size() != 8 or _bytes(indexes[i]) < bt_index_bytes(o.numel(), o.dtype):
                raise ValueError("index %d must hold bt_index_bytes(n, dtype) bytes of 64-bit entries" % i)
            index = indexes[i].data_ptr()
        items[i] = DecompressItem(b.data_ptr(), v.data_ptr(), o.numel(), o.data_ptr(), v.numel(), index)
    return items


def bt_compress_batch(items, count, dtype, workspace, stream=None):
    """Algorithm 1 on every tensor of `items` (from compress_items) in one launch per 64 tensors."""
    _dev(workspace, "workspace")
    _check("bt_compress_batch", lib().bt_compress_batch(
        items, count, dtype if isinstance(dtype, int) else dtype_code(dtype), _ptr(workspace), _bytes(workspace),
        _stream(stream)))


def bt_compress_batch_pruned(items, count, dtype, threshold, workspace, stream=None):
    """bt_compress_pruned (bt_activation_compress where the items carry dense outputs) on every
    tensor of `items`, one threshold for all."""
    _dev(workspace, "workspace")
    _check("bt_compress_batch_pruned", lib().bt_compress_batch_pruned(
        items, count, dtype if isinstance(dtype, int) else dtype_code(dtype), ctypes.c_double(threshold), _ptr(workspace),
        _bytes(workspace), _stream(stream)))


def bt_decompress_batch_indexed(items, count, dtype, stream=None):
    """bt_decompress_indexed on every tensor of `items` (from decompress_items with indexes)."""
    _check("bt_decompress_batch_indexed", lib().bt_decompress_batch_indexed(
        items, count, dtype if isinstance(dtype, int) else dtype_code(dtype), _stream(stream)))


def bt_workspace_status(workspace, status, stream=None):
    """status (int32[2] on the device): [0] = 1 if a call gave up a wait on this workspace, [1] = calls completed."""
    _dev(workspace, "workspace")
    _dev(status, "status")
    if status.element_size() != 4 or status.numel() < 2:
        raise ValueError("status must be two 32-bit integers")
    _check("bt_workspace_status", lib().bt_workspace_status(_ptr(workspace), _ptr(status), _stream(stream)))


def bt_decompress_batch(items, count, dtype, workspace, stream=None):
    """Algorithm 2 on every tensor of `items` (from decompress_items)."""
    _dev(workspace, "workspace")
    _check("bt_decompress_batch", lib().bt_decompress_batch(
        items, count, dtype if isinstance(dtype, int) else dtype_code(dtype), _ptr(workspace), _bytes(workspace),
        _stream(stream)))


def bt_mask_apply(bitmap, x, out, stream=None):
    """Double mask: out[i] = bit(i) ? x[i] : +0 with the bitmap of another tensor; out may be x."""
    for t, name in ((bitmap, "bitmap"), (x, "x"), (out, "out")):
        _dev(t, name)
    if out.dtype != x.dtype or out.numel() != x.numel():
        raise TypeError("out must match x")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(x.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    _check("bt_mask_apply", lib().bt_mask_apply(_ptr(bitmap), _ptr(x), x.numel(), dtype_code(x.dtype), _ptr(out),
                                                _stream(stream)))


def bt_tile_elems(dtype):
    return int(lib().bt_tile_elems(_code(dtype)))


def bt_index_bytes(n, dtype):
    return int(lib().bt_index_bytes(n, _code(dtype)))


def bt_compress_indexed(x, bitmap, values, nnz, index, workspace, stream=None):
    """bt_compress that also leaves the tile index (int64[ceil(n / bt_tile_elems)]) for bt_decompress_indexed."""
    for t, name in ((x, "x"), (bitmap, "bitmap"), (values, "values"), (nnz, "nnz"), (index, "index"),
                    (workspace, "workspace")):
        _dev(t, name)
    if values.dtype != x.dtype:
        raise TypeError("values must have the dtype of x")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(x.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    if nnz.element_size() != 8 or nnz.numel() < 1:
        raise ValueError("nnz must be one 64-bit integer")
    if index.element_size() != 8 or index.numel() * 8 < bt_index_bytes(x.numel(), x.dtype):
        raise ValueError("index must hold one 64-bit integer per tile")
    _check("bt_compress_indexed", lib().bt_compress_indexed(
        _ptr(x), x.numel(), dtype_code(x.dtype), _ptr(bitmap), _ptr(values), values.numel(), _ptr(nnz), _ptr(index),
        _ptr(workspace), _bytes(workspace), _stream(stream)))


def bt_decompress_indexed(bitmap, values, index, out, stream=None):
    """Algorithm 2 started at every tile from the tile index: no workspace, no scan."""
    for t, name in ((bitmap, "bitmap"), (values, "values"), (index, "index"), (out, "out")):
        _dev(t, name)
    if values.dtype != out.dtype:
        raise TypeError("values must have the dtype of out")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(out.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    if index.element_size() != 8 or index.numel() * 8 < bt_index_bytes(out.numel(), out.dtype):
        raise ValueError("index must hold one 64-bit integer per tile")
    _check("bt_decompress_indexed", lib().bt_decompress_indexed(
        _ptr(bitmap), _ptr(values), values.numel(), _ptr(index), out.numel(), dtype_code(out.dtype), _ptr(out),
        _stream(stream)))


def bt_activation_compress(x, threshold, dense_out, bitmap, values, nnz, workspace, stream=None):
    """One pass over x: dense_out = x where x > threshold else +0 (ReLU for threshold 0; dense_out may be x
    itself), and bitmap / values / nnz = the compressed form of that dense_out."""
    for t, name in ((x, "x"), (dense_out, "dense_out"), (bitmap, "bitmap"), (values, "values"), (nnz, "nnz"),
                    (workspace, "workspace")):
        _dev(t, name)
    if values.dtype != x.dtype or dense_out.dtype != x.dtype or dense_out.numel() != x.numel():
        raise TypeError("values and dense_out must match x")
    if bitmap.element_size() != 4 or bitmap.numel() * 4 < bt_bitmap_bytes(x.numel()):
        raise ValueError("bitmap must hold ceil(n/32) 32-bit words")
    if nnz.element_size() != 8 or nnz.numel() < 1:
        raise ValueError("nnz must be one 64-bit integer")
    _check("bt_activation_compress", lib().bt_activation_compress(
        _ptr(x), x.numel(), dtype_code(x.dtype), ctypes.c_double(threshold), _ptr(dense_out), _ptr(bitmap), _ptr(values),
        values.numel(), _ptr(nnz), _ptr(workspace), _bytes(workspace), _stream(stream)))
