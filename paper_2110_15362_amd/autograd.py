"""BitTrain as PyTorch autograd plumbing (the integration the paper describes in its
implementation details and names as future work): activations saved for backward are
kept in the bitmap format between the forward and the backward pass.

Two pieces, both thin: every byte of codec work is done by libbittrain's kernels.

* ``BitmapStash`` -- a ``torch.autograd.graph.saved_tensors_hooks`` context.  Packing a
  saved activation runs ``bt_compress_indexed`` into a reusable worst-case scratch buffer, reads
  nnz and the workspace's status (one host synchronisation per tensor: the price of right-sizing) and keeps
  only ``values[:nnz]`` and the bitmap; if that is not smaller than the dense tensor the
  tensor is kept as it is.  Packing also keeps the tile index (8 bytes per 32 KiB of
  dense data) that compression produces on the way, so unpacking runs
  ``bt_decompress_indexed``, which needs no scan over the bitmap.  The round trip is
  bit-exact, so gradients are identical to those of the unhooked graph.
* ``bitmap_relu`` -- a ReLU whose backward is served by
  ``bt_relu_backward_from_bitmap`` and which saves nothing but the bitmap of its output
  (1/32 of an fp32 activation): compression with a value capacity of 0.
"""
import warnings

import torch

from . import bittrain as bt

_SUPPORTED = (torch.float32, torch.float16, torch.bfloat16, torch.float64)


class _StreamState:
    """Reusable buffers of one (device, stream): workspace, worst-case value scratch, and the words
    read back after a compression (nnz, then the workspace's status).  Work on different streams must
    not share them: a workspace serves one call at a time."""

    def __init__(self, device):
        self.device = device
        self.ws = None
        self.scratch = {}
        self.result = torch.zeros(2, dtype=torch.int64, device=device)      # [0]: nnz; [1]: two status words
        self.nnz = self.result[:1]
        self.status = self.result[1:].view(torch.int32)

    def workspace(self, n, dtype):
        need = bt.bt_workspace_bytes(n, dtype)
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(max(need, 1 << 16), dtype=torch.uint8, device=self.device)
            bt.bt_workspace_init(self.ws)
        return self.ws

    def value_scratch(self, n, dtype):
        buf = self.scratch.get(dtype)
        if buf is None or buf.numel() < n:
            buf = torch.empty(n, dtype=dtype, device=self.device)
            self.scratch[dtype] = buf
        return buf[:n]


_states = {}


def _state(device):
    key = (device, torch.cuda.current_stream(device).cuda_stream)
    st = _states.get(key)
    if st is None:
        st = _states[key] = _StreamState(device)
    return st


class _Packed:
    """A saved activation in the bitmap format.  `dense` is set instead when the tensor turned out not to be
    worth compressing (or its compression failed); `pending` while that is not known yet (deferred mode)."""
    __slots__ = ("bitmap", "values", "index", "shape", "dtype", "device", "dense", "pending")

    def __init__(self, bitmap, values, index, shape, dtype, device):
        self.bitmap, self.values, self.index = bitmap, values, index
        self.shape, self.dtype, self.device = shape, dtype, device
        self.dense, self.pending = None, None


class _Pending:
    """What a deferred packing still waits for: nnz and the workspace's status on their way to pinned host
    memory, the event behind that copy, and the dense tensor, kept until the result is known to be good."""
    __slots__ = ("packed", "dense", "host", "event", "ws")

    def __init__(self, packed, dense, host, event, ws):
        self.packed, self.dense, self.host, self.event, self.ws = packed, dense, host, event, ws


class BitmapStash(torch.autograd.graph.saved_tensors_hooks):
    """``with BitmapStash(): loss = model(x)`` keeps saved activations compressed.

    min_numel: smaller tensors are left alone (a call costs a few microseconds).
    deferred: False (default) reads nnz back right after the compression, which makes the host wait for the
    device once per saved tensor, and stores exactly nnz values at once.  True never waits: the compression
    writes into a buffer of worst-case size, nnz and the status travel to pinned memory behind an event, and
    the buffer is cut down to nnz values (and the dense tensor let go) at the next packing or unpacking after
    the event has passed; until then the tensor costs more memory than it did dense, so at most
    `max_waiting` packings are left in that state (the host waits for the oldest one beyond that).
    ``stats`` counts dense and stored bytes of everything that went through the hooks.
    """

    def __init__(self, min_numel=4096, deferred=False, max_waiting=2):
        self.min_numel = min_numel
        self.deferred = deferred
        self.max_waiting = max(1, max_waiting)
        self.stats = {"tensors": 0, "compressed": 0, "failed": 0, "dense_bytes": 0, "stored_bytes": 0}
        self._waiting = []
        super().__init__(self._pack, self._unpack)

    def _settle(self, p, nnz, gave_up, values_full):
        """The compression of `p` (a _Packed) is over: keep it, cut to size, or go back to the dense tensor."""
        n = 1
        for d in p.shape:
            n *= d
        width = torch.empty(0, dtype=p.dtype).element_size()
        if gave_up:
            self.stats["failed"] += 1
            warnings.warn("BitmapStash: a compression gave up a wait; the tensor is kept dense")
        stored = bt.bt_compressed_size(n, nnz, p.dtype) + 8 * p.index.numel()      # M_b plus the tile index
        if gave_up or stored >= n * width:
            self.stats["stored_bytes"] += n * width
            return False                                           # too dense (the bitmap form would be larger), or no good
        self.stats["compressed"] += 1
        self.stats["stored_bytes"] += stored
        p.values = values_full[:nnz].clone()
        return True

    def _finish_waiting(self, only=None, block=False):
        """Deferred mode: settle every packing whose result has arrived; wait for `only`'s (for all, if `block`)."""
        still = []
        for w in self._waiting:
            if not (block or w.packed is only or w.event.query()):
                still.append(w)
                continue
            w.event.synchronize()
            nnz, gave_up = int(w.host[0]), int(w.host[1:].view(torch.int32)[0])
            if gave_up:
                bt.bt_workspace_init(w.ws)                         # what the kernel wrote is not valid; make the workspace usable again
            if not self._settle(w.packed, nnz, gave_up, w.packed.values):
                w.packed.dense, w.packed.bitmap, w.packed.values, w.packed.index = w.dense, None, None, None
            w.packed.pending = None
        self._waiting = still

    def __exit__(self, *exc):
        self._finish_waiting(block=True)      # leaves nothing behind that still holds a dense tensor
        return super().__exit__(*exc)

    def _pack(self, t):
        if (not t.is_cuda or t.dtype not in _SUPPORTED or t.numel() < self.min_numel or not t.is_contiguous()
                or isinstance(t, torch.nn.Parameter) or t.data_ptr() % 16 != 0):
            return t                      # (a view that starts off a 16-byte boundary is not what the library takes)
        st = _state(t.device)
        n = t.numel()
        self.stats["tensors"] += 1
        self.stats["dense_bytes"] += n * t.element_size()
        bitmap = torch.empty(bt.bt_bitmap_bytes(n) // 4, dtype=torch.int32, device=t.device)
        index = torch.empty(bt.bt_index_bytes(n, t.dtype) // 8, dtype=torch.int64, device=t.device)
        ws = st.workspace(n, t.dtype)
        if self.deferred:
            self._finish_waiting()
            while len(self._waiting) >= self.max_waiting:          # bounds what the unsettled packings hold
                self._finish_waiting(only=self._waiting[0].packed)
            values_full = torch.empty(n, dtype=t.dtype, device=t.device)       # its own: it outlives this call
            result = torch.empty(2, dtype=torch.int64, device=t.device)
            bt.bt_compress_indexed(t.detach(), bitmap, values_full, result[:1], index, ws)
            bt.bt_workspace_status(ws, result[1:].view(torch.int32))
            host = torch.empty(2, dtype=torch.int64, pin_memory=True)
            host.copy_(result, non_blocking=True)
            event = torch.cuda.Event()
            event.record(torch.cuda.current_stream(t.device))
            packed = _Packed(bitmap, values_full, index, t.shape, t.dtype, t.device)
            packed.pending = True
            self._waiting.append(_Pending(packed, t.detach(), host, event, ws))
            return packed
        scratch = st.value_scratch(n, t.dtype)
        bt.bt_compress_indexed(t.detach(), bitmap, scratch, st.nnz, index, ws)
        bt.bt_workspace_status(ws, st.status)
        result = st.result.cpu()                                   # host sync: nnz is needed to right-size
        nnz, gave_up = int(result[0]), int(result[1:].view(torch.int32)[0])
        if gave_up:
            bt.bt_workspace_init(ws)                               # what the kernel wrote is not valid; make the workspace usable again
        packed = _Packed(bitmap, None, index, t.shape, t.dtype, t.device)
        return packed if self._settle(packed, nnz, gave_up, scratch) else t

    def _unpack(self, obj):
        if not isinstance(obj, _Packed):
            return obj
        if obj.pending:
            self._finish_waiting(only=obj)
        if obj.dense is not None:
            return obj.dense
        out = torch.empty(obj.shape, dtype=obj.dtype, device=obj.device)
        bt.bt_decompress_indexed(obj.bitmap, obj.values, obj.index, out)
        return out


class _BitmapReLU(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, fused):
        if not (x.is_cuda and x.dtype in _SUPPORTED and x.is_contiguous()):
            raise TypeError("bitmap_relu needs a contiguous float64/float32/float16/bfloat16 device tensor")
        st = _state(x.device)
        n = x.numel()
        bitmap = torch.empty(bt.bt_bitmap_bytes(n) // 4, dtype=torch.int32, device=x.device)
        empty = torch.empty(0, dtype=x.dtype, device=x.device)
        # capacity 0: only the bitmap (and nnz) are produced, no value is written
        if fused:
            # one pass: y = x where x > 0 else +0, and y's bitmap (a NaN input gives 0 here, NaN in torch.relu)
            y = torch.empty_like(x)
            bt.bt_activation_compress(x, 0.0, y, bitmap, empty, st.nnz, st.workspace(n, x.dtype))
        else:
            y = torch.relu(x)
            bt.bt_compress(y, bitmap, empty, st.nnz, st.workspace(n, y.dtype))
        ctx.bitmap = bitmap
        return y

    @staticmethod
    def backward(ctx, grad_out):
        grad_out = grad_out.contiguous()
        grad_in = torch.empty_like(grad_out)
        bt.bt_relu_backward_from_bitmap(ctx.bitmap, grad_out, grad_in)
        return grad_in, None


def bitmap_relu(x, fused=False):
    """ReLU that keeps only the 1-bit-per-element mask of its output for backward.  fused=True computes the
    output and the mask in one pass over x (bt_activation_compress) instead of torch.relu followed by a pass
    over its output; the two differ only for NaN inputs (0 instead of NaN)."""
    return _BitmapReLU.apply(x, fused)
