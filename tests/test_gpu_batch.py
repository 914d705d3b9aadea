"""GPU parity of the batched calls (many tensors per launch) against the CPU oracle,
byte for byte and tensor by tensor: a batched call must give for every tensor exactly
what Algorithm 1 / Algorithm 2 give for it alone."""
import numpy as np
import pytest
import torch

from paper_2110_15362_amd import workloads as wl

pytestmark = pytest.mark.gpu

SENT = 0x5A
TILE = {4: 8192, 2: 16384, 8: 4096}


@pytest.fixture(scope="module")
def bt():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (they never fall back to the CPU)")
    import paper_2110_15362_amd.bittrain as b
    b.lib()
    return b


def _sentinel(numel, dtype):
    t = torch.empty(numel, dtype=dtype, device="cuda")
    t.view(torch.uint8).fill_(SENT)
    return t


def _sent_of(a):
    return np.frombuffer(bytes([SENT] * a.itemsize), dtype=a.dtype)[0]


def _compress_batch(bt, xs, ws, caps=None):
    """Runs bt_compress_batch on CPU tensors xs; returns per tensor (bitmap, values, nnz) and
    asserts that nothing outside bitmap[0,W) / values[0,min(nnz,cap)) was written."""
    dt = xs[0].dtype
    caps = [x.numel() for x in xs] if caps is None else caps
    xd = [x.cuda() for x in xs]
    bms = [_sentinel((x.numel() + 31) // 32 + 4, torch.int32) for x in xs]
    vbs = [_sentinel(c + 8, dt) for c in caps]
    nnz = torch.full((len(xs) + 1,), -7, dtype=torch.int64, device="cuda")
    items = bt.compress_items(xd, [b[:(x.numel() + 31) // 32] for b, x in zip(bms, xs)],
                              [v[:c] for v, c in zip(vbs, caps)], nnz)
    bt.bt_compress_batch(items, len(xs), dt, ws)
    torch.cuda.synchronize()
    nnz_h = nnz.cpu().numpy()
    assert nnz_h[len(xs)] == -7
    res = []
    for x, b, v, c, k in zip(xs, bms, vbs, caps, nnz_h):
        words = (x.numel() + 31) // 32
        bm = b.cpu().numpy().view(np.uint32)
        vb = wl.bits(v.cpu())
        assert (bm[words:] == 0x5A5A5A5A).all(), "wrote past the bitmap"
        assert (vb[min(int(k), c):] == _sent_of(vb)).all(), "wrote past values[min(nnz, cap))"
        res.append((bm[:words].copy(), vb[:c].copy(), int(k)))
    return res


def _decompress_batch(bt, comp, ns, dt, ws):
    """comp: per tensor (bitmap uint32, values bits); returns the restored bits per tensor."""
    pad = 16 // torch.empty(0, dtype=dt).element_size()
    bms = [torch.from_numpy(b.view(np.int32).copy()).cuda() for b, _ in comp]
    vals = [torch.from_numpy(v.view({2: np.int16, 4: np.int32, 8: np.int64}[v.itemsize]).copy()).view(dt).cuda() for _, v in comp]
    obufs = [_sentinel(n + pad, dt) for n in ns]
    items = bt.decompress_items(bms, vals, [o[:n] for o, n in zip(obufs, ns)])
    bt.bt_decompress_batch(items, len(ns), dt, ws)
    torch.cuda.synchronize()
    outs = []
    for o, n in zip(obufs, ns):
        ob = wl.bits(o.cpu())
        assert (ob[n:] == _sent_of(ob)).all(), "wrote past out[n)"
        outs.append(ob[:n].copy())
    return outs


def _check_batch(bt, oracle, xs, ws=None):
    dt = xs[0].dtype
    ns = [x.numel() for x in xs]
    if ws is None:
        ws = bt.new_batch_workspace(ns, dt)
    got = _compress_batch(bt, xs, ws)
    want = []
    for i, (x, (bitmap, values, nnz)) in enumerate(zip(xs, got)):
        o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
        assert nnz == o_nnz, i
        assert np.array_equal(bitmap, o_bitmap), i
        assert np.array_equal(values[:o_nnz], o_values), i
        want.append((o_bitmap, o_values))
    outs = _decompress_batch(bt, want, ns, dt, ws)
    for i, (x, out, (o_bitmap, o_values)) in enumerate(zip(xs, outs, want)):
        assert np.array_equal(out, oracle.decompress(o_bitmap, o_values, x.numel())), i
        assert np.array_equal(out, wl.bits(x)), i
    return ws


def _mixed_sizes(width):
    t = TILE[width]
    # empty, tiny, around one tile, exactly one scanner row of tiles and one more, a ragged large one
    return [0, 1, 33, t - 1, t, t + 1, 3 * t + 17, 64 * t, 0, 64 * t + 1, 65 * t - 5, 130 * t + 1234, 7]


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16", "f64"])
def test_batch_mixed_sizes(bt, oracle, dt):
    width = {"f32": 4, "f16": 2, "bf16": 2, "f64": 8}[dt]
    xs = [wl.random_sparse(n, dt, 0.1 + 0.07 * (k % 12), 300 + k) for k, n in enumerate(_mixed_sizes(width))]
    _check_batch(bt, oracle, xs)


def test_batch_special_bit_patterns_and_extremes(bt, oracle):
    t = TILE[4]
    xs = [wl.special_values("f32"), torch.zeros(2 * t + 5), torch.ones(t + 3), wl.special_values("f32").repeat(700),
          torch.zeros(1), torch.ones(1)]
    _check_batch(bt, oracle, xs)


def test_batch_of_more_tensors_than_one_launch_takes(bt, oracle):
    """150 tensors: three launches that reuse the workspace back to back."""
    xs = [wl.random_sparse(1 + (k * 7919) % 40000, "f32", 0.5, 1000 + k) for k in range(150)]
    _check_batch(bt, oracle, xs)


def test_batch_and_single_calls_share_a_workspace(bt, oracle):
    """Large batch, small single call, small batch, large single call, large batch: each call
    cleans up what the one before it left, whatever their sizes."""
    from tests import gpu_util
    t = TILE[4]
    big = [wl.random_sparse(n, "f32", 0.5, 40 + k) for k, n in enumerate([70 * t + 3, 5, 200 * t, t])]
    small = [wl.random_sparse(n, "f32", 0.7, 50 + k) for k, n in enumerate([100, 2 * t])]
    n_single = 300 * t + 11
    ws_bytes = max(bt.bt_batch_workspace_bytes([x.numel() for x in big], torch.float32),
                   bt.bt_workspace_bytes(n_single, torch.float32))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    bt.bt_workspace_init(ws)
    xs_small = wl.random_sparse(1000, "f32", 0.3, 60)
    xs_large = wl.random_sparse(n_single, "f32", 0.6, 61)
    for _ in range(2):
        _check_batch(bt, oracle, big, ws)
        bitmap, values, nnz, ok = gpu_util.gpu_compress(xs_small, ws=ws)
        o = oracle.compress(wl.bits(xs_small))
        assert ok and nnz == o[2] and np.array_equal(bitmap, o[0]) and np.array_equal(values[:nnz], o[1])
        _check_batch(bt, oracle, small, ws)
        bitmap, values, nnz, ok = gpu_util.gpu_compress(xs_large, ws=ws)
        o = oracle.compress(wl.bits(xs_large))
        assert ok and nnz == o[2] and np.array_equal(bitmap, o[0]) and np.array_equal(values[:nnz], o[1])
        out, ok = gpu_util.gpu_decompress(o[0], o[1], n_single, torch.float32, ws=ws)
        assert ok and np.array_equal(out, wl.bits(xs_large))
    hdr = ws[:12].cpu().numpy().view(np.uint32)
    assert hdr[2] == 0, "a bounded wait ran out"


def test_batch_capacity_of_one_tensor_does_not_touch_the_others(bt, oracle):
    t = TILE[4]
    xs = [wl.random_sparse(n, "f32", 0.5, 70 + k) for k, n in enumerate([3 * t, 2 * t + 9, t])]
    want = [oracle.compress(wl.bits(x)) for x in xs]
    caps = [xs[0].numel(), want[1][2] // 2, 0]
    ws = bt.new_batch_workspace([x.numel() for x in xs], torch.float32)
    got = _compress_batch(bt, xs, ws, caps)
    for (bitmap, values, nnz), (o_bitmap, o_values, o_nnz), cap in zip(got, want, caps):
        assert nnz == o_nnz and np.array_equal(bitmap, o_bitmap)
        w = min(o_nnz, cap)
        assert np.array_equal(values[:w], o_values[:w])


def test_batch_empty_list_and_host_errors(bt):
    ws = bt.new_batch_workspace([], torch.float32)
    assert ws.numel() == bt.bt_workspace_bytes(0, torch.float32)
    bt.bt_compress_batch(bt.compress_items([], [], [], torch.zeros(1, dtype=torch.int64, device="cuda")), 0,
                         torch.float32, ws)
    bt.bt_decompress_batch(bt.decompress_items([], [], []), 0, torch.float32, ws)
    x = torch.ones(100000, device="cuda")
    bitmap = torch.zeros(3125, dtype=torch.int32, device="cuda")
    values = torch.zeros(100000, device="cuda")
    nnz = torch.zeros(1, dtype=torch.int64, device="cuda")
    items = bt.compress_items([x], [bitmap], [values], nnz)
    with pytest.raises(bt.BitTrainError) as e:
        bt.bt_compress_batch(items, 1, torch.float32, ws[:512])
    assert e.value.status == 4
    items[0].d_in += 4
    with pytest.raises(bt.BitTrainError) as e:
        bt.bt_compress_batch(items, 1, torch.float32, bt.new_batch_workspace([100000], torch.float32))
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert int(nnz.item()) == 0 and int(bitmap.abs().sum().item()) == 0    # nothing was launched


def test_batch_config4_resnet50_set_full_size(bt, oracle):
    """The 49 activations of the ResNet-50 set in one compress launch and one restore launch."""
    dt = torch.float32
    shapes = wl.config4_shapes()
    ns = [int(np.prod(s)) for s in shapes]
    ws = bt.new_batch_workspace(ns, dt)
    xd, bms, vals = [], [], []
    want_nnz = []
    for cfg in wl.config4_tensors():
        x = cfg["x"].reshape(-1)
        xd.append(x.cuda())
        bms.append(torch.empty((x.numel() + 31) // 32, dtype=torch.int32, device="cuda"))
        want_nnz.append(int((x != 0).sum()))
        vals.append(torch.empty(want_nnz[-1], dtype=dt, device="cuda"))          # right-sized
    nnz = torch.zeros(len(ns), dtype=torch.int64, device="cuda")
    bt.bt_compress_batch(bt.compress_items(xd, bms, vals, nnz), len(ns), dt, ws)
    torch.cuda.synchronize()
    assert nnz.cpu().tolist() == want_nnz
    outs = [torch.empty(n, dtype=dt, device="cuda") for n in ns]
    bt.bt_decompress_batch(bt.decompress_items(bms, vals, outs), len(ns), dt, ws)
    torch.cuda.synchronize()
    for k, (x, b, v, o) in enumerate(zip(xd, bms, vals, outs)):
        xb = wl.bits(x.cpu())
        o_bitmap, o_values, o_nnz = oracle.compress(xb)
        assert o_nnz == want_nnz[k]
        assert np.array_equal(b.cpu().numpy().view(np.uint32), o_bitmap), k
        assert np.array_equal(wl.bits(v.cpu()), o_values), k
        assert np.array_equal(wl.bits(o.cpu()), xb), k


# ---- the pruning batch, the dense outputs, the tile indexes --------------------------------------

_ORACLE_DT = {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16", torch.float64: "f64"}


def _pruned_batch_against_oracle(bt, oracle, xs, thr, dense, in_place=False):
    """bt_compress_batch_pruned (with dense outputs and tile indexes) on CPU tensors xs, every output against
    the oracle's pruning followed by Algorithm 1, then bt_decompress_batch_indexed of the result."""
    dt = xs[0].dtype
    ns = [x.numel() for x in xs]
    ws = bt.new_batch_workspace(ns, dt)
    xd = [x.clone().cuda() for x in xs]
    bms = [torch.empty((n + 31) // 32, dtype=torch.int32, device="cuda") for n in ns]
    vals = [_sentinel(n + 8, dt) for n in ns]
    idx = [torch.full((max(bt.bt_index_bytes(n, dt) // 8, 1) + 1,), -3, dtype=torch.int64, device="cuda") for n in ns]
    dense_outs = None
    if dense:
        dense_outs = xd if in_place else [_sentinel(n + 16 // x.element_size(), dt) for n, x in zip(ns, xs)]
    nnz = torch.full((len(xs),), -7, dtype=torch.int64, device="cuda")
    items = bt.compress_items(xd, bms, [v[:n] for v, n in zip(vals, ns)], nnz, indexes=[i[:-1] for i in idx],
                              dense_outs=None if not dense else [d[:n] for d, n in zip(dense_outs, ns)])
    bt.bt_compress_batch_pruned(items, len(xs), dt, thr, ws)
    torch.cuda.synchronize()
    tile = bt.bt_tile_elems(dt)
    pruned = []
    for k, x in enumerate(xs):
        want = oracle.prune(wl.bits(x), _ORACLE_DT[dt], thr)
        o_bitmap, o_values, o_nnz = oracle.compress(want)
        pruned.append(want)
        assert int(nnz[k].item()) == o_nnz, k
        assert np.array_equal(bms[k].cpu().numpy().view(np.uint32), o_bitmap), k
        vb = wl.bits(vals[k].cpu())
        assert np.array_equal(vb[:o_nnz], o_values), k
        assert (vb[o_nnz:] == _sent_of(vb)).all(), k
        tiles = bt.bt_index_bytes(ns[k], dt) // 8
        got_index = idx[k].cpu().numpy()
        assert np.array_equal(got_index[:tiles].view(np.uint64), oracle.tile_index(o_bitmap, ns[k], tile)), k
        assert (got_index[tiles:] == -3).all(), k
        if dense:
            db = wl.bits(dense_outs[k].cpu())
            assert np.array_equal(db[:ns[k]], want), k
            if not in_place:
                assert (db[ns[k]:] == _sent_of(db)).all(), k
    outs = [_sentinel(n + 16 // xs[0].element_size(), dt) for n in ns]
    ditems = bt.decompress_items(bms, [v[:max(int(k), 0)] for v, k in zip(vals, nnz.cpu().tolist())], [o[:n] for o, n in zip(outs, ns)],
                                 indexes=[i[:-1] for i in idx])
    bt.bt_decompress_batch_indexed(ditems, len(xs), dt)
    torch.cuda.synchronize()
    for k, n in enumerate(ns):
        ob = wl.bits(outs[k].cpu())
        assert np.array_equal(ob[:n], pruned[k]), k
        assert (ob[n:] == _sent_of(ob)).all(), k


@pytest.mark.gpu
@pytest.mark.parametrize("dt,thr", [(torch.float32, 0.0), (torch.float32, 0.1), (torch.float16, 0.1), (torch.bfloat16, 0.01),
                                    (torch.float64, 0.1), (torch.float32, -1.0)])
def test_pruned_batch_with_dense_outputs_and_tile_indexes(bt, oracle, dt, thr):
    width = torch.empty(0, dtype=dt).element_size()
    xs = []
    for k, n in enumerate(_mixed_sizes(width)):
        g = torch.Generator().manual_seed(100 + k)
        x = torch.randn(n, generator=g, dtype=torch.float64) * 0.3
        x[torch.rand(n, generator=g) < 0.3] = 0
        xs.append(x.to(dt))
    # values on both sides of the threshold's nearest narrower numbers
    edge = torch.tensor([thr, np.nextafter(thr, 1.0), np.nextafter(thr, -1.0), float(np.float32(thr)), float(np.float16(thr)), 0.0, -0.0],
                        dtype=torch.float64).repeat(300).to(dt)
    xs.append(edge)
    _pruned_batch_against_oracle(bt, oracle, xs, thr, dense=True)
    _pruned_batch_against_oracle(bt, oracle, xs[:5], thr, dense=True, in_place=True)
    _pruned_batch_against_oracle(bt, oracle, xs, thr, dense=False)


@pytest.mark.gpu
def test_pruned_single_calls_take_a_double_threshold(bt, oracle):
    """bt_compress_pruned / bt_activation_compress on doubles and singles around a threshold that is no single."""
    thr = 0.1
    for dt in (torch.float64, torch.float32):
        base = torch.tensor([thr, np.nextafter(thr, 1.0), np.nextafter(thr, -1.0), float(np.float32(thr)),
                             float(np.nextafter(np.float32(thr), np.float32(0))), 0.25, -0.25, 0.0], dtype=torch.float64)
        x = base.repeat(5000).to(dt)
        n = x.numel()
        ws = bt.new_workspace(n, dt)
        bm = torch.empty((n + 31) // 32, dtype=torch.int32, device="cuda")
        vals, dense = torch.empty(n, dtype=dt, device="cuda"), torch.empty(n, dtype=dt, device="cuda")
        nnz = torch.zeros(1, dtype=torch.int64, device="cuda")
        want = oracle.prune(wl.bits(x), _ORACLE_DT[dt], thr)
        o_bitmap, o_values, o_nnz = oracle.compress(want)
        for call in ("pruned", "activation"):
            nnz.fill_(-1)
            if call == "pruned":
                bt.bt_compress_pruned(x.cuda(), thr, bm, vals, nnz, ws)
            else:
                bt.bt_activation_compress(x.cuda(), thr, dense, bm, vals, nnz, ws)
            torch.cuda.synchronize()
            assert int(nnz.item()) == o_nnz
            assert np.array_equal(bm.cpu().numpy().view(np.uint32), o_bitmap)
            assert np.array_equal(wl.bits(vals.cpu())[:o_nnz], o_values)
        assert np.array_equal(wl.bits(dense.cpu()), want)


@pytest.mark.gpu
def test_config4_full_size_pruned_activation_batch_and_indexed_restore(bt, oracle):
    """The 49 activations of the ResNet-50 set at full size: one pruning launch that also writes the dense pruned
    tensors (in place) and the tile indexes, one restoration launch from the indexes; all against the oracle."""
    xs = [cfg["x"].reshape(-1) for cfg in wl.config4_tensors()]
    _pruned_batch_against_oracle(bt, oracle, xs, 0.05, dense=True, in_place=True)


@pytest.mark.gpu
def test_workspace_status_reports_a_given_up_wait(bt):
    n = 50 * TILE[4] + 17
    x = wl.random_sparse(n, torch.float32, 0.5, 9).cuda()
    ws = bt.new_workspace(n, torch.float32)
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    bm = torch.empty((n + 31) // 32, dtype=torch.int32, device="cuda")
    vals, nnz = torch.empty(n, dtype=torch.float32, device="cuda"), torch.zeros(1, dtype=torch.int64, device="cuda")
    bt.bt_workspace_status(ws, status)
    assert status.cpu().tolist() == [0, 0]
    bt.bt_compress(x, bm, vals, nnz, ws)
    bt.bt_decompress(bm, vals, torch.empty_like(x), ws)
    bt.bt_workspace_status(ws, status)
    assert status.cpu().tolist() == [0, 2]
    ws.view(torch.int32)[bt.BT_WS_ERROR_WORD] = 1          # what a kernel that gave up a wait leaves behind
    bt.bt_workspace_status(ws, status)
    assert status.cpu().tolist()[0] == 1
    bt.bt_workspace_init(ws)
    bt.bt_workspace_status(ws, status)
    assert status.cpu().tolist() == [0, 0]
