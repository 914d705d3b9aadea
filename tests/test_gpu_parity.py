"""GPU parity: libbittrain (through its C ABI) against the CPU oracle, byte for byte.

Integer / bit work throughout, so the bar is exact equality of the bitmap, the
value array [0, nnz), nnz, the restored tensor and the ReLU-backward output."""
import numpy as np
import pytest
import torch

from paper_2110_15362_amd import workloads as wl

pytestmark = pytest.mark.gpu

DTYPES = ["f32", "f16", "bf16", "f64"]
# tile = 8192 fp32 / 16384 16-bit / 4096 fp64 elements; wave strip = a quarter of it; row = 256 / 512 / 128
SIZES = [1, 3, 4, 5, 7, 8, 9, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 2049,
         4095, 4096, 4097, 8191, 8192, 8193, 12305, 16384, 3 * 8192 + 17, 100003, 5 * 8192, 1000000 + 37]


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (they never fall back to the CPU)")
    import paper_2110_15362_amd.bittrain as bt
    bt.lib()
    from tests import gpu_util
    return gpu_util


def _check_compress(gpu, oracle, x, **kw):
    xb = wl.bits(x)
    o_bitmap, o_values, o_nnz = oracle.compress(xb)
    bitmap, values, nnz, tail_ok = gpu.gpu_compress(x, **kw)
    assert nnz == o_nnz
    assert np.array_equal(bitmap, o_bitmap)
    cap = kw.get("cap")
    written = o_nnz if cap is None else min(o_nnz, cap)
    assert np.array_equal(values[:written], o_values[:written])
    assert tail_ok, "wrote outside bitmap[0,W) or values[0,min(nnz,cap))"
    return o_bitmap, o_values, o_nnz


def _check_decompress(gpu, oracle, o_bitmap, o_values, n, dtype, expect_bits, **kw):
    out, guard_ok = gpu.gpu_decompress(o_bitmap, o_values, n, dtype, **kw)
    assert np.array_equal(out, oracle.decompress(o_bitmap, o_values, n))
    assert np.array_equal(out, expect_bits)
    assert guard_ok, "wrote past out[n)"


@pytest.mark.parametrize("dt", DTYPES)
def test_compress_sizes_and_tails(gpu, oracle, dt):
    for i, n in enumerate(SIZES):
        for zf in (0.5, 0.0, 1.0, 0.93):
            x = wl.random_sparse(n, dt, zf, seed=1000 + i)
            _check_compress(gpu, oracle, x)


@pytest.mark.parametrize("dt", DTYPES)
def test_decompress_sizes_and_tails(gpu, oracle, dt):
    for i, n in enumerate(SIZES):
        for zf in (0.5, 0.0, 1.0, 0.93):
            x = wl.random_sparse(n, dt, zf, seed=2000 + i)
            xb = wl.bits(x)
            o_bitmap, o_values, _ = oracle.compress(xb)
            _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, xb)


@pytest.mark.parametrize("dt", DTYPES)
def test_relu_backward_sizes_and_tails(gpu, oracle, dt):
    for i, n in enumerate(SIZES):
        x = torch.relu(wl.random_sparse(n, dt, 0.2, seed=3000 + i))
        g = wl.random_sparse(n, dt, 0.0, seed=4000 + i)
        o_bitmap, _, _ = oracle.compress(wl.bits(x))
        expect = oracle.relu_backward(o_bitmap, wl.bits(g))
        for inplace in (False, True):
            out, guard_ok = gpu.gpu_relu_backward(o_bitmap, g, inplace=inplace)
            assert np.array_equal(out, expect)
            assert guard_ok


@pytest.mark.parametrize("dt", DTYPES)
def test_special_bit_patterns(gpu, oracle, dt):
    """-0.0, denormals, NaN payloads and infinities are values; the round trip is bit exact."""
    base = wl.special_values(dt)
    x = base.repeat(700)[:11111]
    o_bitmap, o_values, o_nnz = _check_compress(gpu, oracle, x)
    _check_decompress(gpu, oracle, o_bitmap, o_values, x.numel(), x.dtype, wl.bits(x))
    # ReLU backward is a select: NaN / Inf gradients under a cleared bit give +0
    g = base.flip(0).repeat(700)[:11111]
    out, guard_ok = gpu.gpu_relu_backward(o_bitmap, g)
    assert np.array_equal(out, oracle.relu_backward(o_bitmap, wl.bits(g))) and guard_ok


def test_single_nonzero_first_and_last(gpu, oracle):
    for n in (4096, 4097, 50000):
        for pos in (0, n - 1, n // 2):
            x = torch.zeros(n)
            x[pos] = -3.25
            o_bitmap, o_values, o_nnz = _check_compress(gpu, oracle, x)
            assert o_nnz == 1
            _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x))


def test_values_capacity_is_respected(gpu, oracle):
    """nnz > values_cap: nothing beyond the capacity is written, bitmap and nnz are complete."""
    x = wl.random_sparse(70001, "f32", 0.5, seed=5)
    for cap in (0, 1, 1000, 17000, 34999):
        _check_compress(gpu, oracle, x, cap=cap)
    xh = wl.random_sparse(70001, "f16", 0.3, seed=6)
    for cap in (0, 3, 8191, 30001):
        _check_compress(gpu, oracle, xh, cap=cap)


@pytest.mark.parametrize("dt", DTYPES)
def test_values_pointer_only_element_aligned(gpu, oracle, dt):
    for off in (1, 2, 3, 5, 7):
        x = wl.random_sparse(40000 + off, dt, 0.4, seed=70 + off)
        o_bitmap, o_values, _ = _check_compress(gpu, oracle, x, values_offset=off)
        _check_decompress(gpu, oracle, o_bitmap, o_values, x.numel(), x.dtype, wl.bits(x), values_offset=off)


def test_workspace_reuse_across_calls_and_sizes(gpu, oracle):
    """One workspace, initialised once, serves many calls of different sizes and kinds
    (the kernels leave it ready for the next call)."""
    import paper_2110_15362_amd.bittrain as bt
    ws = bt.new_workspace(300000, torch.float32)
    for rep, n in enumerate([300000, 17, 4096, 250001, 8192, 1, 300000, 123457]):
        x = wl.random_sparse(n, "f32", 0.6, seed=900 + rep)
        o_bitmap, o_values, _ = _check_compress(gpu, oracle, x, ws=ws)
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x), ws=ws)
        xh = wl.random_sparse(n, "bf16", 0.6, seed=950 + rep)
        o_bitmap, o_values, _ = _check_compress(gpu, oracle, xh, ws=ws)
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, xh.dtype, wl.bits(xh), ws=ws)
    hdr = ws[:16].cpu().numpy().view(np.uint32)
    assert hdr[0] == 32          # calls completed on this workspace (8 sizes x 4 calls)
    assert hdr[2] == 0           # no tile ever gave up waiting for another tile's count


@pytest.mark.parametrize("dt", ["f32", "bf16", "f64"])
def test_tile_record_and_scan_window_boundaries(gpu, oracle, dt):
    """Sizes around the bookkeeping granularities: a tile (8192 fp32 / 16384 16-bit elements), a
    workspace record (32 tiles), a scanner row (64 tiles) and a scanner pass (448 tiles; 384 and 512 in earlier builds)."""
    tile = {"f32": 8192, "bf16": 16384, "f64": 4096}[dt]
    sizes = []
    for tiles in (1, 31, 32, 33, 63, 64, 65, 383, 384, 385, 447, 448, 449, 511, 512, 513, 897, 1025):
        sizes += [tiles * tile - 1, tiles * tile, tiles * tile + 1]
    for i, n in enumerate(sizes):
        x = wl.random_sparse(n, dt, 0.5 if i % 3 else 0.97, seed=6000 + i)
        o_bitmap, o_values, _ = _check_compress(gpu, oracle, x)
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x))


def test_workspace_reuse_large_small_large(gpu, oracle):
    """What a call leaves in the workspace must never be mistaken for the next call's
    counts, whatever the order of sizes (more tiles, fewer tiles, more again)."""
    import paper_2110_15362_amd.bittrain as bt
    ws = bt.new_workspace(8192 * 1300, torch.float32)
    for rep, tiles in enumerate([1300, 3, 700, 1, 1299, 64, 65, 1300, 513]):
        n = 8192 * tiles - 5 * rep
        x = wl.random_sparse(n, "f32", 0.3 + 0.07 * rep, seed=7000 + rep)
        o_bitmap, o_values, _ = _check_compress(gpu, oracle, x, ws=ws)
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x), ws=ws)
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x), ws=ws)
    assert ws[:16].cpu().numpy().view(np.uint32)[2] == 0


def test_all_zero_and_all_nonzero_large(gpu, oracle):
    n = 8192 * 700 + 123
    for x in (torch.zeros(n), torch.full((n,), -1.5), torch.zeros(n, dtype=torch.float16),
              torch.full((n,), 0.25, dtype=torch.bfloat16)):
        o_bitmap, o_values, o_nnz = _check_compress(gpu, oracle, x)
        assert o_nnz in (0, n)
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x))


def test_empty_tensor(gpu):
    import paper_2110_15362_amd.bittrain as bt
    dev = "cuda"
    x = torch.empty(0, device=dev)
    nnz = torch.full((1,), 99, dtype=torch.int64, device=dev)
    bitmap = torch.empty(0, dtype=torch.int32, device=dev)
    ws = bt.new_workspace(0, torch.float32)
    bt.bt_compress(x, bitmap, x, nnz, ws)
    bt.bt_decompress(bitmap, x, x, ws)
    bt.bt_relu_backward_from_bitmap(bitmap, x, x)
    torch.cuda.synchronize()
    assert int(nnz.item()) == 0


def test_config1(gpu, oracle):
    cfg = wl.config1()
    x, g = cfg["x"], cfg["grad"]
    o_bitmap, o_values, _ = _check_compress(gpu, oracle, x)
    _check_decompress(gpu, oracle, o_bitmap, o_values, x.numel(), x.dtype, wl.bits(x))
    out, ok = gpu.gpu_relu_backward(o_bitmap, g)
    assert np.array_equal(out, oracle.relu_backward(o_bitmap, wl.bits(g))) and ok


@pytest.mark.parametrize("z", [0.5, 0.7, 0.9])
def test_config2_full_size(gpu, oracle, z):
    x = wl.config2(z)["x"]
    o_bitmap, o_values, o_nnz = _check_compress(gpu, oracle, x)
    assert abs(1 - o_nnz / x.numel() - z) < 1e-3
    _check_decompress(gpu, oracle, o_bitmap, o_values, x.numel(), x.dtype, wl.bits(x))
    g = torch.randn(x.numel(), generator=torch.Generator().manual_seed(12))
    out, ok = gpu.gpu_relu_backward(o_bitmap, g)
    assert np.array_equal(out, oracle.relu_backward(o_bitmap, wl.bits(g))) and ok


@pytest.mark.parametrize("variant", ["a", "b"])
def test_config3_full_size(gpu, oracle, variant):
    x = wl.config3(variant)["x"]
    o_bitmap, o_values, o_nnz = _check_compress(gpu, oracle, x)
    assert abs(1 - o_nnz / x.numel() - 0.65) < 5e-3
    _check_decompress(gpu, oracle, o_bitmap, o_values, x.numel(), x.dtype, wl.bits(x))
    g = torch.randn(x.numel(), generator=torch.Generator().manual_seed(13)).to(torch.bfloat16)
    out, ok = gpu.gpu_relu_backward(o_bitmap, g)
    assert np.array_equal(out, oracle.relu_backward(o_bitmap, wl.bits(g))) and ok


def test_config4_resnet50_set_full_size(gpu, oracle):
    """All 49 tensors compressed in forward order with one workspace on one stream, then
    restored in reverse order; every bitmap, value array, nnz and restored tensor is compared."""
    import paper_2110_15362_amd.bittrain as bt
    dev = "cuda"
    shapes = wl.config4_shapes()
    n_max = max(int(np.prod(s)) for s in shapes)
    ws = bt.new_workspace(n_max, torch.float32)
    scratch = torch.empty(n_max, dtype=torch.float32, device=dev)      # worst-case value buffer
    nnz_d = torch.zeros(1, dtype=torch.int64, device=dev)
    stash, dense_bytes, comp_bytes = [], 0, 0
    for cfg in wl.config4_tensors():
        x = cfg["x"].reshape(-1)
        n = x.numel()
        o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
        xd = x.to(dev)
        bitmap = torch.empty((n + 31) // 32, dtype=torch.int32, device=dev)
        bt.bt_compress(xd, bitmap, scratch[:n], nnz_d, ws)
        nnz = int(nnz_d.item())
        assert nnz == o_nnz
        values = scratch[:nnz].clone()                                 # right-sized stash
        assert np.array_equal(bitmap.cpu().numpy().view(np.uint32), o_bitmap), cfg["name"]
        assert np.array_equal(wl.bits(values.cpu()), o_values), cfg["name"]
        stash.append((bitmap, values, n, o_nnz))
        dense_bytes += 4 * n
        comp_bytes += bt.bt_compressed_size(n, nnz, torch.float32)
        assert bt.bt_compressed_size(n, nnz, torch.float32) == oracle.compressed_size(n, o_nnz, 4)
    # backward sweep: regenerate the inputs (same seed) and walk them in reverse
    xs = [c["x"].reshape(-1) for c in wl.config4_tensors()]
    out = torch.empty(n_max, dtype=torch.float32, device=dev)
    for (bitmap, values, n, _), x in zip(reversed(stash), reversed(xs)):
        bt.bt_decompress(bitmap, values, out[:n], ws)
        assert np.array_equal(wl.bits(out[:n].cpu()), wl.bits(x))
    assert dense_bytes == 4 * 614957056
    saved = 1 - comp_bytes / dense_bytes
    assert 0.66 < saved < 0.68, saved        # 70 % zeros: 1 - (0.3 + 1/32)


@pytest.mark.parametrize("p", [0.05, 0.95])
def test_config5_full_size(gpu, oracle, p):
    x = wl.config5(p)["x"]
    n = x.numel()
    o_bitmap, o_values, o_nnz = _check_compress(gpu, oracle, x)
    if p == 0.05:
        assert oracle.compressed_size(n, o_nnz, 2) > 2 * n      # the compressed form is larger
    _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x))


def test_repeated_calls_are_identical(gpu, oracle):
    """The grid scan is the only place where tiles talk to each other: 300 back-to-back
    calls on inputs with whole empty tiles must give the same bytes every time."""
    import paper_2110_15362_amd.bittrain as bt
    dev = "cuda"
    x = wl.config3("b", batch=1)["x"].reshape(-1)
    n = x.numel()
    o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
    xd = x.to(dev)
    ws = bt.new_workspace(n, x.dtype)
    bitmap = torch.empty((n + 31) // 32, dtype=torch.int32, device=dev)
    values = torch.empty(n, dtype=x.dtype, device=dev)
    out = torch.empty_like(xd)
    nnz = torch.zeros(1, dtype=torch.int64, device=dev)
    ref_bitmap = torch.from_numpy(o_bitmap.view(np.int32)).to(dev)
    ref_values = torch.from_numpy(o_values.view(np.int16)).to(dev)
    for it in range(300):
        bitmap.zero_(); values.zero_(); out.fill_(1.0)
        bt.bt_compress(xd, bitmap, values, nnz, ws)
        bt.bt_decompress(bitmap, values, out, ws)
        assert int(nnz.item()) == o_nnz
        assert torch.equal(bitmap, ref_bitmap)
        assert torch.equal(values[:o_nnz].view(torch.int16), ref_values)
        assert torch.equal(out.view(torch.int16), xd.view(torch.int16))


# ---- activation pruning fused into compression (Section 4.3) ------------------------------


def _check_compress_pruned(gpu, oracle, x, dt, thr, **kw):
    o_bitmap, o_values, o_nnz = oracle.compress_pruned(wl.bits(x), dt, thr)
    bitmap, values, nnz, tail_ok = gpu.gpu_compress(x, threshold=thr, **kw)
    assert nnz == o_nnz
    assert np.array_equal(bitmap, o_bitmap)
    assert np.array_equal(values[:o_nnz], o_values)
    assert tail_ok
    return o_bitmap, o_values, o_nnz


@pytest.mark.parametrize("dt", DTYPES)
def test_compress_pruned_thresholds_and_tails(gpu, oracle, dt):
    """The paper's thresholds (0, 0.01, 0.05, 0.1) plus a negative and an infinite one, on
    pre-activation tensors (no ReLU applied), at sizes that cover tiles and ragged tails."""
    for i, n in enumerate([1, 7, 33, 4097, 8192, 8193, 16385, 3 * 16384 + 5, 100003, 600001]):
        x = wl.random_sparse(n, dt, 0.1, seed=8000 + i)      # N(0,1) with a few exact zeros
        for thr in (0.0, 0.01, 0.05, 0.1, -0.5, float("inf")):
            o_bitmap, o_values, o_nnz = _check_compress_pruned(gpu, oracle, x, dt, thr)
        # decompressing the threshold-0 form gives ReLU(x) bit for bit (ReLU(-0.0) = +0 here)
        o_bitmap, o_values, o_nnz = oracle.compress_pruned(wl.bits(x), dt, 0.0)
        relu_bits = wl.bits(torch.where(x.double() > 0, x, torch.zeros_like(x)))
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, relu_bits)


@pytest.mark.parametrize("dt", DTYPES)
def test_compress_pruned_special_values(gpu, oracle, dt):
    """Denormals, -0.0, infinities and NaNs against thresholds that are themselves tiny:
    the comparison is the IEEE single-precision one on both sides."""
    x = wl.special_values(dt).repeat(1100)[:17000]
    tiny = {"f32": 1e-45, "f16": 6e-8, "bf16": 1e-40, "f64": 1e-45}[dt]
    for thr in (0.0, tiny, -tiny, 1.0, float("-inf"), float("nan")):
        _check_compress_pruned(gpu, oracle, x, dt, thr)


def test_compress_pruned_config2_full_size(gpu, oracle):
    x = wl.config2(0.5)["base"]                      # the pre-activation draw: N(0,1), no zeros
    for thr in (0.0, 0.1):
        o_bitmap, o_values, o_nnz = _check_compress_pruned(gpu, oracle, x, "f32", thr)
        assert abs(o_nnz / x.numel() - (0.5 if thr == 0.0 else 0.4602)) < 2e-3


@pytest.mark.parametrize("dt", DTYPES)
def test_mask_apply_with_a_foreign_bitmap(gpu, oracle, dt):
    """Double mask: the bitmap of one tensor (a normalisation layer's input) applied to another
    (its output); out of place and in place; the result compresses to the same bitmap."""
    import paper_2110_15362_amd.bittrain as bt
    for k, n in enumerate((1, 33, 8191, 8193, 3 * 16384 + 5, 1000003)):
        src = wl.random_sparse(n, dt, 0.6, 900 + k)
        y = torch.randn(n, generator=torch.Generator().manual_seed(950 + k)).to(src.dtype)   # dense, like a BN output
        bitmap, _, nnz = oracle.compress(wl.bits(src))
        want = oracle.mask_apply(bitmap, wl.bits(y))
        for inplace in (False, True):
            out, ok = gpu.gpu_relu_backward(bitmap, y, inplace=inplace, call=bt.bt_mask_apply)
            assert ok and np.array_equal(out, want), (n, inplace)
        got_bitmap, _, got_nnz, ok = gpu.gpu_compress(torch.from_numpy(want.view({2: np.int16, 4: np.int32, 8: np.int64}[want.itemsize])).view(src.dtype))
        y_nonzero_under_mask = int(((wl.bits(y) != 0) & (wl.bits(src) != 0)).sum())
        assert ok and got_nnz == y_nonzero_under_mask and got_nnz <= nnz


def test_a_wait_that_runs_out_ends_the_kernel_and_raises_the_flag(gpu, oracle):
    """Failure path, forced from the host: with the wait limit of the workspace set to one pass, the grid scan
    gives up on a tensor that needs two.  The kernels must still end, stay inside their buffers and leave the
    error word set; after bt_workspace_init the workspace works again."""
    import paper_2110_15362_amd.bittrain as bt
    n = 600 * 8192 + 77
    x = wl.random_sparse(n, "f32", 0.5, seed=31337)
    ws = bt.new_workspace(n, torch.float32)
    words = ws.view(torch.int32)
    words[bt.BT_WS_WAIT_LIMIT_WORD] = 1            # one pass of the scan
    bitmap, values, nnz, tail_ok = gpu.gpu_compress(x, ws=ws)          # synchronises; returns at all
    assert tail_ok, "wrote outside bitmap[0,W) or values[0,min(nnz,cap))"
    assert int(words[bt.BT_WS_ERROR_WORD].item()) == 1
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    bt.bt_workspace_status(ws, status)
    assert int(status[0].item()) == 1
    o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
    # a later call on the failed workspace writes nothing: the output keeps the test's fill pattern
    out, guard_ok = gpu.gpu_decompress(o_bitmap, o_values, n, torch.float32, ws=ws)
    assert guard_ok and int(words[bt.BT_WS_ERROR_WORD].item()) == 1
    assert (out == 0x5A5A5A5A).all()
    # whatever a failing call reports as nnz, nothing at or beyond the capacity is written
    bt.bt_workspace_init(ws)
    words[bt.BT_WS_WAIT_LIMIT_WORD] = 1
    cap, guard = n // 8, 4096
    xd = x.cuda()
    vbuf = torch.full((cap + guard,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    bm = torch.empty((n + 31) // 32, dtype=torch.int32, device="cuda")
    nnz_d = torch.zeros(1, dtype=torch.int64, device="cuda")
    bt.bt_compress(xd, bm, vbuf[:cap].view(torch.float32), nnz_d, ws)
    torch.cuda.synchronize()
    assert bool((vbuf[cap:] == 0x5A5A5A5A).all()), "wrote at or beyond the capacity"
    bt.bt_workspace_init(ws)
    assert int(words[bt.BT_WS_ERROR_WORD].item()) == 0 and int(words[bt.BT_WS_WAIT_LIMIT_WORD].item()) == 0
    _check_compress(gpu, oracle, x, ws=ws)
    _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x), ws=ws)
    assert int(words[bt.BT_WS_ERROR_WORD].item()) == 0


@pytest.mark.parametrize("dt", DTYPES)
def test_compression_that_stops_waiting_counts_the_input_itself(gpu, oracle, dt):
    """Forced from the host: with the patience word at one poll a compressing workgroup does not wait for the
    scanner but counts the kept elements before its tile itself.  Every output must be right all the same,
    with and without pruning, and nothing has failed."""
    import paper_2110_15362_amd.bittrain as bt
    n = 70 * bt.bt_tile_elems(wl.DTYPES[dt]) + 4321
    x = wl.random_sparse(n, dt, 0.6, seed=98)
    ws = bt.new_workspace(n, x.dtype)
    ws.view(torch.int32)[bt.BT_WS_PATIENCE_WORD] = 1
    _check_compress(gpu, oracle, x, ws=ws)
    o_bitmap, o_values, o_nnz = oracle.compress(oracle.prune(wl.bits(x), dt, 0.25))
    bitmap, values, nnz, tail_ok = gpu.gpu_compress(x, ws=ws, threshold=0.25)
    assert tail_ok and nnz == o_nnz
    assert np.array_equal(bitmap, o_bitmap) and np.array_equal(values[:o_nnz], o_values)
    assert int(ws.view(torch.int32)[bt.BT_WS_ERROR_WORD].item()) == 0


@pytest.mark.parametrize("dt", DTYPES)
def test_restoration_that_stops_waiting_counts_the_bitmap_itself(gpu, oracle, dt):
    """Forced from the host: with the patience word at one poll a restoring workgroup does not wait for the scanner
    but counts the set bits before its tile itself.  The output must be right all the same, and nothing has failed."""
    import paper_2110_15362_amd.bittrain as bt
    n = 150 * bt.bt_tile_elems(wl.DTYPES[dt]) + 4321
    x = wl.random_sparse(n, dt, 0.6, seed=99)
    o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
    ws = bt.new_workspace(n, x.dtype)
    ws.view(torch.int32)[bt.BT_WS_PATIENCE_WORD] = 1
    for _ in range(2):
        out, guard_ok = gpu.gpu_decompress(o_bitmap, o_values, n, x.dtype, ws=ws)
        assert guard_ok
        assert np.array_equal(out, wl.bits(x))
    assert int(ws.view(torch.int32)[bt.BT_WS_ERROR_WORD].item()) == 0


@pytest.mark.parametrize("dt", DTYPES)
def test_wide_prefix_entries_give_the_same_results(gpu, oracle, dt):
    """Forced from the host: the scanner of a call on one tensor writes 8-byte entries (what it does by itself only
    once the offsets reach 2^32) instead of pairs of lower halves.  Several passes of the scanner, a ragged last tile;
    compression and restoration, two calls in a row on the same workspace."""
    import paper_2110_15362_amd.bittrain as bt
    n = 1100 * bt.bt_tile_elems(wl.DTYPES[dt]) + 77
    x = wl.random_sparse(n, dt, 0.55, seed=123)
    ws = bt.new_workspace(n, x.dtype)
    ws.view(torch.int32)[bt.BT_WS_WIDE_WORD] = 1
    o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
    for _ in range(2):
        bitmap, values, nnz, tail_ok = gpu.gpu_compress(x, ws=ws)
        assert tail_ok and nnz == o_nnz
        assert np.array_equal(bitmap, o_bitmap) and np.array_equal(values[:o_nnz], o_values)
        out, guard_ok = gpu.gpu_decompress(o_bitmap, o_values, n, x.dtype, ws=ws)
        assert guard_ok and np.array_equal(out, wl.bits(x))
    assert int(ws.view(torch.int32)[bt.BT_WS_ERROR_WORD].item()) == 0
    assert int(ws.view(torch.int32)[bt.BT_WS_WIDE_WORD].item()) == 1      # the kernels leave the caller's words alone


def test_stream_probe_stays_inside_its_buffers(gpu):
    """The benchmark's plain stream reads tiles * read_rows * 4 KiB and writes tiles * write_rows * 4 KiB, no more."""
    from paper_2110_15362_amd import bench_aids as bt
    tiles = 777
    for r, w in ((8, 4), (4, 8), (8, 8), (8, 0), (0, 8)):
        src = torch.arange(tiles * max(r, 1) * 1024, dtype=torch.int32, device="cuda")
        guard = 4096
        dst = torch.full((max(tiles * w * 1024, 4 * tiles) + guard,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        bt.bt_stream_probe(src, dst[:dst.numel() - guard], tiles, r, w)
        torch.cuda.synchronize()
        assert bool((dst[dst.numel() - guard:] == 0x5A5A5A5A).all()), (r, w)
        if w:
            assert not bool((dst[:tiles * w * 1024] == 0x5A5A5A5A).all()), (r, w)


@pytest.mark.parametrize("dt", DTYPES)
def test_activation_compress_dense_and_stash_in_one_pass(gpu, oracle, dt):
    """bt_activation_compress: the dense pruned tensor equals the oracle's pruning, the compressed form
    equals Algorithm 1 on it; out of place and in place; ReLU for threshold 0."""
    import paper_2110_15362_amd.bittrain as bt
    dev = "cuda"
    for i, n in enumerate([1, 33, 4097, 8193, 3 * 16384 + 5, 100003, 600001]):
        x = wl.random_sparse(n, dt, 0.1, seed=8500 + i)
        if n > 100:
            x[:16] = wl.special_values(dt)
        xb = wl.bits(x)
        for thr in (0.0, 0.05, -0.5):
            want_dense = oracle.prune(xb, dt, thr)
            o_bitmap, o_values, o_nnz = oracle.compress(want_dense)
            for inplace in (False, True):
                pad = 16 // x.element_size()
                xd = x.to(dev)
                dbuf = xd if inplace else torch.empty(n + pad, dtype=x.dtype, device=dev)
                if not inplace:
                    dbuf.view(torch.uint8).fill_(0x5A)
                dense = xd if inplace else dbuf[:n]
                words = (n + 31) // 32
                bitmap = torch.full((words + 4,), 0x5A5A5A5A, dtype=torch.int32, device=dev)
                values = torch.empty(n + 8, dtype=x.dtype, device=dev)
                values.view(torch.uint8).fill_(0x5A)
                nnz = torch.full((1,), -7, dtype=torch.int64, device=dev)
                ws = bt.new_workspace(n, x.dtype)
                bt.bt_activation_compress(xd, thr, dense, bitmap[:words], values[:n], nnz, ws)
                torch.cuda.synchronize()
                assert int(nnz.item()) == o_nnz, (n, thr, inplace)
                assert np.array_equal(wl.bits(dense.cpu()), want_dense), (n, thr, inplace)
                assert np.array_equal(bitmap[:words].cpu().numpy().view(np.uint32), o_bitmap)
                assert np.array_equal(wl.bits(values[:o_nnz].cpu()), o_values)
                sent = np.frombuffer(bytes([0x5A] * x.element_size()), dtype=wl.bits(values.cpu()).dtype)[0]
                assert (wl.bits(values[o_nnz:].cpu()) == sent).all() and bool((bitmap[words:] == 0x5A5A5A5A).all())
                if not inplace:
                    assert (wl.bits(dbuf[n:].cpu()) == sent).all(), "wrote past dense[n)"
    # threshold 0 on pre-activations is ReLU
    x = wl.random_sparse(50000, "f32", 0.0, seed=8600)
    xd = x.to(dev)
    y = torch.empty_like(xd)
    bitmap = torch.empty((50000 + 31) // 32, dtype=torch.int32, device=dev)
    values = torch.empty(50000, device=dev)
    nnz = torch.zeros(1, dtype=torch.int64, device=dev)
    bt.bt_activation_compress(xd, 0.0, y, bitmap, values, nnz, bt.new_workspace(50000, torch.float32))
    torch.cuda.synchronize()
    assert torch.equal(y, torch.relu(xd))


@pytest.mark.parametrize("dt", ["f32", "bf16", "f64"])
def test_bitmap_bits_beyond_n_are_ignored(gpu, oracle, dt):
    """A bitmap whose last word carries set bits at positions >= n (not what bt_compress writes, but allowed
    on input): Algorithm 2 and the select run over the n valid bits only."""
    import paper_2110_15362_amd.bittrain as bt
    for n in (5, 33, 8191, 3 * 16384 + 7, 100001):
        x = wl.random_sparse(n, dt, 0.5, seed=9100 + n % 97)
        o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
        dirty = o_bitmap.copy()
        dirty[-1] |= np.uint32((0xFFFFFFFF << (n % 32)) & 0xFFFFFFFF)          # n % 32 != 0 for these sizes
        assert not np.array_equal(dirty, o_bitmap)
        out, ok = gpu.gpu_decompress(dirty, o_values, n, x.dtype)
        assert ok and np.array_equal(out, wl.bits(x))
        g = torch.randn(n, generator=torch.Generator().manual_seed(n)).to(x.dtype)
        got, ok = gpu.gpu_relu_backward(dirty, g)
        assert ok and np.array_equal(got, oracle.relu_backward(o_bitmap, wl.bits(g)))
        # the indexed restoration too
        tile = bt.bt_tile_elems(x.dtype)
        index = torch.from_numpy(oracle.tile_index(o_bitmap, n, tile).view(np.int64).copy()).cuda()
        bm = torch.from_numpy(dirty.view(np.int32).copy()).cuda()
        vals = x[x.view({2: torch.int16, 4: torch.int32, 8: torch.int64}[x.element_size()]) != 0].cuda()
        outd = torch.empty(n, dtype=x.dtype, device="cuda")
        bt.bt_decompress_indexed(bm, vals, index, outd)
        torch.cuda.synchronize()
        assert np.array_equal(wl.bits(outd.cpu()), wl.bits(x))


def test_two_streams_with_their_own_workspaces(gpu, oracle):
    """Calls that use distinct workspaces are independent: two streams (default priority) compress and
    restore different tensors at the same time, several times over."""
    import paper_2110_15362_amd.bittrain as bt
    dev = "cuda"
    xs = [wl.random_sparse(n, "f32", z, seed=9300 + k) for k, (n, z) in enumerate(((300 * 8192 + 5, 0.5), (170 * 8192 + 9, 0.8)))]
    want = [oracle.compress(wl.bits(x)) for x in xs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bufs = []
    for x in xs:
        n = x.numel()
        bufs.append(dict(x=x.to(dev), bitmap=torch.empty((n + 31) // 32, dtype=torch.int32, device=dev),
                         values=torch.empty(n, device=dev), out=torch.empty(n, device=dev),
                         nnz=torch.zeros(1, dtype=torch.int64, device=dev), ws=bt.new_workspace(n, torch.float32)))
    torch.cuda.synchronize()
    for rep in range(5):
        for b in bufs:
            b["values"].fill_(7); b["out"].fill_(7); b["bitmap"].fill_(-1)
        torch.cuda.synchronize()
        for s, b in zip(streams, bufs):
            with torch.cuda.stream(s):
                for _ in range(3):
                    bt.bt_compress(b["x"], b["bitmap"], b["values"], b["nnz"], b["ws"])
                    bt.bt_decompress(b["bitmap"], b["values"], b["out"], b["ws"])
        torch.cuda.synchronize()
        for b, x, (o_bitmap, o_values, o_nnz) in zip(bufs, xs, want):
            assert int(b["nnz"].item()) == o_nnz
            assert np.array_equal(b["bitmap"].cpu().numpy().view(np.uint32), o_bitmap)
            assert np.array_equal(wl.bits(b["values"][:o_nnz].cpu()), o_values)
            assert np.array_equal(wl.bits(b["out"].cpu()), wl.bits(x))
            assert int(b["ws"].view(torch.int32)[2].item()) == 0


def _pattern_masks(n, tile):
    """Zero / non-zero layouts whose run lengths sit on, just before and just after the sizes the kernels
    work in: a 16-byte vector, a bitmap word, a wave row, a wave strip, a tile."""
    i = np.arange(n)
    row, strip = tile // 32, tile // 4
    masks = {"alternate": i % 2 == 0, "every_32nd": i % 32 == 31, "every_33rd": i % 33 == 0,
             "first_of_each_word_missing": i % 32 != 0, "dense_then_empty": i < n // 2, "empty_then_dense": i >= n // 2,
             "only_the_last_tile": i >= (n // tile) * tile, "only_the_last_element": i == n - 1}
    for name, period in (("row", row), ("strip", strip), ("tile", tile)):
        masks["every_other_%s" % name] = (i // period) % 2 == 0
        masks["runs_of_%s_minus_1" % name] = (i // (period - 1)) % 2 == 1
        masks["runs_of_%s_plus_1" % name] = (i // (period + 1)) % 2 == 1
        masks["one_per_%s" % name] = i % period == period - 1
    rng = np.random.default_rng(17)
    for block in (3, 64, 1000):
        masks["random_blocks_of_%d" % block] = np.repeat(rng.random(n // block + 1) < 0.4, block)[:n]
    return masks


@pytest.mark.parametrize("dt", ["f32", "f16", "f64"])
def test_structured_zero_patterns(gpu, oracle, dt):
    """The ranks, the scatter through LDS and the tile offsets depend on where the zeros are, not
    only on how many there are: run lengths on and around every internal size."""
    tile = {"f32": 8192, "f16": 16384, "f64": 4096}[dt]
    n = 3 * tile + tile // 4 + 37
    base = wl.random_sparse(n, dt, 0.0, 23)                    # no zeros: every kept element is distinct enough
    g = wl.random_sparse(n, dt, 0.0, 24)
    assert int((wl.bits(base) == 0).sum()) == 0
    for name, keep in _pattern_masks(n, tile).items():
        x = base.clone()
        x[torch.from_numpy(~keep)] = 0
        o_bitmap, o_values, o_nnz = _check_compress(gpu, oracle, x)
        assert o_nnz == int(keep.sum()), name
        _check_decompress(gpu, oracle, o_bitmap, o_values, n, x.dtype, wl.bits(x))
        out, guard_ok = gpu.gpu_relu_backward(o_bitmap, g)
        assert np.array_equal(out, oracle.relu_backward(o_bitmap, wl.bits(g))) and guard_ok, name
