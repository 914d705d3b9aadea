"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, its host-only functions agree with the paper's numbers, and argument
errors are reported before anything is launched (so none of this needs a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bittrain.h")


@pytest.fixture(scope="module")
def bt():
    import paper_2110_15362_amd.bittrain as bt
    if not os.path.exists(bt.LIB_PATH):
        from paper_2110_15362_amd import build
        build.build()
    bt.lib()
    return bt


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(bt_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(bt):
    names = _declared_functions()
    assert {"bt_compress", "bt_compressed_size", "bt_decompress", "bt_relu_backward_from_bitmap",
            "bt_compress_pruned", "bt_compress_batch", "bt_decompress_batch", "bt_batch_workspace_bytes",
            "bt_mask_apply", "bt_dense_size", "bt_coo_size", "bt_compress_indexed", "bt_decompress_indexed",
            "bt_tile_elems", "bt_index_bytes", "bt_activation_compress"} <= set(names)
    raw = ctypes.CDLL(bt.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), name
    # and nothing else: the benchmark's measurement aids live in a library of their own
    assert not hasattr(raw, "bt_stream_probe") and not hasattr(raw, "bt_timeline_set")


def test_binding_constants_are_the_headers(bt):
    text = open(os.path.join(os.path.dirname(__file__), "..", "include", "bittrain.h")).read()
    for name in ("BT_WS_ERROR_WORD", "BT_WS_WAIT_LIMIT_WORD", "BT_WS_PATIENCE_WORD", "BT_WS_WIDE_WORD", "BT_STATIC_MAX_TILES"):
        assert int(re.search(r"#define\s+%s\s+(\d+)" % name, text).group(1)) == getattr(bt, name)


def test_header_compiles_as_plain_c(tmp_path):
    import subprocess
    src = tmp_path / "t.c"
    src.write_text('#include "bittrain.h"\nint main(void){return (int)bt_bitmap_bytes(0);}\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])


def test_compressed_size_matches_table1(bt):
    golden = os.path.join(ROOT, "tests", "golden", "table1_theoretical.txt")
    rows = 0
    for line in open(golden):
        if line.startswith("#") or not line.strip():
            continue
        _, _, _, _, n, pct, dense_mb, bitmap_mb, improv = line.split()
        n, pct = int(n), int(pct)
        size = bt.bt_compressed_size(n, n * pct // 100, bt.BT_F32)
        assert abs(size / 2**20 - float(bitmap_mb)) <= 0.005 + 1e-9
        assert abs(100 * (1 - size / (4 * n)) - float(improv)) <= 0.005 + 1e-9
        rows += 1
    assert rows == 30


def test_size_helpers(bt, oracle):
    for n in (0, 1, 31, 32, 33, 4096, 25690112):
        assert bt.bt_bitmap_bytes(n) == 4 * ((n + 31) // 32)
        for code, width in ((bt.BT_F32, 4), (bt.BT_F16, 2), (bt.BT_BF16, 2), (bt.BT_F64, 8)):
            for nnz in (0, n // 3, n):
                assert bt.bt_compressed_size(n, nnz, code) == oracle.compressed_size(n, nnz, width)
            assert bt.lib().bt_dtype_size(code) == width
            assert bt.bt_workspace_bytes(n, code) >= 256 + 8
    assert bt.bt_compressed_size(10, 11, bt.BT_F32) == 0
    assert bt.bt_compressed_size(10, 1, 9) == 0
    assert bt.bt_workspace_bytes(10, 9) == 0
    assert bt.bt_workspace_bytes(10**6, bt.BT_F32) <= bt.bt_workspace_bytes(10**7, bt.BT_F32)
    assert bt.status_str(0) == "ok" and bt.status_str(4) == "workspace too small"


def test_argument_errors_are_found_on_the_host(bt):
    L = bt.lib()
    A = 0x10000          # a fake, well aligned "device" address: never dereferenced on an error path
    ws_bytes = bt.bt_workspace_bytes(1000, bt.BT_F32)
    ok_args = dict(d_in=A, n=1000, dt=bt.BT_F32, bm=A, val=A, cap=1000, nnz=A, ws=A, wsb=ws_bytes)

    def compress(**kw):
        a = dict(ok_args, **kw)
        return L.bt_compress(a["d_in"], a["n"], a["dt"], a["bm"], a["val"], a["cap"], a["nnz"], a["ws"], a["wsb"], None)

    assert compress(dt=7) == 2                      # BT_ERR_DTYPE
    assert compress(d_in=None) == 1                 # BT_ERR_NULL
    assert compress(bm=None) == 1
    assert compress(val=None) == 1
    assert compress(nnz=None) == 1
    assert compress(ws=None) == 1
    assert compress(d_in=A + 4) == 3                # BT_ERR_ALIGN: input needs 16 bytes
    assert compress(bm=A + 2) == 3
    assert compress(val=A + 2) == 3                 # fp32 values need 4 bytes
    assert compress(nnz=A + 4) == 3
    assert compress(ws=A + 4) == 3
    assert compress(wsb=ws_bytes - 1) == 4          # BT_ERR_WORKSPACE
    assert compress(n=(1 << 37) + 1) == 6           # BT_ERR_SIZE

    def decompress(bm=A, val=A, n=1000, dt=bt.BT_F32, out=A, ws=A, wsb=ws_bytes):
        return L.bt_decompress(bm, val, n, dt, out, ws, wsb, None)

    assert decompress(dt=-1) == 2
    assert decompress(bm=None) == 1 and decompress(out=None) == 1 and decompress(ws=None) == 1
    assert decompress(out=A + 8) == 3 and decompress(val=A + 1) == 3
    assert decompress(wsb=8) == 4
    assert decompress(n=0, bm=None, val=None, out=None, ws=None, wsb=0) == 0     # nothing to do

    def relu(bm=A, g=A, n=1000, dt=bt.BT_BF16, gi=A):
        return L.bt_relu_backward_from_bitmap(bm, g, n, dt, gi, None)

    assert relu(dt=4) == 2
    assert relu(bm=None) == 1 and relu(g=None) == 1 and relu(gi=None) == 1
    assert relu(g=A + 2) == 3 and relu(gi=A + 8) == 3 and relu(bm=A + 1) == 3
    assert relu(n=0, bm=None, g=None, gi=None) == 0
    assert L.bt_workspace_init(None, 100, None) == 1
    assert L.bt_workspace_init(A + 1, 100, None) == 3


def test_batch_workspace_bytes_and_host_errors(bt):
    L = bt.lib()
    f32, f16 = bt.BT_F32, bt.BT_F16
    tile = {f32: 8192, f16: 16384}

    def expect(ns, code):
        # every tensor takes its tiles rounded up to whole rows of 128 slots (at least one row);
        # 24 bytes per slot in blocks of 256 slots, plus the 256-byte header; the largest launch decides,
        # whether the batch is cut into launches of 52 tensors (compression) or of 64 (restoration)
        need = 256 + 6144
        for per_launch in (52, 64):
            for first in range(0, len(ns), per_launch):
                slots = sum(max(1, -(-(-(-n // tile[code])) // 128)) * 128 for n in ns[first:first + per_launch])
                need = max(need, 256 + 6144 * -(-slots // 256))
        return need

    for code in (f32, f16):
        t = tile[code]
        for ns in ([], [0], [1], [t], [64 * t], [64 * t + 1], [5, 0, 200 * t, 3 * t + 1],
                   [t + 1] * 64, [t + 1] * 65, [1] * 130 + [1000 * t]):
            assert bt.bt_batch_workspace_bytes(ns, code) == expect(ns, code), (code, ns)
        # a batch of one tensor never needs less than the single-tensor call
        for n in (1, t, 63 * t, 64 * t + 1, 25690112):
            assert bt.bt_batch_workspace_bytes([n], code) >= bt.bt_workspace_bytes(n, code)
    assert bt.bt_batch_workspace_bytes([10], 9) == 0
    assert L.bt_batch_workspace_bytes(None, 3, f32) == 0

    A = 0x10000

    def c_items(**kw):
        a = dict(d_in=A, n=1000, d_bitmap=A, d_values=A, values_cap=1000, d_nnz=A)
        a.update(kw)
        good = bt.CompressItem(A, 1000, A, A, 1000, A)
        return (bt.CompressItem * 3)(good, bt.CompressItem(a["d_in"], a["n"], a["d_bitmap"], a["d_values"],
                                                            a["values_cap"], a["d_nnz"]), good)

    wsb = bt.bt_batch_workspace_bytes([1000] * 3, f32)

    def compress(items=None, count=3, dt=f32, ws=A, wsb=wsb, **kw):
        return L.bt_compress_batch(c_items(**kw) if items is None else items, count, dt, ws, wsb, None)

    assert compress(dt=5) == 2
    assert compress(ws=None) == 1
    assert compress(ws=A + 64) == 3
    assert compress(d_in=None) == 1 and compress(d_bitmap=None) == 1 and compress(d_nnz=None) == 1
    assert compress(d_values=None) == 1
    assert compress(d_in=A + 8) == 3 and compress(d_values=A + 2) == 3 and compress(d_nnz=A + 4) == 3
    assert compress(n=(1 << 37) + 1) == 6
    assert compress(wsb=wsb - 1) == 4
    assert compress(n=0, d_nnz=None) == 1             # an empty tensor still reports its nnz
    assert L.bt_compress_batch(None, 3, f32, A, wsb, None) == 1
    assert L.bt_compress_batch(None, 0, f32, None, 0, None) == 0     # nothing to do

    def d_items(bm=A, val=A, n=1000, out=A):
        good = bt.DecompressItem(A, A, 1000, A)
        return (bt.DecompressItem * 3)(good, good, bt.DecompressItem(bm, val, n, out))

    def decompress(count=3, dt=f32, ws=A, wsb=wsb, **kw):
        return L.bt_decompress_batch(d_items(**kw), count, dt, ws, wsb, None)

    assert decompress(dt=-1) == 2
    assert decompress(ws=None) == 1 and decompress(ws=A + 32) == 3
    assert decompress(bm=None) == 1 and decompress(out=None) == 1
    assert decompress(out=A + 4) == 3 and decompress(val=A + 1) == 3 and decompress(bm=A + 2) == 3
    assert decompress(n=(1 << 37) + 1) == 6
    assert decompress(wsb=wsb - 1) == 4
    assert L.bt_decompress_batch(None, 0, f32, None, 0, None) == 0

    # the pruning batch: one dense output for every tensor that has elements, or for none; never without pruning
    def c_dense(dense, index=None, n=1000):
        good = bt.CompressItem(A, 1000, A, A, 1000, A, None, A)
        return (bt.CompressItem * 3)(good, bt.CompressItem(A, n, A, A, 1000, A, index, dense), good)

    pruned = lambda items, thr=0.0: L.bt_compress_batch_pruned(items, 3, f32, ctypes.c_double(thr), A, wsb, None)
    assert pruned(c_dense(None)) == 1                      # two tensors have one, the third has not
    assert pruned(c_dense(A + 8)) == 3
    assert pruned(c_dense(A, index=A + 4)) == 3
    assert L.bt_compress_batch(c_dense(A), 3, f32, A, wsb, None) == 1      # a dense output without pruning
    assert L.bt_compress_batch_pruned(None, 3, f32, ctypes.c_double(0.0), A, wsb, None) == 1
    assert L.bt_compress_batch_pruned(None, 0, f32, ctypes.c_double(0.0), None, 0, None) == 0
    assert compress(items=c_items(), wsb=wsb - 1) == 4

    # restoration from tile indexes: no workspace, the index required
    def di_items(bm=A, val=A, n=1000, out=A, cap=1000, index=A):
        good = bt.DecompressItem(A, A, 1000, A, 1000, A)
        return (bt.DecompressItem * 3)(good, good, bt.DecompressItem(bm, val, n, out, cap, index))

    indexed = lambda dt=f32, count=3, **kw: L.bt_decompress_batch_indexed(di_items(**kw), count, dt, None)
    assert indexed(dt=7) == 2
    assert indexed(index=None) == 1 and indexed(bm=None) == 1 and indexed(out=None) == 1 and indexed(val=None) == 1
    assert indexed(index=A + 4) == 3 and indexed(out=A + 8) == 3
    assert indexed(n=(1 << 37) + 1) == 6
    assert L.bt_decompress_batch_indexed(None, 3, f32, None) == 1
    assert L.bt_decompress_batch_indexed(None, 0, f32, None) == 0

    # the workspace's state
    assert L.bt_workspace_status(None, A, None) == 1 and L.bt_workspace_status(A, None, None) == 1
    assert L.bt_workspace_status(A + 64, A, None) == 3 and L.bt_workspace_status(A, A + 2, None) == 3

    # the entry point without a workspace refuses what its own workspace cannot hold, before anything else
    assert L.bt_compress_static(None, 16385 * 8192, f32, None, None, 0, None, None) == 6
    assert L.bt_compress_static(None, 16384 * 16384 + 1, f16, None, None, 0, None, None) == 6
    assert L.bt_compress_static(None, 10, 9, None, None, 0, None, None) == 2


def test_dense_and_coo_sizes_match_the_oracle(bt, oracle):
    for code, width in ((bt.BT_F32, 4), (bt.BT_F16, 2), (bt.BT_BF16, 2), (bt.BT_F64, 8)):
        for n in (0, 1, 33, 3211264, 25690112):
            assert bt.bt_dense_size(n, code) == oracle.dense_size(n, width)
            for ndim in (1, 2, 3, 4):
                for ib in (4, 8):
                    assert bt.bt_coo_size(n // 3, ndim, ib, code) == oracle.coo_size(n // 3, ndim, ib, width)
    assert bt.bt_dense_size(10, 9) == 0
    assert bt.bt_coo_size(10, 0, 4, bt.BT_F32) == 0 and bt.bt_coo_size(10, 4, 2, bt.BT_F32) == 0
    assert bt.bt_coo_size(10, 4, 4, 9) == 0
    L = bt.lib()
    A = 0x10000
    assert L.bt_mask_apply(None, A, 10, bt.BT_F32, A, None) == 1
    assert L.bt_mask_apply(A, A + 4, 10, bt.BT_F32, A, None) == 3
    assert L.bt_mask_apply(A, A, 10, 7, A, None) == 2
    assert L.bt_mask_apply(None, None, 0, bt.BT_F32, None, None) == 0


def test_footprint_calculator_reproduces_table1_and_the_coo_break_even(bt):
    import torch
    from paper_2110_15362_amd import footprint as fp
    golden = os.path.join(ROOT, "tests", "golden", "table1_theoretical.txt")
    rows = 0
    for line in open(golden):
        if line.startswith("#") or not line.strip():
            continue
        b, c, w, h, n, pct, dense_mb, bitmap_mb, improv = line.split()
        r = fp.footprint((int(b), int(c), int(w), int(h)), int(pct) / 100.0)
        assert r["elements"] == int(n)
        assert abs(r["dense_bytes"] / 2**20 - float(dense_mb)) <= 0.005 + 1e-9
        assert abs(r["bitmap_bytes"] / 2**20 - float(bitmap_mb)) <= 0.005 + 1e-9
        assert abs(r["bitmap_improvement_pct"] - float(improv)) <= 0.005 + 1e-9
        rows += 1
    assert rows == 30
    # Section 3.2: COO pays off only at about 20 % non-zeros or fewer (4-D activation, integer indices)
    be = fp.break_even_nonzero_fraction(4, 4)
    assert be["coo_vs_dense"] == 0.2 and be["bitmap_vs_dense"] == 31 / 32
    sw = fp.sweep((16, 64, 56, 56), fractions=(0.1, 0.2, 0.3, 0.9))
    assert sw[0]["coo_int_bytes"] < sw[0]["dense_bytes"] and sw[2]["coo_int_bytes"] > sw[2]["dense_bytes"]
    assert all(r["bitmap_bytes"] < r["dense_bytes"] and r["bitmap_bytes"] < r["coo_int_bytes"] for r in sw)
    assert fp.footprint((8, 2048, 4096), 0.35, torch.bfloat16)["bitmap_bytes"] == 2 * int(8 * 2048 * 4096 * 0.35) + 8 * 2048 * 4096 // 8


def test_tile_index_sizes_and_host_errors(bt):
    for code, width in ((bt.BT_F32, 4), (bt.BT_F16, 2), (bt.BT_BF16, 2), (bt.BT_F64, 8)):
        tile = bt.bt_tile_elems(code)
        assert tile * width == 32 * 1024
        for n in (0, 1, tile - 1, tile, tile + 1, 25690112):
            assert bt.bt_index_bytes(n, code) == 8 * -(-n // tile)
    assert bt.bt_tile_elems(9) == 0 and bt.bt_index_bytes(100, 9) == 0
    L = bt.lib()
    A = 0x10000
    wsb = bt.bt_workspace_bytes(1000, bt.BT_F32)

    def compress(d_in=A, n=1000, dt=bt.BT_F32, bm=A, val=A, cap=1000, nnz=A, idx=A, ws=A, wsb=wsb):
        return L.bt_compress_indexed(d_in, n, dt, bm, val, cap, nnz, idx, ws, wsb, None)

    assert compress(idx=None) == 1 and compress(idx=A + 4) == 3
    assert compress(dt=8) == 2 and compress(d_in=None) == 1 and compress(nnz=None) == 1
    assert compress(d_in=A + 8) == 3 and compress(wsb=wsb - 1) == 4 and compress(n=(1 << 37) + 1) == 6

    def decompress(bm=A, val=A, cap=1000, idx=A, n=1000, dt=bt.BT_F32, out=A):
        return L.bt_decompress_indexed(bm, val, cap, idx, n, dt, out, None)

    assert decompress(dt=4) == 2 and decompress(n=(1 << 37) + 1) == 6
    assert decompress(bm=None) == 1 and decompress(out=None) == 1 and decompress(idx=None) == 1
    assert decompress(val=None) == 1                       # a capacity without a buffer
    assert decompress(out=A + 4) == 3 and decompress(idx=A + 2) == 3 and decompress(val=A + 2) == 3
    assert decompress(n=0, bm=None, val=None, cap=0, idx=None, out=None) == 0


def test_activation_compress_host_errors(bt):
    L = bt.lib()
    A = 0x10000
    wsb = bt.bt_workspace_bytes(1000, bt.BT_F32)

    def call(d_in=A, n=1000, dt=bt.BT_F32, thr=0.0, dense=A + 0x10000, bm=A, val=A, cap=1000, nnz=A, ws=A, wsb=wsb):
        return L.bt_activation_compress(d_in, n, dt, ctypes.c_double(thr), dense, bm, val, cap, nnz, ws, wsb, None)

    assert call(dense=None) == 1 and call(dense=A + 8) == 3
    assert call(dt=9) == 2 and call(d_in=None) == 1 and call(nnz=None) == 1 and call(bm=None) == 1
    assert call(wsb=wsb - 1) == 4 and call(n=(1 << 37) + 1) == 6 and call(d_in=A + 4) == 3


def test_bench_aids_host_errors(bt):
    """libbittrain_bench.so (bench.py's measurement aids: the codec with time stamps, and a plain stream)
    exports the whole interface too and checks its own two calls' arguments on the host."""
    from paper_2110_15362_amd import bench_aids
    L = bench_aids.lib()
    for name in _declared_functions():
        assert hasattr(L, name), name
    A = 0x10000
    assert L.bt_stream_probe(None, A, 10, 8, 4, None) == 1 and L.bt_stream_probe(A, None, 10, 8, 4, None) == 1
    assert L.bt_stream_probe(A + 8, A, 10, 8, 4, None) == 3
    assert L.bt_stream_probe(A, A, 10, 3, 5, None) == 6          # not one of the listed shapes
    assert L.bt_stream_probe(A, A, 1 << 31, 8, 4, None) == 6
    assert L.bt_stream_probe(A, A, 0, 8, 4, None) == 0
    assert L.bt_timeline_set(0x10000, 8 * 100 + 2 * 10 - 1, 100, 10) == 6      # buffer one word too small
    assert L.bt_timeline_set(0x10004, 8 * 100 + 2 * 10, 100, 10) == 3          # misaligned


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2
    assert "single-GPU" in res.stderr


def test_workspace_bytes_cover_every_tile(bt):
    # 256-byte header + one 6 KiB block per 256 tiles of 32 KiB of dense data
    for code, elems_per_tile in ((bt.BT_F32, 8192), (bt.BT_F16, 16384), (bt.BT_BF16, 16384), (bt.BT_F64, 4096)):
        for tiles in (1, 255, 256, 257, 3136, 100000):
            n = tiles * elems_per_tile
            assert bt.bt_workspace_bytes(n, code) == 256 + 6144 * ((tiles + 255) // 256)
            assert bt.bt_workspace_bytes(n + 1, code) == 256 + 6144 * ((tiles + 1 + 255) // 256)
