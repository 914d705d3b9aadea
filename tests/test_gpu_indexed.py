"""GPU parity of the tile index and of Algorithm 2 started from it, against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2110_15362_amd import workloads as wl

pytestmark = pytest.mark.gpu

SENT = 0x5A
DTYPES = ["f32", "f16", "bf16", "f64"]


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


def _values_tensor(values_np, dtype):
    return torch.from_numpy(values_np.view({2: np.int16, 4: np.int32, 8: np.int64}[values_np.itemsize]).copy()).view(dtype)


def _compress_indexed(bt, x, ws=None):
    n = x.numel()
    words, tiles = (n + 31) // 32, bt.bt_index_bytes(n, x.dtype) // 8
    bitmap = _sentinel(words + 4, torch.int32)
    values = _sentinel(n + 8, x.dtype)
    index = _sentinel(tiles + 2, torch.int64)
    nnz = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    ws = bt.new_workspace(n, x.dtype) if ws is None else ws
    bt.bt_compress_indexed(x.cuda(), bitmap[:words], values[:n], nnz, index[:tiles], ws)
    torch.cuda.synchronize()
    k = int(nnz.item())
    bm, vb, ib = bitmap.cpu().numpy().view(np.uint32), wl.bits(values.cpu()), index.cpu().numpy().view(np.uint64)
    sent = np.frombuffer(bytes([SENT] * vb.itemsize), dtype=vb.dtype)[0]
    assert (bm[words:] == 0x5A5A5A5A).all() and (vb[k:] == sent).all() and (ib[tiles:] == 0x5A5A5A5A5A5A5A5A).all()
    return bm[:words].copy(), vb[:k].copy(), k, ib[:tiles].copy()


def _decompress_indexed(bt, bitmap_np, values_np, index_np, n, dtype, values_offset=0):
    pad = 16 // torch.empty(0, dtype=dtype).element_size()
    bitmap = torch.from_numpy(bitmap_np.view(np.int32).copy()).cuda()
    vbuf = _sentinel(values_np.size + values_offset + 8, dtype)
    vbuf[values_offset:values_offset + values_np.size] = _values_tensor(values_np, dtype).cuda()
    index = torch.from_numpy(index_np.view(np.int64).copy()).cuda()
    obuf = _sentinel(n + pad, dtype)
    bt.bt_decompress_indexed(bitmap, vbuf[values_offset:values_offset + values_np.size], index, obuf[:n])
    torch.cuda.synchronize()
    ob = wl.bits(obuf.cpu())
    sent = np.frombuffer(bytes([SENT] * ob.itemsize), dtype=ob.dtype)[0]
    assert (ob[n:] == sent).all(), "wrote past out[n)"
    return ob[:n].copy()


@pytest.mark.parametrize("dt", DTYPES)
def test_index_and_indexed_decompress_sizes_and_tails(bt, oracle, dt):
    tile = bt.bt_tile_elems(wl.DTYPES[dt])
    sizes = [1, 33, tile - 1, tile, tile + 1, 2 * tile + 17, 64 * tile, 65 * tile + 3, 100003, 1000037]
    for i, n in enumerate(sizes):
        x = wl.random_sparse(n, dt, [0.5, 0.97, 0.0, 0.7][i % 4], seed=7000 + i)
        xb = wl.bits(x)
        o_bitmap, o_values, o_nnz = oracle.compress(xb)
        o_index = oracle.tile_index(o_bitmap, n, tile)
        bitmap, values, nnz, index = _compress_indexed(bt, x)
        assert nnz == o_nnz and np.array_equal(bitmap, o_bitmap) and np.array_equal(values, o_values), n
        assert np.array_equal(index, o_index), n
        # Algorithm 2 from the oracle's index and the oracle's compressed form
        out = _decompress_indexed(bt, o_bitmap, o_values, o_index, n, x.dtype, values_offset=i % 3)
        assert np.array_equal(out, oracle.decompress(o_bitmap, o_values, n)), n
        assert np.array_equal(out, xb), n


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_indexed_special_patterns_and_extremes(bt, oracle, dt):
    tile = bt.bt_tile_elems(wl.DTYPES[dt])
    cases = [wl.special_values(dt).repeat(900), torch.zeros(3 * tile + 5).to(wl.DTYPES[dt]),
             torch.ones(2 * tile + 1).to(wl.DTYPES[dt]),
             torch.cat([torch.zeros(2 * tile), torch.ones(7), torch.zeros(tile)]).to(wl.DTYPES[dt])]
    for x in cases:
        n = x.numel()
        o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
        bitmap, values, nnz, index = _compress_indexed(bt, x)
        assert nnz == o_nnz and np.array_equal(index, oracle.tile_index(o_bitmap, n, tile))
        out = _decompress_indexed(bt, bitmap, values, index, n, x.dtype)
        assert np.array_equal(out, wl.bits(x))


def test_indexed_decompress_never_reads_beyond_the_values_it_was_given(bt, oracle):
    """An index that does not belong to the bitmap gives a wrong tensor, but the call stays inside its
    buffers: with the capacity cut to half the values, everything restored from the first half is right."""
    tile = bt.bt_tile_elems(torch.float32)
    n = 40 * tile + 11
    x = wl.random_sparse(n, "f32", 0.5, seed=7100)
    o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
    o_index = oracle.tile_index(o_bitmap, n, tile)
    half = o_nnz // 2
    out = _decompress_indexed(bt, o_bitmap, o_values[:half], o_index, n, torch.float32)
    # tiles whose values all lie below `half` are exact
    ends = np.append(o_index[1:], o_nnz)
    good_tiles = int((ends <= half).sum())
    assert good_tiles >= 15
    assert np.array_equal(out[:good_tiles * tile], wl.bits(x)[:good_tiles * tile])
    # an index of garbage: any result, no fault, guards intact (checked inside the helper)
    garbage = (np.arange(o_index.size, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15))
    _decompress_indexed(bt, o_bitmap, o_values, garbage, n, torch.float32)


def test_indexed_config2_full_size(bt, oracle):
    x = wl.config2(0.5)["x"].reshape(-1)
    n = x.numel()
    tile = bt.bt_tile_elems(torch.float32)
    o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(x))
    bitmap, values, nnz, index = _compress_indexed(bt, x)
    assert nnz == o_nnz and np.array_equal(bitmap, o_bitmap) and np.array_equal(values, o_values)
    assert np.array_equal(index, oracle.tile_index(o_bitmap, n, tile))
    out = _decompress_indexed(bt, bitmap, values, index, n, torch.float32)
    assert np.array_equal(out, wl.bits(x))
