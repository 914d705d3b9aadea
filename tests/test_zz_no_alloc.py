"""bt_compress_static (the entry point that allocates nothing) against bt_compress, through the C ABI:
two calls in a row on the library's own workspace, the second on a smaller tensor, then a size beyond
the limit."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(bt, n, dtype, zero_fraction, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn(n, generator=g)
    x[torch.rand(n, generator=g) < zero_fraction] = 0
    x = x.to(dtype).cuda()
    words = (n + 31) // 32
    got = dict(bitmap=torch.full((words,), -1, dtype=torch.int32, device="cuda"), values=torch.full((n,), 7, dtype=dtype, device="cuda"),
               nnz=torch.full((1,), -1, dtype=torch.int64, device="cuda"))
    ref = {k: v.clone() for k, v in got.items()}
    ws = bt.new_workspace(n, dtype)
    bt.bt_compress(x, ref["bitmap"], ref["values"], ref["nnz"], ws)
    bt.bt_compress_static(x, got["bitmap"], got["values"], got["nnz"])
    torch.cuda.synchronize()
    iv = {2: torch.int16, 4: torch.int32, 8: torch.int64}[x.element_size()]
    assert int(got["nnz"].item()) == int(ref["nnz"].item()) == int((x.view(iv) != 0).sum().item())
    assert torch.equal(got["bitmap"], ref["bitmap"])
    assert torch.equal(got["values"].view(iv), ref["values"].view(iv))      # untouched tail included


def test_two_calls_in_a_row_second_smaller():
    import paper_2110_15362_amd.bittrain as bt
    tile = bt.bt_tile_elems(torch.float32)
    _case(bt, 300 * tile + 1234, torch.float32, 0.5, 1)       # several scanner windows and a ragged tail
    _case(bt, 37 * tile + 5, torch.float32, 0.7, 2)           # smaller: what the first call left must not matter
    _case(bt, 3 * bt.bt_tile_elems(torch.bfloat16) + 77, torch.bfloat16, 0.3, 3)
    _case(bt, 1, torch.float32, 0.0, 4)


def test_size_limit_and_empty():
    import paper_2110_15362_amd.bittrain as bt
    L = bt.lib()
    code = bt.dtype_code(torch.float32)
    too_many = (16384 + 1) * bt.bt_tile_elems(torch.float32)
    # refused on the host before any pointer is looked at
    assert L.bt_compress_static(None, too_many, code, None, None, 0, None, None) == 6      # BT_ERR_SIZE
    nnz = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    x = torch.empty(0, dtype=torch.float32, device="cuda")
    bt.bt_compress_static(x, torch.empty(0, dtype=torch.int32, device="cuda"), x.clone(), nnz)
    torch.cuda.synchronize()
    assert int(nnz.item()) == 0
