"""The library's calls under HIP graph capture: a captured compress -> decompress ->
ReLU-backward sequence is replayed several times, with eager work and synchronisations
between the replays, and every replay is checked against the CPU oracle.  The calls keep
their state (which copy of the workspace entries is in use) in device memory, so a replay
must behave exactly like an eager call, also when eager calls on the same workspace come
in between."""
import numpy as np
import pytest
import torch

from paper_2110_15362_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bt():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (they never fall back to the CPU)")
    import paper_2110_15362_amd.bittrain as b
    b.lib()
    return b


@pytest.mark.parametrize("dt,n", [("f32", 200704), ("bf16", 3 * 16384 + 77), ("f32", 70 * 8192 + 5)])
def test_captured_sequence_replays_like_eager_calls(bt, oracle, dt, n):
    dev = "cuda"
    inputs = [wl.random_sparse(n, dt, z, seed=4000 + k) for k, z in enumerate((0.5, 0.9, 0.0, 0.7, 1.0, 0.3))]
    grads = [torch.randn(n, generator=torch.Generator().manual_seed(4100 + k)).to(inputs[0].dtype) for k in range(6)]
    x = torch.empty(n, dtype=inputs[0].dtype, device=dev)
    g = torch.empty_like(x)
    words = (n + 31) // 32
    bitmap = torch.empty(words, dtype=torch.int32, device=dev)
    values = torch.empty(n, dtype=x.dtype, device=dev)
    out = torch.empty_like(x)
    gin = torch.empty_like(x)
    nnz = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = bt.new_workspace(n, x.dtype)

    def sequence():
        bt.bt_compress(x, bitmap, values, nnz, ws)
        bt.bt_decompress(bitmap, values, out, ws)
        bt.bt_relu_backward_from_bitmap(bitmap, g, gin)

    # warm up on a side stream, then capture (the binding launches on torch's current stream)
    x.copy_(inputs[0]); g.copy_(grads[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sequence()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence()

    def check(k):
        torch.cuda.synchronize()
        o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(inputs[k]))
        assert int(nnz.item()) == o_nnz, k
        assert np.array_equal(bitmap.cpu().numpy().view(np.uint32), o_bitmap), k
        assert np.array_equal(wl.bits(values[:o_nnz].cpu()), o_values), k
        assert np.array_equal(wl.bits(out.cpu()), wl.bits(inputs[k])), k
        assert np.array_equal(wl.bits(gin.cpu()), oracle.relu_backward(o_bitmap, wl.bits(grads[k]))), k

    for k in range(len(inputs)):
        x.copy_(inputs[k]); g.copy_(grads[k])
        values.fill_(7); out.fill_(7); gin.fill_(7); bitmap.fill_(-1); nnz.fill_(-1)
        if k % 3 == 2:
            sequence()                       # an eager call in between, on the same workspace
        else:
            graph.replay()
        check(k)
        if k % 2 == 1:
            # an odd number of eager calls between two replays flips which copy of the entries is in use
            bt.bt_compress(x, bitmap, values, nnz, ws)
            check(k)
    hdr = ws[:12].cpu().numpy().view(np.uint32)
    assert hdr[2] == 0, "a bounded wait ran out"


def test_captured_batched_calls_replay(bt, oracle):
    dev = "cuda"
    ns = [5, 8192 * 3 + 1, 0, 8192 * 70, 100]
    sets = [[wl.random_sparse(n, "f32", 0.2 + 0.15 * i, seed=4200 + 10 * r + i) for i, n in enumerate(ns)] for r in range(4)]
    xs = [torch.empty(n, device=dev) for n in ns]
    bms = [torch.empty((n + 31) // 32, dtype=torch.int32, device=dev) for n in ns]
    vals = [torch.empty(max(n, 1), device=dev) for n in ns]
    outs = [torch.empty(n, device=dev) for n in ns]
    nnz = torch.zeros(len(ns), dtype=torch.int64, device=dev)
    ws = bt.new_batch_workspace(ns, torch.float32)
    c_items = bt.compress_items(xs, bms, vals, nnz)
    d_items = bt.decompress_items(bms, vals, outs)

    def sequence():
        bt.bt_compress_batch(c_items, len(ns), torch.float32, ws)
        bt.bt_decompress_batch(d_items, len(ns), torch.float32, ws)

    for x, src in zip(xs, sets[0]):
        x.copy_(src)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sequence()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence()
    for r in range(len(sets)):
        for x, src, o in zip(xs, sets[r], outs):
            x.copy_(src)
            o.fill_(3)
        nnz.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        for i, src in enumerate(sets[r]):
            o_bitmap, o_values, o_nnz = oracle.compress(wl.bits(src))
            assert int(nnz[i].item()) == o_nnz, (r, i)
            assert np.array_equal(bms[i].cpu().numpy().view(np.uint32), o_bitmap), (r, i)
            assert np.array_equal(wl.bits(vals[i][:o_nnz].cpu()), o_values), (r, i)
            assert np.array_equal(wl.bits(outs[i].cpu()), wl.bits(src)), (r, i)
