"""The codec inside a PyTorch graph (GPU): because the round trip is bit-exact, gradients
with compressed saved activations are identical to those of the plain graph."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ag():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2110_15362_amd import autograd
    return autograd


def _mlp(seed, dtype):
    g = torch.Generator().manual_seed(seed)
    w1 = (torch.randn(1024, 512, generator=g) * 0.05).to(dtype).cuda().requires_grad_()
    w2 = (torch.randn(768, 1024, generator=g) * 0.05).to(dtype).cuda().requires_grad_()
    w3 = (torch.randn(64, 768, generator=g) * 0.05).to(dtype).cuda().requires_grad_()
    x = torch.randn(2048, 512, generator=g).to(dtype).cuda().requires_grad_()
    return x, (w1, w2, w3)


def _forward(x, ws, relu):
    h = relu(torch.nn.functional.linear(x, ws[0]))
    h = relu(torch.nn.functional.linear(h, ws[1]))
    return torch.nn.functional.linear(h, ws[2]).float().pow(2).mean()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_saved_tensor_hooks_give_identical_gradients(ag, dtype):
    x, ws = _mlp(1, dtype)
    _forward(x, ws, torch.relu).backward()
    ref = [t.grad.clone() for t in (x,) + ws]
    for t in (x,) + ws:
        t.grad = None
    stash = ag.BitmapStash(min_numel=1024)
    with stash:
        loss = _forward(x, ws, torch.relu)
    loss.backward()
    for r, t in zip(ref, (x,) + ws):
        assert torch.equal(r, t.grad)
    # the two ReLU outputs (about half zeros) were compressed; the dense input was not worth it
    assert stash.stats["compressed"] >= 2
    assert stash.stats["stored_bytes"] < 0.8 * stash.stats["dense_bytes"]


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_bitmap_relu_backward_matches_torch(ag, dtype, fused):
    x, ws = _mlp(2, dtype)
    ref_loss = _forward(x, ws, torch.relu)
    ref_loss.backward()
    ref = [t.grad.clone() for t in (x,) + ws]
    for t in (x,) + ws:
        t.grad = None
    loss = _forward(x, ws, lambda t: ag.bitmap_relu(t, fused=fused))
    loss.backward()
    assert torch.equal(loss, ref_loss)
    for r, t in zip(ref, (x,) + ws):
        assert torch.equal(r, t.grad)


def _relu_mlp_step(ag, stash, layers, batch, hidden, seed=0, deferred=False):
    """Forward and backward of y = relu(... relu(x W_0) ... W_{L-1}), sum as loss.  Returns the gradients, the
    peak of allocated device memory above what was allocated before the step, and the stash's counters."""
    import contextlib
    g = torch.Generator(device="cuda").manual_seed(seed)
    ws = [(torch.randn(hidden, hidden, device="cuda", generator=g) / hidden ** 0.5).requires_grad_() for _ in range(layers)]
    x = torch.randn(batch, hidden, device="cuda", generator=g)
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    before = torch.cuda.memory_allocated()
    ctx = ag.BitmapStash(deferred=deferred) if stash else contextlib.nullcontext()
    with ctx:
        y = x
        for w in ws:
            y = ag.bitmap_relu(y @ w) if stash else torch.relu(y @ w)
        loss = y.sum()
    loss.backward()
    torch.cuda.synchronize()
    peak = torch.cuda.max_memory_allocated() - before
    return [w.grad for w in ws], peak, (ctx.stats if stash else None)


def test_stash_lowers_peak_memory_of_a_step(ag):
    """16 layers whose saved activations are 32 MiB each (512 MiB dense, about half of the elements zero): with the
    stash the step's peak of allocated memory is clearly lower, and the gradients are the same bits."""
    layers, batch, hidden = 16, 8192, 1024
    grads_off, peak_off, _ = _relu_mlp_step(ag, False, layers, batch, hidden)
    grads_on, peak_on, stats = _relu_mlp_step(ag, True, layers, batch, hidden)
    assert stats["dense_bytes"] >= 100 * 1000 * 1000 and stats["compressed"] >= layers - 1 and stats["failed"] == 0
    assert stats["stored_bytes"] < 0.65 * stats["dense_bytes"]
    assert peak_on < 0.85 * peak_off, (peak_on, peak_off)
    for a, b in zip(grads_on, grads_off):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    print("peak MiB without / with the stash: %.0f / %.0f; stored %.0f of %.0f MiB" % (
        peak_off / 2**20, peak_on / 2**20, stats["stored_bytes"] / 2**20, stats["dense_bytes"] / 2**20))


def test_deferred_stash_gives_the_same_gradients_without_waiting_for_the_device(ag):
    layers, batch, hidden = 8, 4096, 1024
    grads_off, peak_off, _ = _relu_mlp_step(ag, False, layers, batch, hidden, seed=3)
    grads_on, peak_on, stats = _relu_mlp_step(ag, True, layers, batch, hidden, seed=3, deferred=True)
    assert stats["tensors"] >= layers and stats["compressed"] >= layers - 1 and stats["failed"] == 0
    assert stats["stored_bytes"] < 0.75 * stats["dense_bytes"]        # (the dense input and the weights pass through too)
    for a, b in zip(grads_on, grads_off):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
