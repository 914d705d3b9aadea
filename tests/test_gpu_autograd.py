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
