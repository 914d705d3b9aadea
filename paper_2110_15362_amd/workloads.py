"""Seeded synthetic activation tensors for the bitmap codec.

This module only draws random numbers and zeroes some of them; it holds none of
the codec's arithmetic (no bitmap, no prefix sum, no compaction) and imports
neither the GPU library nor the CPU oracle, so both can be fed the same bytes.

The shapes are ResNet convolution activations as in Table 1 of the paper with
the batch dimension scaled up, the sparsity levels are the paper's (about 50 %
zeros after ReLU, 70 % and more after pruning near-zero activations, Section
4.3), and the pre-activation distribution is a unit Gaussian.  They stand in
for the ImageNet / CIFAR-10 activations the paper measured, which need datasets
and trained weights.  Everything is drawn on the host with
``torch.Generator().manual_seed(seed)`` in fp32, zeroed in fp32, then cast
(round to nearest even) to the target dtype.
"""
import numpy as np
import torch

# Two-sided Gaussian quantiles: P(|x| < t) = z for z = 0.5, 0.7, 0.9.
_T_ABS = {0.5: 0.6744897501960817, 0.7: 1.0364333894937898, 0.9: 1.6448536269514722}
# One-sided: P(x < t) = 0.7.
_T_70 = 0.5244005127080407

DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "f64": torch.float64}
_BITS = {torch.float32: torch.int32, torch.float16: torch.int16, torch.bfloat16: torch.int16,
         torch.float64: torch.int64}
_NP_BITS = {4: np.uint32, 2: np.uint16, 8: np.uint64}


def bits(t):
    """Flat numpy view of a CPU tensor's raw element bits (uint16/uint32/uint64)."""
    t = t.detach().contiguous().reshape(-1)
    a = t.view(_BITS[t.dtype]).numpy()
    return a.view(_NP_BITS[a.dtype.itemsize])


def _gen(seed):
    return torch.Generator(device="cpu").manual_seed(seed)


def _scaled(shape, batch):
    return (batch,) + tuple(shape[1:]) if batch is not None else tuple(shape)


def config1(batch=None):
    """fp32 [1,64,56,56]: x = ReLU(N(0,1)) (about half zeros), grad ~ N(0,1); seed 0."""
    g = _gen(0)
    shape = _scaled((1, 64, 56, 56), batch)
    x = torch.relu(torch.randn(shape, generator=g))
    grad = torch.randn(shape, generator=g)
    return {"name": "c1_f32_1x64x56x56", "x": x, "grad": grad}


def config2(sparsity, batch=None, base=None):
    """fp32 [32,256,56,56]: x ~ N(0,1) zeroed where |x| < t, t set for 50/70/90 %
    zeros at i.i.d. positions; one base draw (seed 1) serves the three levels."""
    shape = _scaled((32, 256, 56, 56), batch)
    if base is None:
        base = torch.randn(shape, generator=_gen(1))
    x = base.clone()
    x[x.abs() < _T_ABS[sparsity]] = 0.0
    return {"name": "c2_f32_32x256x56x56_z%d" % round(100 * sparsity), "x": x, "base": base}


def config3(variant="a", batch=None):
    """bf16 [8,2048,4096] post-ReLU MLP activation with 30 % dead units (seed 3).

    Variant "a": dead units are feature columns (last axis), so every row has
    the same comb of empty positions.  Variant "b": dead units are on axis 1, so
    whole 4096-element rows are empty, which is what unbalances the scan.
    """
    g = _gen(3)
    shape = _scaled((8, 2048, 4096), batch)
    axis_len = shape[2] if variant == "a" else shape[1]
    perm = torch.randperm(axis_len, generator=g)
    dead = perm[: round(0.3 * axis_len)]
    x = torch.relu(torch.randn(shape, generator=g))
    if variant == "a":
        x[:, :, dead] = 0.0
    else:
        x[:, dead, :] = 0.0
    return {"name": "c3%s_bf16_8x2048x4096" % variant, "x": x.to(torch.bfloat16)}


def config4_shapes(batch=64):
    """The 49 post-ReLU activation shapes of a bottleneck ResNet-50 (stride on
    the 3x3 convolution), in forward order: stem, then 3+4+6+3 blocks of three."""
    shapes = [(batch, 64, 112, 112)]
    hw, planes_list, blocks = 56, (64, 128, 256, 512), (3, 4, 6, 3)
    for stage, (planes, nblk) in enumerate(zip(planes_list, blocks)):
        for b in range(nblk):
            in_hw = hw
            if stage > 0 and b == 0:
                hw //= 2  # the 3x3 convolution of the first block strides
            shapes.append((batch, planes, in_hw, in_hw))        # after conv1 (1x1)
            shapes.append((batch, planes, hw, hw))              # after conv2 (3x3)
            shapes.append((batch, 4 * planes, hw, hw))          # after the residual add
    return shapes


def config4_tensors(batch=64):
    """Yield the ResNet-50 activation set, fp32: ReLU(N(0,1)) pruned to 70 % zeros;
    one generator (seed 4), tensors drawn in forward order."""
    g = _gen(4)
    for k, shape in enumerate(config4_shapes(batch)):
        x = torch.relu(torch.randn(shape, generator=g))
        x[x < _T_70] = 0.0
        yield {"name": "c4_f32_%02d_%s" % (k, "x".join(map(str, shape))), "x": x}


def config5(zero_prob, batch=None, draws=None):
    """fp16 [256,64,112,112]: x ~ N(0,1) zeroed where u < p for one uniform draw u
    (seed 2); p = 0.05 (the compressed form is larger than the dense one) and
    p = 0.95 (tiny value array).  ``draws`` lets two levels share (x, u)."""
    shape = _scaled((256, 64, 112, 112), batch)
    if draws is None:
        g = _gen(2)
        draws = (torch.randn(shape, generator=g), torch.rand(shape, generator=g))
    base, u = draws
    x = base.clone()
    x[u < zero_prob] = 0.0
    return {"name": "c5_f16_256x64x112x112_z%d" % round(100 * zero_prob),
            "x": x.to(torch.float16), "draws": draws}


def random_sparse(n, dtype, zero_frac, seed):
    """Flat tensor of n elements, i.i.d. zeros with probability zero_frac."""
    g = _gen(seed)
    dt = DTYPES[dtype] if isinstance(dtype, str) else dtype
    # doubles are drawn as doubles, so that all 64 bits of an element vary
    x = torch.randn(n, generator=g, dtype=torch.float64 if dt == torch.float64 else torch.float32)
    u = torch.rand(n, generator=g)
    x[u < zero_frac] = 0.0
    return x.to(dt)


def special_values(dtype):
    """A short tensor of the awkward bit patterns: +0, -0, smallest denormal, NaNs
    with payloads, infinities, largest finite, interleaved with zeros."""
    dt = DTYPES[dtype] if isinstance(dtype, str) else dtype
    if dt == torch.float64:
        pats = [0x0000000000000000, 0x8000000000000000, 0x0000000000000001, 0x8000000000000001,
                0x7FF8000000000000, 0xFFF8000000000001, 0x7FF0000000000001, 0x7FF0000000000000,
                0xFFF0000000000000, 0x7FEFFFFFFFFFFFFF, 0x0000000000000000, 0x3FF0000000000000,
                0x0000000000000000, 0x0000000000000000, 0xBFF0000000000000, 0x0000000100000000]
        a = np.array(pats, dtype=np.uint64).view(np.int64)
        return torch.from_numpy(a.copy()).view(torch.float64)
    if dt == torch.float32:
        pats = [0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x7FC00000, 0xFFC00001,
                0x7F800001, 0x7F800000, 0xFF800000, 0x7F7FFFFF, 0x00000000, 0x3F800000,
                0x00000000, 0x00000000, 0xBF800000, 0x00800000]
        a = np.array(pats, dtype=np.uint32).view(np.int32)
        return torch.from_numpy(a.copy()).view(torch.float32)
    if dt == torch.float16:
        pats = [0x0000, 0x8000, 0x0001, 0x8001, 0x7E00, 0xFE01, 0x7C01, 0x7C00, 0xFC00, 0x7BFF,
                0x0000, 0x3C00, 0x0000, 0x0000, 0xBC00, 0x0400]
    else:  # bfloat16
        pats = [0x0000, 0x8000, 0x0001, 0x8001, 0x7FC0, 0xFFC1, 0x7F81, 0x7F80, 0xFF80, 0x7F7F,
                0x0000, 0x3F80, 0x0000, 0x0000, 0xBF80, 0x0080]
    a = np.array(pats, dtype=np.uint16).view(np.int16)
    return torch.from_numpy(a.copy()).view(dt)
