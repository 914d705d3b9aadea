"""Property tests of the CPU oracle (hypothesis): invariants of the format that hold for every
input, on arrays hypothesis makes up and shrinks.  They complement the pins: a pin fixes a value,
a property fixes a relation."""
import numpy as np
from hypothesis import given, settings, strategies as st
from hypothesis.extra import numpy as hnp

WIDTHS = {2: np.uint16, 4: np.uint32, 8: np.uint64}


def _arrays(width):
    dt = WIDTHS[width]
    # mostly zeros and small numbers, so that zero runs, single survivors and full words all occur
    elems = st.one_of(st.just(0), st.just(0), st.integers(0, 3), st.integers(0, np.iinfo(dt).max))
    return hnp.arrays(dt, st.integers(0, 300), elements=elems)


@settings(max_examples=150, deadline=None)
@given(st.sampled_from([2, 4, 8]).flatmap(_arrays))
def test_round_trip_and_counts(oracle, x):
    n = x.size
    bitmap, values, nnz = oracle.compress(x)
    assert nnz == int(np.count_nonzero(x)) == values.size
    assert bitmap.size == (n + 31) // 32
    assert sum(bin(int(w)).count("1") for w in bitmap) == nnz                # popcount(bitmap) == nnz, tail bits are 0
    assert np.array_equal(values, x[x != 0])                                 # index order
    assert np.array_equal(oracle.decompress(bitmap, values, n), x)           # Algorithm 2 undoes Algorithm 1
    assert oracle.compressed_size(n, nnz, x.itemsize) == 4 * bitmap.size + values.nbytes
    # compressing again what was restored changes nothing
    b2, v2, k2 = oracle.compress(oracle.decompress(bitmap, values, n))
    assert k2 == nnz and np.array_equal(b2, bitmap) and np.array_equal(v2, values)


@settings(max_examples=100, deadline=None)
@given(st.sampled_from([2, 4, 8]).flatmap(lambda w: st.tuples(_arrays(w), st.integers(0, 2**32 - 1))))
def test_mask_select_and_concatenation(oracle, xs):
    x, seed = xs
    n = x.size
    bitmap, values, nnz = oracle.compress(x)
    g = np.random.default_rng(seed).integers(1, 1000, size=n).astype(x.dtype)
    # the ReLU-backward / double-mask select keeps exactly the positions of the non-zeros
    out = oracle.relu_backward(bitmap, g)
    assert np.array_equal(out != 0, x != 0) and np.array_equal(out[x != 0], g[x != 0])
    assert np.array_equal(oracle.mask_apply(bitmap, g), out)
    # Algorithm 1 on a concatenation at a word boundary is the concatenation of the parts
    cut = (n // 64) * 32
    ba, va, ka = oracle.compress(x[:cut])
    bb, vb, kb = oracle.compress(x[cut:])
    assert ka + kb == nnz and np.array_equal(np.concatenate([ba, bb]), bitmap) and np.array_equal(np.concatenate([va, vb]), values)
    # and the tile index is the running total at the cut
    if cut:
        assert oracle.tile_index(bitmap, n, cut)[1:2].tolist() == ([ka] if n > cut else [])


@settings(max_examples=100, deadline=None)
@given(hnp.arrays(np.float32, st.integers(0, 200), elements=st.floats(-2, 2, width=32)),
       st.sampled_from([0.0, 0.01, 0.05, 0.1, -1.0]))
def test_pruning_is_monotone_and_idempotent(oracle, x, thr):
    bits = x.view(np.uint32)
    kept = oracle.prune(bits, "f32", thr)
    assert np.array_equal(oracle.prune(kept, "f32", thr) if thr >= 0 else kept, kept)       # pruning twice changes nothing
    higher = oracle.prune(bits, "f32", thr + 0.5)
    assert np.all((higher != 0) <= (kept != 0) | (bits == 0))                # a higher threshold keeps a subset
    assert np.array_equal(kept.view(np.float32)[kept != 0].astype(np.float64) > thr, np.ones(int((kept != 0).sum()), dtype=bool))
