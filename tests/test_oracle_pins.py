"""Pins for the CPU oracle: each test checks oracle/bt_oracle.c against something
other than itself -- numbers the paper prints, closed forms, library routines of
numpy (bit packing, boolean selection) and brute-force enumeration.  A dropped term, a wrong bit order, a reversed value order,
an off-by-one at a word boundary or an IEEE (instead of bit-pattern) zero test
each fail at least one of them."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_theoretical.txt")


def _table1():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        b, c, w, h, n, pct, dense, bitmap, improv = line.split()
        rows.append((int(b), int(c), int(w), int(h), int(n), int(pct), float(dense), float(bitmap),
                     float(improv)))
    return rows


def test_table1_has_30_rows():
    rows = _table1()
    assert len(rows) == 30
    for b, c, w, h, n, *_ in rows:
        assert b * c * w * h == n


@pytest.mark.parametrize("row", _table1(), ids=lambda r: "%dx%dx%dx%d_nz%d" % (r[0], r[1], r[2], r[3], r[5]))
def test_size_reproduces_table1(oracle, row):
    """Table 1, theoretical columns: dense MB, bitmap MB and improvement %, fp32.
    The paper prints two decimals, so agreement is to half a unit of the last one."""
    b, c, w, h, n, pct, dense_mb, bitmap_mb, improv = row
    nnz = n * pct // 100
    md = oracle.dense_size(n, 4)
    mb = oracle.compressed_size(n, nnz, 4)
    assert abs(md / 2**20 - dense_mb) <= 0.005 + 1e-9
    assert abs(mb / 2**20 - bitmap_mb) <= 0.005 + 1e-9
    assert abs(100.0 * (1.0 - mb / md) - improv) <= 0.005 + 1e-9


def test_size_formula_section_3_2(oracle):
    """M_d = 4 * total and M_b = 4 * nnz + total / 8 for fp32 whenever 32 | total."""
    for n in (32, 64, 3211264, 25690112):
        for nnz in (0, 1, n // 4, n // 2, n):
            assert oracle.dense_size(n, 4) == 4 * n
            assert oracle.compressed_size(n, nnz, 4) == 4 * nnz + n // 8
            assert oracle.compressed_size(n, nnz, 2) == 2 * nnz + n // 8


def test_size_closed_forms_and_rounding(oracle):
    # all-zero tensor: only the bitmap; all-non-zero: expansion by 1/(8*width)
    n = 25690112
    assert oracle.compressed_size(n, 0, 4) * 32 == oracle.dense_size(n, 4)
    assert oracle.compressed_size(n, n, 4) * 32 == 33 * oracle.dense_size(n, 4)
    assert oracle.compressed_size(n, n, 2) * 16 == 17 * oracle.dense_size(n, 2)
    # bitmap is rounded up to whole 32-bit words
    assert [oracle.compressed_size(k, 0, 4) for k in (0, 1, 31, 32, 33, 64, 65)] == [0, 4, 4, 4, 8, 8, 12]
    # nonsense arguments
    assert oracle.compressed_size(10, 11, 4) == 0
    assert oracle.compressed_size(10, 1, 3) == 0
    # one more value moves the size by exactly one element, one more element by a word every 32
    assert oracle.compressed_size(77, 14, 2) - oracle.compressed_size(77, 13, 2) == 2
    assert oracle.compressed_size(1000, 1000, 8) == 4 * 32 + 8000


def test_hand_built_tensor(oracle):
    """A 40-element tensor written out by hand: non-zeros at 1, 2, 5, 31, 32, 39."""
    x = np.zeros(40, dtype=np.float32)
    x[1], x[2], x[5], x[31], x[32], x[39] = 1.0, -2.0, 3.5, 4.0, -5.0, 6.0
    bitmap, values, nnz = oracle.compress(x)
    assert nnz == 6
    assert bitmap.tolist() == [(1 << 1) | (1 << 2) | (1 << 5) | (1 << 31), (1 << 0) | (1 << 7)]
    assert values.tolist() == [1.0, -2.0, 3.5, 4.0, -5.0, 6.0]
    back = oracle.decompress(bitmap, values, 40)
    assert back.view(np.uint32).tolist() == x.view(np.uint32).tolist()
    # bitmap bytes in memory are little-endian: elements 1, 2, 5 live in byte 0, elements 32 and 39 in byte 4
    assert bitmap.view(np.uint8)[:5].tolist() == [0b00100110, 0, 0, 0x80, 0x81]


def test_zero_is_the_bit_pattern(oracle):
    """-0.0, denormals, NaN payloads and infinities are values; only all-zero bits are dropped."""
    pats = np.array([0x80000000, 0, 0x00000001, 0x7FC00123, 0, 0xFF800000, 0, 0x80000000], dtype=np.uint32)
    bitmap, values, nnz = oracle.compress(pats.view(np.float32))
    assert nnz == 5
    assert bitmap.tolist() == [0b10101101]
    assert values.view(np.uint32).tolist() == [0x80000000, 0x00000001, 0x7FC00123, 0xFF800000, 0x80000000]
    back = oracle.decompress(bitmap, values, 8)
    assert back.view(np.uint32).tolist() == pats.tolist()
    h = np.array([0x8000, 0x0000, 0x7E01, 0x0001], dtype=np.uint16)
    bitmap, values, nnz = oracle.compress(h)
    assert (nnz, bitmap.tolist(), values.tolist()) == (3, [0b1101], [0x8000, 0x7E01, 0x0001])


@pytest.mark.parametrize("npdt", [np.uint16, np.uint32, np.uint64])
def test_against_numpy_library_routines(oracle, npdt):
    """bitmap == numpy.packbits(little) as uint32; values == boolean indexing;
    decompress == zeros with values scattered at the mask; relu == numpy.where."""
    rng = np.random.default_rng(7)
    for n in (1, 31, 32, 33, 1000, 4096, 70001):
        for zf in (0.0, 0.3, 0.9, 1.0):
            x = rng.integers(1, np.iinfo(npdt).max, size=n, dtype=npdt)
            x[rng.random(n) < zf] = 0
            mask = x != 0
            packed = np.packbits(mask, bitorder="little")
            packed = np.concatenate([packed, np.zeros((-packed.size) % 4, np.uint8)]).view("<u4")
            bitmap, values, nnz = oracle.compress(x)
            assert nnz == np.count_nonzero(x)
            assert np.array_equal(bitmap, packed)
            assert np.array_equal(values, x[mask])
            # popcount invariant and zero tail bits
            assert int(np.unpackbits(bitmap.view(np.uint8)).sum()) == nnz
            expect = np.zeros(n, npdt)
            expect[mask] = values
            assert np.array_equal(oracle.decompress(bitmap, values, n), expect)
            assert np.array_equal(oracle.decompress(bitmap, values, n), x)
            g = rng.integers(0, np.iinfo(npdt).max, size=n, dtype=npdt)
            assert np.array_equal(oracle.relu_backward(bitmap, g), np.where(mask, g, 0).astype(npdt))
            assert oracle.compressed_size(n, nnz, x.itemsize) == bitmap.nbytes + values.nbytes


@pytest.mark.parametrize("npdt", [np.uint16, np.uint32])
def test_all_2_to_16_zero_patterns(oracle, npdt):
    """Every zero pattern p of a 16-element tensor with a distinct payload per
    position: the bitmap word is p itself, the values are the payloads of the set
    bits in ascending position, and the round trip is exact."""
    payload = (np.arange(16, dtype=np.uint32) * 0x0111 + 0x8001).astype(npdt)
    assert len(set(payload.tolist())) == 16 and payload.min() > 0
    pos = np.arange(16)
    for p in range(1 << 16):
        sel = ((p >> pos) & 1).astype(bool)
        x = np.where(sel, payload, 0).astype(npdt)
        bitmap, values, nnz = oracle.compress(x)
        assert bitmap[0] == p and bitmap.size == 1
        assert nnz == bin(p).count("1")
        assert values.tolist() == payload[sel].tolist()
        if p % 97 == 0 or p > 65000:   # the decoder on a spread of patterns + the dense end
            assert oracle.decompress(bitmap, values, 16).tolist() == x.tolist()


def test_all_2_to_16_patterns_decode(oracle):
    """Decoder alone on every 16-bit pattern, fed hand-made (bitmap, values)."""
    payload = np.arange(1, 17, dtype=np.uint32) * 1000003
    pos = np.arange(16)
    for p in range(1 << 16):
        sel = ((p >> pos) & 1).astype(bool)
        out = oracle.decompress(np.array([p], np.uint32), payload[sel], 16)
        assert out.tolist() == np.where(sel, payload, 0).tolist()


def test_every_length_0_to_130_against_numpy_routines(oracle):
    """Word and tail boundaries: for every n in [0,130] the bitmap is numpy's little-endian bit packing of
    (x != 0), the values are numpy's boolean selection, restoration gives x back, and the backward is a select."""
    rng = np.random.default_rng(11)
    for n in range(0, 131):
        x = rng.integers(1, 2**32, size=n, dtype=np.uint32)
        x[rng.random(n) < 0.5] = 0
        bitmap, values, nnz = oracle.compress(x)
        assert bitmap.size == (n + 31) // 32
        packed = np.packbits(x != 0, bitorder="little")
        packed = np.concatenate([packed, np.zeros(4 * bitmap.size - packed.size, np.uint8)])
        assert bitmap.tolist() == packed.view("<u4").tolist()
        assert values.tolist() == x[x != 0].tolist() and nnz == int(np.count_nonzero(x))
        assert oracle.decompress(bitmap, values, n).tolist() == x.tolist()
        g = rng.integers(0, 2**32, size=n, dtype=np.uint32)
        assert oracle.relu_backward(bitmap, g).tolist() == np.where(x != 0, g, 0).tolist()
        if n % 32:
            assert int(bitmap[-1]) >> (n % 32) == 0      # unused high bits stay clear


def test_relu_backward_special_cases(oracle):
    n = 100
    g = np.arange(1, n + 1, dtype=np.float32)
    ones = np.array([0xFFFFFFFF] * 3 + [0xF], dtype=np.uint32)
    assert np.array_equal(oracle.relu_backward(ones, g), g)                       # identity
    assert not oracle.relu_backward(np.zeros(4, np.uint32), g).view(np.uint32).any()  # all blocked
    # select, not multiply: NaN / Inf / -1 under a cleared bit give +0 (bits 0), not NaN or -0
    bad = np.array([np.nan, np.inf, -1.0, 5.0], dtype=np.float32)
    out = oracle.relu_backward(np.array([0b1000], np.uint32), bad)
    assert out.view(np.uint32).tolist() == [0, 0, 0, np.float32(5.0).view(np.uint32)]
    # it is the ReLU derivative: for y = relu(x), bit set <=> x > 0
    rng = np.random.default_rng(3)
    x = rng.standard_normal(1000).astype(np.float32)
    go = rng.standard_normal(1000).astype(np.float32)
    bitmap, _, _ = oracle.compress(np.maximum(x, 0))
    assert np.array_equal(oracle.relu_backward(bitmap, go), np.where(x > 0, go, np.float32(0)))


def test_degenerate_inputs(oracle):
    e = np.zeros(0, np.float32)
    bitmap, values, nnz = oracle.compress(e)
    assert (bitmap.size, values.size, nnz) == (0, 0, 0)
    assert oracle.decompress(bitmap, values, 0).size == 0
    z = np.zeros(1000, np.float32)
    bitmap, values, nnz = oracle.compress(z)
    assert nnz == 0 and not bitmap.any() and bitmap.size == 32
    assert not oracle.decompress(bitmap, values, 1000).view(np.uint32).any()
    f = np.full(1000, 2.5, np.float32)
    bitmap, values, nnz = oracle.compress(f)
    assert nnz == 1000 and np.array_equal(values, f)
    assert bitmap.tolist() == [0xFFFFFFFF] * 31 + [0xFF]
    one = np.zeros(1000, np.float32)
    one[999] = 1.0
    bitmap, values, nnz = oracle.compress(one)
    assert nnz == 1 and bitmap[31] == 1 << 7 and not bitmap[:31].any()


def test_workload_recipes_round_trip(oracle):
    """Scaled-down versions of the benchmark configurations: round trip exact,
    invariants hold, sparsity is what the recipe says."""
    from paper_2110_15362_amd import workloads as wl
    c1 = wl.config1()
    cases = [(c1["x"], 0.5), (wl.config2(0.5, batch=1)["x"], 0.5), (wl.config2(0.7, batch=1)["x"], 0.7),
             (wl.config2(0.9, batch=1)["x"], 0.9), (wl.config3("a", batch=1)["x"], 0.65),
             (wl.config3("b", batch=1)["x"], 0.65), (wl.config5(0.05, batch=1)["x"], 0.05),
             (wl.config5(0.95, batch=1)["x"], 0.95), (next(iter(wl.config4_tensors(batch=1)))["x"], 0.7)]
    for x, z in cases:
        xb = wl.bits(x)
        bitmap, values, nnz = oracle.compress(xb)
        assert abs((1 - nnz / xb.size) - z) < 0.01
        assert nnz == np.count_nonzero(xb)
        assert np.array_equal(oracle.decompress(bitmap, values, xb.size), xb)
        assert oracle.compressed_size(xb.size, nnz, xb.itemsize) == bitmap.nbytes + values.nbytes
    for dt in ("f32", "f16", "bf16"):
        xb = wl.bits(wl.special_values(dt))
        bitmap, values, nnz = oracle.compress(xb)
        assert nnz == 12 and bitmap.tolist() == [0b1100101111111110]
        assert np.array_equal(oracle.decompress(bitmap, values, 16), xb)


# ---- activation pruning (Section 4.3) -----------------------------------------------------


def _f16_bits_to_f32(bits):
    return bits.view(np.float16).astype(np.float32)


def _bf16_bits_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("thr", [0.0, 1e-6, 0.01, 0.05, 0.1, -2.0, float("inf")])
def test_prune_every_16_bit_pattern(oracle, thr):
    """All 65536 half and bfloat16 patterns: kept exactly where numpy's widened value, as a double,
    exceeds the threshold; NaNs (for which no comparison holds) are dropped."""
    allbits = np.arange(65536, dtype=np.uint16)
    with np.errstate(invalid="ignore"):
        for dt, widen in (("f16", _f16_bits_to_f32), ("bf16", _bf16_bits_to_f32)):
            expect = np.where(widen(allbits).astype(np.float64) > thr, allbits, 0).astype(np.uint16)
            assert np.array_equal(oracle.prune(allbits, dt, thr), expect)


def test_prune_fp32_special_values(oracle):
    f = np.array([0.0, -0.0, 1e-45, -1e-45, 0.01, 0.0100001, -0.5, np.inf, -np.inf, np.nan, 0.1, 3.0], dtype=np.float32)
    bits = f.view(np.uint32)
    kept0 = oracle.prune(bits, "f32", 0.0).view(np.float32)
    assert kept0.view(np.uint32).tolist() == np.array([0, 0, 1e-45, 0, 0.01, 0.0100001, 0, np.inf, 0, 0, 0.1, 3.0], np.float32).view(np.uint32).tolist()
    kept = oracle.prune(bits, "f32", 0.01).view(np.float32)     # the single nearest 0.01 lies below it: pruned
    assert kept.view(np.uint32).tolist() == np.array([0, 0, 0, 0, 0, 0.0100001, 0, np.inf, 0, 0, 0.1, 3.0], np.float32).view(np.uint32).tolist()
    assert not oracle.prune(bits, "f32", float("nan")).any()    # nothing exceeds NaN
    everything = oracle.prune(bits, "f32", float("-inf")).view(np.uint32)
    assert everything.tolist() == np.where(np.isnan(f) | np.isneginf(f), 0, bits).tolist()


def test_prune_with_threshold_zero_is_relu(oracle):
    """Section 4.3 with threshold 0 on a pre-activation tensor: pruning then Algorithm 1
    equals Algorithm 1 on ReLU(x), and decompressing gives ReLU(x)."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal(50000).astype(np.float32)
    relu = np.maximum(x, np.float32(0))
    b1, v1, n1 = oracle.compress_pruned(x.view(np.uint32), "f32", 0.0)
    b2, v2, n2 = oracle.compress(relu.view(np.uint32))
    assert n1 == n2 and np.array_equal(b1, b2) and np.array_equal(v1, v2)
    assert np.array_equal(oracle.decompress(b1, v1, x.size).view(np.float32), relu)
    # thresholds of the paper raise the sparsity monotonically
    kept = [oracle.compress_pruned(x.view(np.uint32), "f32", t)[2] for t in (0.0, 0.01, 0.05, 0.1)]
    assert kept == sorted(kept, reverse=True) and kept[0] > kept[-1]
    for t, k in zip((0.0, 0.01, 0.05, 0.1), kept):
        assert k == int((x > np.float32(t)).sum())


# ---- the COO comparison format (Section 3.2) and the double mask (Section 3.1) ----

def test_coo_size_formula_and_the_papers_break_even(oracle):
    """M_c = (4 + [4|8] * dimensions) * non-zeros for fp32.  The paper's reading of its
    footprint figure: COO only pays off at 80 % sparsity or more (about 20 % non-zeros),
    which is the break-even against the dense format of a 4-D activation with 4-byte
    indices, (4 + 16) * nnz = 4 * n."""
    n = 5 * 9 * 128 * 1000                                    # divisible by every break-even ratio below
    assert oracle.coo_size(1, 4, 4, 4) == 20 and oracle.coo_size(1, 4, 8, 4) == 36
    assert oracle.coo_size(7, 2, 8, 2) == 7 * (2 + 16)
    assert oracle.coo_size(n // 5, 4, 4, 4) == oracle.dense_size(n, 4)            # exactly 20 % non-zeros
    assert oracle.coo_size(n // 5 - 1, 4, 4, 4) < oracle.dense_size(n, 4) < oracle.coo_size(n // 5 + 1, 4, 4, 4)
    # long indices (the frameworks' default) move the break-even down to 1/9 non-zeros
    assert oracle.coo_size(n // 9, 4, 8, 4) == oracle.dense_size(n, 4) < oracle.coo_size(n // 9 + 1, 4, 8, 4)
    # the bitmap format beats dense up to 31/32 non-zeros (Table 1: -3.13 % at 100 %, +21.88 % at 75 %) ...
    assert oracle.compressed_size(n, n * 31 // 32, 4) == oracle.dense_size(n, 4)
    # ... and beats COO (4-byte indices, 4-D) as soon as more than 1/128 of the elements are non-zero:
    # 4 nnz + n/8 < 20 nnz  <=>  nnz > n/128
    assert oracle.compressed_size(n, n // 128, 4) == oracle.coo_size(n // 128, 4, 4, 4)
    assert oracle.compressed_size(n, n // 128 + 1, 4) < oracle.coo_size(n // 128 + 1, 4, 4, 4)
    # nonsense arguments
    assert oracle.coo_size(5, 0, 4, 4) == 0 and oracle.coo_size(5, 4, 2, 4) == 0 and oracle.coo_size(5, 4, 4, 3) == 0


@pytest.mark.parametrize("npdt", [np.uint16, np.uint32, np.uint64])
def test_mask_apply_is_a_select_by_another_tensors_bitmap(oracle, npdt):
    rng = np.random.default_rng(77)
    for n in (0, 1, 31, 32, 33, 100, 1000):
        x = rng.integers(1, 2**16, size=n).astype(npdt)                   # the masked tensor: no zeros
        src = rng.integers(0, 2**16, size=n).astype(npdt) * (rng.random(n) < 0.4)   # the tensor that gives the pattern
        bitmap, _, nnz = oracle.compress(src)
        out = oracle.mask_apply(bitmap, x)
        assert np.array_equal(out, np.where(src != 0, x, 0).astype(npdt))
        # the point of the double mask: the output has exactly the input's sparsity pattern
        out_bitmap, out_values, out_nnz = oracle.compress(out)
        assert np.array_equal(out_bitmap, bitmap) and out_nnz == nnz
        assert np.array_equal(out_values, x[src != 0])
        # brute force over the bits, pure Python
        want = [int(x[i]) if (int(bitmap[i // 32]) >> (i % 32)) & 1 else 0 for i in range(n)]
        assert out.tolist() == want


def test_mask_apply_special_cases(oracle):
    # a select, not a multiply: what sits under a cleared bit never leaks; kept elements keep their bits
    x = np.array([0x7FC00000, 0xFF800000, 0x80000000, 0x00000001, 0x3F800000], dtype=np.uint32)
    out = oracle.mask_apply(np.array([0b10110], dtype=np.uint32), x)
    assert out.tolist() == [0, 0xFF800000, 0x80000000, 0, 0x3F800000]
    # bits at positions >= n are ignored; all-ones and all-zero masks
    assert oracle.mask_apply(np.array([0xFFFFFFFF], dtype=np.uint32), x).tolist() == x.tolist()
    assert oracle.mask_apply(np.array([0xFFFFFFE0], dtype=np.uint32), x).tolist() == [0] * 5
    # it is the same function of (bitmap, tensor) as the ReLU backward
    g = np.arange(1, 71, dtype=np.uint16)
    bm = np.array([0xDEADBEEF, 0x12345678, 0x2A], dtype=np.uint32)
    assert np.array_equal(oracle.mask_apply(bm, g), oracle.relu_backward(bm, g))


def test_prune_fp64_against_numpy_and_special_values(oracle):
    """Double-precision elements: kept where the double exceeds the threshold, a double."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal(5000)
    x[::7] = 0.0
    specials = np.array([0.0, -0.0, 5e-324, -5e-324, np.nan, np.inf, -np.inf, 0.01, np.float64(np.float32(0.01)),
                         np.nextafter(0.01, 1.0), 1.7976931348623157e308], dtype=np.float64)
    x = np.concatenate([specials, x])
    for thr in (0.0, 0.01, 0.05, 0.1, -1.0, float("inf"), float("-inf")):
        with np.errstate(invalid="ignore"):
            want = np.where(x > thr, x.view(np.uint64), 0).astype(np.uint64)     # kept elements keep their bits
        got = oracle.prune(x.view(np.uint64), "f64", thr)
        assert np.array_equal(got, want), thr
    assert oracle.prune(specials.view(np.uint64), "f64", float("nan")).any() == False


def test_prune_threshold_that_is_no_single(oracle):
    """Section 4.3's thresholds (0.01, 0.05, 0.1) are not single-precision numbers.  The comparison is between
    real values, so it must not matter on which side of the threshold its nearest single lies.  Written out by
    hand for 0.1, whose nearest single, 0.100000001490116..., is ABOVE it, and 0.01, whose nearest single,
    0.00999999977648..., is BELOW it."""
    f32 = np.float32
    up = np.float64(f32(0.1))              # the single above 0.1
    dn = np.float64(np.nextafter(f32(0.1), f32(0)))   # the single below 0.1
    assert dn < 0.1 < up
    # doubles around 0.1: the threshold itself goes (strict), everything above it stays, however little above
    d = np.array([0.1, np.nextafter(0.1, 1.0), up, np.nextafter(0.1, 0.0), dn, -up], dtype=np.float64)
    got = oracle.prune(d.view(np.uint64), "f64", 0.1).view(np.float64)
    assert got.tolist() == [0.0, float(np.nextafter(0.1, 1.0)), float(up), 0.0, 0.0, 0.0]
    # singles around 0.1: the nearest single exceeds 0.1 and stays (a threshold rounded to single would drop it)
    s = np.array([f32(0.1), np.nextafter(f32(0.1), f32(0)), np.nextafter(f32(0.1), f32(1))], dtype=np.float32)
    got = oracle.prune(s.view(np.uint32), "f32", 0.1).view(np.float32)
    assert got.tolist() == [float(f32(0.1)), 0.0, float(np.nextafter(f32(0.1), f32(1)))]
    # singles around 0.01: its nearest single is below it and goes; the next one up stays
    s = np.array([f32(0.01), np.nextafter(f32(0.01), f32(1))], dtype=np.float32)
    assert np.float64(s[0]) < 0.01 < np.float64(s[1])
    got = oracle.prune(s.view(np.uint32), "f32", 0.01).view(np.float32)
    assert got.tolist() == [0.0, float(s[1])]
    # half precision: 0.0999755859375 is the half nearest 0.1 (below it), 0.10003662109375 the next
    h = np.array([0x2E66, 0x2E67], dtype=np.uint16)
    assert np.float64(h.view(np.float16)[0]) < 0.1 < np.float64(h.view(np.float16)[1])
    assert oracle.prune(h, "f16", 0.1).tolist() == [0, 0x2E67]


# ---- Algorithm 2's counter at tile boundaries ----

@pytest.mark.parametrize("tile", [1, 5, 32, 33, 64, 4096])
def test_tile_index_is_the_prefix_count_at_tile_starts(oracle, tile):
    rng = np.random.default_rng(31)
    for n in (0, 1, 31, 32, 33, 100, 4095, 4096, 4097, 10000):
        x = (rng.integers(1, 2**31, size=n) * (rng.random(n) < 0.35)).astype(np.uint32)
        bitmap, values, nnz = oracle.compress(x)
        index = oracle.tile_index(bitmap, n, tile)
        tiles = (n + tile - 1) // tile
        assert index.size == tiles
        # numpy: cumulative count of non-zeros before each tile start
        before = np.concatenate([[0], np.cumsum(x != 0)])
        assert np.array_equal(index, before[np.arange(tiles) * tile].astype(np.uint64))
        # what it is for: the values of tile t are values[index[t] : index[t+1]], so Algorithm 2 can start at any tile
        ends = np.append(index[1:], nnz) if tiles else np.array([], dtype=np.uint64)
        for t in range(0, tiles, max(1, tiles // 7)):
            lo, hi = t * tile, min((t + 1) * tile, n)
            chunk = x[lo:hi]
            assert np.array_equal(values[int(index[t]):int(ends[t])], chunk[chunk != 0])
            if lo % 32 == 0 and tile % 32 == 0:
                # restarting Algorithm 2 at element lo with j = index[t] restores exactly that tile
                part = oracle.decompress(bitmap[lo // 32:(hi + 31) // 32], values[int(index[t]):int(ends[t])], hi - lo)
                assert np.array_equal(part, chunk)


def test_tile_index_hand_built_and_degenerate(oracle):
    bm = np.array([0b1011, 0xFFFFFFFF, 0x0, 0x80000001], dtype=np.uint32)
    assert oracle.tile_index(bm, 128, 32).tolist() == [0, 3, 35, 35]
    assert oracle.tile_index(bm, 128, 64).tolist() == [0, 35]
    assert oracle.tile_index(bm, 100, 48).tolist() == [0, 19, 35]      # bits 0..47: 3 + 16
    assert oracle.tile_index(bm[:1], 4, 1).tolist() == [0, 1, 2, 2]
    assert oracle.tile_index(bm[:0], 0, 32).tolist() == []
    assert oracle.tile_index(np.zeros(4, dtype=np.uint32), 128, 32).tolist() == [0, 0, 0, 0]
    assert oracle.tile_index(np.full(4, 0xFFFFFFFF, dtype=np.uint32), 128, 32).tolist() == [0, 32, 64, 96]
