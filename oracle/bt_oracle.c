/*
 * bt_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded CPU statement of the sparse bitmap codec of
 * BitTrain (Section 3.2 "Bitmap Format"; Algorithm 1, dense -> bitmap;
 * Algorithm 2, bitmap -> dense; the footprint formulas M_d and M_b).  It is
 * the definition the GPU library is checked against.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it; the product path
 * never does.  It shares no code, header, table or constant with the GPU
 * library.
 *
 * Readings of the paper that this file fixes (each is a deliberate choice):
 *   - "zero" is the all-zero bit pattern of the element, not an IEEE compare:
 *     -0.0, NaN, denormals and infinities are kept as values, so the round
 *     trip of Algorithm 1 followed by Algorithm 2 is bit-exact.
 *   - element i owns bit (i mod 32), least significant bit first, of the
 *     32-bit word (i div 32); the bitmap has ceil(n/32) words and the unused
 *     high bits of the last word are zero.  The paper's N/8 bytes is the same
 *     number whenever 32 divides N.
 *   - Algorithm 2's loop runs over the n valid bits.
 *   - a cleared bit restores the all-zero pattern (+0.0) of the element width.
 *   - values are appended in ascending flattened index order.
 *   - the element is defined by its width only (2, 4 or 8 bytes): fp16 and
 *     bf16 are the same codec.
 *
 * Activation pruning (Section 4.3) is bt_oracle_prune: an element is kept where its
 * value exceeds the threshold (strictly, and as real numbers: every element format widens
 * exactly to double, where it is compared with the threshold, a double; a NaN exceeds nothing) and becomes +0
 * elsewhere.  With threshold 0 on a pre-activation tensor this is ReLU.  Pruning
 * followed by Algorithm 1 is what the fused GPU call is checked against.
 *
 * The COO footprint M_c of Section 3.2 is bt_oracle_coo_size (a value plus one index per
 * dimension for every non-zero).  The double-mask batch normalisation of Section 3.1
 * (the sparsity pattern of a layer's input is applied to its output) is
 * bt_oracle_mask_apply: out[i] = x[i] where the other tensor's bitmap has bit i set, +0
 * elsewhere -- the same select as the ReLU backward, stated on its own.
 *
 * bt_oracle_tile_index is Algorithm 2's counter j sampled at regular positions: entry t
 * is the value j has when the loop reaches element t * tile_elems, i.e. the number of
 * values consumed before that element.  With it Algorithm 2 can start anywhere.
 *
 * Parity pins (tests/test_oracle_*.py): the theoretical columns of Table 1,
 * hand-built tensors, numpy.packbits / boolean indexing, enumeration of all
 * 2^16 zero patterns of a 16-element tensor, every n in [0,130], closed forms
 * for the all-zero and all-non-zero tensors, and a pruning threshold that no
 * single-precision number equals.  No function here is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* Element i of a flat buffer of width-byte elements, as an unsigned integer
 * holding its raw bit pattern. */
static uint64_t load_bits(const unsigned char *base, uint64_t i, int width)
{
    uint64_t v = 0;
    memcpy(&v, base + i * (uint64_t)width, (size_t)width); /* little-endian host */
    return v;
}

static void store_bits(unsigned char *base, uint64_t i, int width, uint64_t v)
{
    memcpy(base + i * (uint64_t)width, &v, (size_t)width);
}

static int width_ok(int width) { return width == 2 || width == 4 || width == 8; }

/* M_b generalised to any element width: one bit per element, rounded up to
 * whole 32-bit words, plus the non-zero values.  Returns 0 when the arguments
 * make no sense (unknown width, nnz > n). */
uint64_t bt_oracle_compressed_size(uint64_t n, uint64_t nnz, int width)
{
    if (!width_ok(width) || nnz > n) return 0;
    uint64_t words = n / 32 + (n % 32 != 0);
    return 4 * words + nnz * (uint64_t)width;
}

/* M_d: the dense footprint. */
uint64_t bt_oracle_dense_size(uint64_t n, int width)
{
    if (!width_ok(width)) return 0;
    return n * (uint64_t)width;
}

/* Algorithm 1.  T is the flat dense tensor of n elements.  bitmap must hold
 * ceil(n/32) words and values up to n elements.  Returns nnz, or UINT64_MAX
 * for an unknown width. */
uint64_t bt_oracle_compress(const void *T, uint64_t n, int width,
                            uint32_t *bitmap, void *values)
{
    if (!width_ok(width)) return UINT64_MAX;
    const unsigned char *t = (const unsigned char *)T;
    unsigned char *vals = (unsigned char *)values;
    uint64_t words = n / 32 + (n % 32 != 0);
    for (uint64_t w = 0; w < words; ++w) bitmap[w] = 0;

    uint64_t j = 0;                          /* values stored so far */
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t bits = load_bits(t, i, width);
        if (bits == 0) {
            /* a zero element: its bit stays clear (the word was cleared above) */
        } else {
            store_bits(vals, j, width, bits);             /* a non-zero element is appended to the values */
            j += 1;
            bitmap[i / 32] |= (uint32_t)1 << (i % 32);    /* and its bit is set */
        }
    }
    return j;
}

/* Algorithm 2.  Rebuilds the n-element dense tensor.  Returns the number of
 * values consumed (the final j), or UINT64_MAX for an unknown width. */
uint64_t bt_oracle_decompress(const uint32_t *bitmap, const void *values,
                              uint64_t n, int width, void *T)
{
    if (!width_ok(width)) return UINT64_MAX;
    const unsigned char *vals = (const unsigned char *)values;
    unsigned char *t = (unsigned char *)T;
    uint64_t j = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if ((bitmap[i / 32] >> (i % 32)) & 1u) {
            store_bits(t, i, width, load_bits(vals, j, width));
            j += 1;
        } else {
            store_bits(t, i, width, 0);
        }
    }
    return j;
}

/* The bitmap of y = ReLU(x) is the ReLU derivative mask (bit set <=> y != 0
 * <=> x > 0), so the backward pass of ReLU needs only the bitmap:
 * grad_in[i] = bit(i) ? grad_out[i] : +0.  A select, not a multiply: a NaN or
 * Inf in grad_out under a cleared bit does not leak. */
int bt_oracle_relu_backward(const uint32_t *bitmap, const void *grad_out,
                            uint64_t n, int width, void *grad_in)
{
    if (!width_ok(width)) return -1;
    const unsigned char *g = (const unsigned char *)grad_out;
    unsigned char *o = (unsigned char *)grad_in;
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t keep = (bitmap[i / 32] >> (i % 32)) & 1u;
        store_bits(o, i, width, keep ? load_bits(g, i, width) : 0);
    }
    return 0;
}

/* ---- activation pruning (Section 4.3) ---------------------------------------- */

/* dtype codes of this file only: 0 = fp32, 1 = fp16, 2 = bfloat16 (3 = fp64 is not widened: see bt_oracle_prune) */
static float widen_to_f32(uint64_t bits, int dtype)
{
    uint32_t u;
    float f;
    if (dtype == 0) {
        u = (uint32_t)bits;
    } else if (dtype == 2) {
        u = (uint32_t)bits << 16;                       /* bfloat16 is the top half of fp32 */
    } else {
        uint32_t sign = ((uint32_t)bits >> 15) & 1u;
        uint32_t exp = ((uint32_t)bits >> 10) & 0x1Fu;
        uint32_t man = (uint32_t)bits & 0x3FFu;
        if (exp == 0x1F) {                              /* infinity or NaN */
            u = (sign << 31) | 0x7F800000u | (man << 13);
        } else if (exp != 0) {                          /* normal: rebias 15 -> 127 */
            u = (sign << 31) | ((exp + 112u) << 23) | (man << 13);
        } else if (man == 0) {                          /* zero */
            u = sign << 31;
        } else {                                        /* subnormal: man * 2^-24, normal in fp32 */
            int shift = 0;
            while ((man & 0x400u) == 0) { man <<= 1; ++shift; }
            man &= 0x3FFu;
            u = (sign << 31) | ((uint32_t)(113 - shift) << 23) | (man << 13);
        }
    }
    memcpy(&f, &u, sizeof f);
    return f;
}

/* out[i] = T[i] where value(T[i]) > threshold, +0 (all-zero bits) elsewhere.
 * The element is widened to double (exact for all four formats) and compared there.
 * Returns the number of kept elements, or UINT64_MAX for an unknown dtype. */
uint64_t bt_oracle_prune(const void *T, uint64_t n, int dtype, double threshold, void *out)
{
    if (dtype < 0 || dtype > 3) return UINT64_MAX;
    const int width = dtype == 3 ? 8 : (dtype == 0 ? 4 : 2);
    const unsigned char *t = (const unsigned char *)T;
    unsigned char *o = (unsigned char *)out;
    uint64_t kept = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t bits = load_bits(t, i, width);
        int keep;
        if (dtype == 3) {
            double d;
            memcpy(&d, &bits, sizeof d);
            keep = d > threshold;
        } else {
            keep = (double)widen_to_f32(bits, dtype) > threshold;
        }
        if (keep) {
            store_bits(o, i, width, bits);
            kept += 1;
        } else {
            store_bits(o, i, width, 0);
        }
    }
    return kept;
}

/* ---- the comparison format and the double mask -------------------------------- */

/* M_c of Section 3.2: every non-zero activation is stored as its value plus one index
 * per dimension; indices are 4-byte integers or 8-byte longs.  Returns 0 when the
 * arguments make no sense. */
uint64_t bt_oracle_coo_size(uint64_t nnz, int ndim, int index_bytes, int width)
{
    if (!width_ok(width) || ndim < 1 || (index_bytes != 4 && index_bytes != 8)) return 0;
    return ((uint64_t)width + (uint64_t)index_bytes * (uint64_t)ndim) * nnz;
}

/* Double mask (Section 3.1): the bitmap of one tensor (a normalisation layer's input)
 * masks another tensor x of the same length (that layer's output). */
int bt_oracle_mask_apply(const uint32_t *bitmap, const void *x, uint64_t n, int width, void *out)
{
    if (!width_ok(width)) return -1;
    const unsigned char *src = (const unsigned char *)x;
    unsigned char *dst = (unsigned char *)out;
    for (uint64_t i = 0; i < n; ++i) {
        if ((bitmap[i / 32] >> (i % 32)) & 1u)
            store_bits(dst, i, width, load_bits(src, i, width));
        else
            store_bits(dst, i, width, 0);
    }
    return 0;
}

/* Algorithm 2's counter j at the start of every block of tile_elems elements:
 * index[t] = number of set bits among bits [0, min(t * tile_elems, n)).  Writes
 * ceil(n / tile_elems) entries and returns that number (0 when tile_elems is 0). */
uint64_t bt_oracle_tile_index(const uint32_t *bitmap, uint64_t n, uint64_t tile_elems, uint64_t *index)
{
    if (tile_elems == 0) return 0;
    uint64_t j = 0, tiles = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i % tile_elems == 0) index[tiles++] = j;      /* j before element i */
        if ((bitmap[i / 32] >> (i % 32)) & 1u) j += 1;    /* Algorithm 2: a set bit consumes a value */
    }
    return tiles;
}
