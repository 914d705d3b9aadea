"""Footprint calculator for the formats of Section 3.2: dense (M_d), sparse bitmap
(M_b) and coordinate list (M_c), as in the paper's footprint figure and the
theoretical columns of Table 1.  Host arithmetic only; every number comes from the
size functions of the C library.
"""
import math

import torch

from . import bittrain as bt


def footprint(shape, nonzero_fraction, dtype=torch.float32):
    """Bytes needed to stash one activation tensor of `shape` of which
    `nonzero_fraction` is non-zero, in each format."""
    n = math.prod(shape)
    nnz = int(n * nonzero_fraction)
    dense = bt.bt_dense_size(n, dtype)
    bitmap = bt.bt_compressed_size(n, nnz, dtype)
    return {
        "elements": n,
        "non_zeros": nnz,
        "dense_bytes": dense,
        "bitmap_bytes": bitmap,
        "coo_int_bytes": bt.bt_coo_size(nnz, len(shape), 4, dtype),
        "coo_long_bytes": bt.bt_coo_size(nnz, len(shape), 8, dtype),
        "bitmap_improvement_pct": 100.0 * (1.0 - bitmap / dense) if dense else 0.0,
    }


def sweep(shape, fractions=(0.0, 0.25, 0.5, 0.75, 1.0), dtype=torch.float32):
    """The footprint of one shape over a range of non-zero fractions (Table 1 uses 0, 25, 50, 75 and 100 %)."""
    return [dict(footprint(shape, f, dtype), nonzero_fraction=f) for f in fractions]


def break_even_nonzero_fraction(ndim, index_bytes, dtype=torch.float32):
    """Largest non-zero fraction at which COO is no larger than dense, and the one at which
    the bitmap format is no larger than dense (31/32 for fp32)."""
    # per element: dense bytes, bytes of a COO entry, bitmap bytes and bytes of a stored value, all from the library
    dense32 = bt.bt_dense_size(32, dtype)
    coo_entry = bt.bt_coo_size(1, ndim, index_bytes, dtype)
    bitmap32 = bt.bt_compressed_size(32, 0, dtype)
    value = bt.bt_compressed_size(32, 1, dtype) - bitmap32
    return {"coo_vs_dense": (dense32 / 32) / coo_entry, "bitmap_vs_dense": (dense32 - bitmap32) / (32 * value)}
