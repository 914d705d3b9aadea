"""TEST INFRASTRUCTURE ONLY: Algorithms 1 and 2 of BitTrain as Python lists.

The smallest possible statement of the codec, for inputs of a few hundred
elements: the dense tensor is a list of unsigned integers (the raw bit pattern
of each element), the bitmap is a list of 0/1 ints, one per element, exactly as
the two algorithms push them.  ``pack_words`` then lays the bit list out as the
32-bit words the C oracle and the GPU library use (element i -> bit i mod 32,
least significant first, of word i div 32).  Used to pin ``bt_oracle.c``.
"""


def to_bitmap(T):
    """Algorithm 1: scan T once, pushing one bit per element and each
    non-zero element (by bit pattern) to the values list."""
    bitmap, values = [], []
    for t in T:
        if t == 0:
            bitmap.append(0)
        else:
            values.append(t)
            bitmap.append(1)
    return bitmap, values


def to_dense(bitmap, values):
    """Algorithm 2: scan the bits once, consuming values[j] at each set bit."""
    T, j = [], 0
    for b in bitmap:
        if b:
            T.append(values[j])
            j += 1
        else:
            T.append(0)
    return T


def relu_backward(bitmap, grad_out):
    """ReLU backward from the bitmap of the ReLU output: a select."""
    return [g if b else 0 for b, g in zip(bitmap, grad_out)]


def pack_words(bitmap):
    """Bit list -> list of uint32 words, zero-padded in the last word."""
    words = [0] * ((len(bitmap) + 31) // 32)
    for i, b in enumerate(bitmap):
        if b:
            words[i // 32] |= 1 << (i % 32)
    return words


def footprint_bytes(n, nnz, width):
    """M_b with the bitmap rounded up to 32-bit words; M_d = n * width."""
    return 4 * ((n + 31) // 32) + nnz * width
