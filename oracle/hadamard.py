"""Random Hadamard rotation in front of the stochastically rounded quantizer -- oracle side.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper compares Metis with a recipe that rotates tensors by a random Hadamard transform before rounding them
stochastically (Sec. 4.3, the comparison with another FP4 recipe; Sec. 5, Hadamard transformations) and gives no
further definition.  Readings of
this build: the rotation acts on the blocks of 16 consecutive elements that the quantizer scales together,
    z = (x * d) H_16 / 4,
H_16 the 16 x 16 Sylvester Hadamard matrix (natural order), d in {+1, -1}^16 one random sign per position in the
block, the same for every block of the tensor: d_i = -1 iff the top bit of word i of Philox stream 5 under the seed
is set.  H_16 / 4 is orthogonal, so rotating both operands of a product along its contraction axis leaves the
product unchanged.  The rotation is evaluated in fp32 (the kernels' precision: the rounded values are what the
quantizer sees, and its decisions are taken on exactly those) by the radix-2 butterfly in natural order: for
h = 1, 2, 4, 8 every pair (i, i + h) with bit h of i clear becomes (a + b, a - b); then the exact factor 1/4.
"""
import numpy as np
from . import quant, rng

STREAM_RHT = 5


def sign_vector(seed):
    w = rng.philox_words(seed, STREAM_RHT, 0, 16)
    return np.where((w >> np.uint32(31)) & np.uint32(1), -1.0, 1.0)


def rht16(x, seed, dtype=np.float32):
    """Rotate every block of 16 along the last axis of x[rows, cols]; arithmetic in `dtype`, result as fp64."""
    x = np.asarray(x, dtype=np.float64)
    rows, cols = x.shape
    assert cols % 16 == 0
    v = (x.reshape(rows, cols // 16, 16) * sign_vector(seed)).astype(dtype)
    for h in (1, 2, 4, 8):
        i = np.array([t for t in range(16) if not t & h])
        a, b = v[:, :, i].copy(), v[:, :, i + h].copy()
        v[:, :, i] = (a + b).astype(dtype)
        v[:, :, i + h] = (a - b).astype(dtype)
    return (v * dtype(0.25)).astype(np.float64).reshape(rows, cols)


def quantize_rht_sr(x, g, seed):
    """Rotate (draws of the signs: `seed`, stream 5), then quantize with stochastic rounding (draws: `seed`,
    stream 3, as quant.quantize_sr).  Returns (codes, scales)."""
    return quant.quantize_sr(rht16(x, seed), g, seed)
