"""MXFP4 block quantizer (microscaling format cited in Sec. 2.3 next to NVFP4) -- oracle side.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper names the microscaling (MX) family as the other block-wise FP4 scheme and defines none
of its details, so this follows the published OCP Microscaling Formats (MX) v1.0 specification:
  * a block is 32 consecutive elements along the last axis;
  * the shared scale X is a power of two stored as E8M0 (one byte, value 2^(byte - 127));
  * X = 2^(floor(log2(amax)) - emax), emax = 2 being the exponent of the largest E2M1 value 6 = 1.5 * 2^2
    (conversion rule of the specification, Sec. 6.3);
  * every element becomes round(e / X) on the E2M1 grid +-{0, .5, 1, 1.5, 2, 3, 4, 6}; the quotient is exact
    (X is a power of two), magnitudes beyond 6 (they reach up to 8) saturate to 6.
Readings of this build where the specification leaves a choice:
  * round() is round-to-nearest, ties to the even E2M1 code (the specification lets the
    implementation choose; the NVFP4 path of this build rounds the same way);
  * an all-zero block stores scale byte 0 and codes that keep only the sign bit;
  * the shared exponent is clamped to the E8M0 range [-127, 127].

Storage: codes[rows, cols/2] uint8, low nibble = even column, nibble = sign<<3 | magnitude code
(the same as the NVFP4 path); scales[rows, cols/32] uint8 = E8M0 bit pattern.
"""
import numpy as np
from .quant import E2M1_GRID, E2M1_MID

BLOCK = 32
EMAX_E2M1 = 2


def quantize_mx(x):
    """Quantize x[rows, cols] (cols % 32 == 0).  Returns (codes, scales)."""
    x = np.asarray(x, dtype=np.float64)
    rows, cols = x.shape
    assert cols % BLOCK == 0
    xb = x.reshape(rows, cols // BLOCK, BLOCK)
    amax = np.abs(xb).max(axis=2)
    nz = amax > 0
    # floor(log2(amax)) from the binary exponent: amax = m * 2^ex with m in [0.5, 1)
    _, ex = np.frexp(np.where(nz, amax, 1.0))
    shared = np.clip(ex - 1 - EMAX_E2M1, -127, 127)
    shared = np.where(nz, shared, -127)
    X = np.exp2(shared.astype(np.float64))
    a = np.abs(xb) / X[:, :, None]                 # exact: a power-of-two divisor
    mag = np.zeros(xb.shape, dtype=np.int64)
    for j, mid in enumerate(E2M1_MID):
        if (j + 1) % 2 == 0:                       # a tie goes to the even code
            mag += (a >= mid)
        else:
            mag += (a > mid)
    sign = np.signbit(xb).astype(np.int64)
    nib = ((sign << 3) | mag).reshape(rows, cols)
    codes = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return codes, (shared + 127).astype(np.uint8)


def dequantize_mx(codes, scales):
    """fp64 values of an MXFP4 matrix."""
    codes = np.asarray(codes)
    rows = codes.shape[0]
    nib = np.empty((rows, codes.shape[1] * 2), dtype=np.int64)
    nib[:, 0::2] = codes & 15
    nib[:, 1::2] = codes >> 4
    val = E2M1_GRID[nib & 7] * np.where(nib & 8, -1.0, 1.0)
    X = np.exp2(np.asarray(scales).astype(np.float64) - 127.0)
    return (val.reshape(rows, -1, BLOCK) * X[:, :, None]).reshape(rows, -1)


def mx_gemm_nt(a, b):
    """C = A B^T of two MXFP4 matrices given as (codes, scales), blocks along the contraction axis."""
    return dequantize_mx(*a) @ dequantize_mx(*b).T
