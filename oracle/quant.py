"""NVFP4 block quantizer Q_4^NV (Sec. 2.3; value set in App. C.1) -- oracle side.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

A row-major matrix is cut into blocks of 16 consecutive elements along its
last axis.  Per block one scale s in FP8-E4M3 is chosen from the block's
largest magnitude, rounded UP so that the largest element is covered
(6*s*g >= amax, 6 being the largest E2M1 magnitude); every element becomes
round(e / (s*g)) * (s*g) on the grid +-{0, .5, 1, 1.5, 2, 3, 4, 6}.

Readings of this build where the paper is silent:
  * g is a per-tensor power-of-two scale (g = 1 is the paper's text verbatim);
  * round(e / (s*g)) is taken in real arithmetic: |e| is compared with midpoint * s * g for
    the seven midpoints between neighbouring grid values (Sec. 2.3).  No division is done:
    midpoint * s * g has at most 7 significant bits and e is a float, so every comparison is
    exact in fp64;
  * round() is round-to-nearest, ties to the even E2M1 code;
  * a block whose amax exceeds 6*448*g saturates (scale 448, elements clamp to 6);
  * an all-zero block gets scale byte 0 and codes that keep only the sign bit.

Storage: codes[rows, cols/2] uint8, low nibble = even column, nibble =
sign<<3 | magnitude code; scales[rows, cols/16] uint8 = E4M3 bit pattern.
"""
import numpy as np

BLOCK = 16
E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
# decision boundaries between neighbouring grid values
E2M1_MID = (E2M1_GRID[:-1] + E2M1_GRID[1:]) / 2.0


def e4m3_value(byte):
    """Value of a non-negative FP8-E4M3 (4 exponent bits, bias 7, 3 mantissa
    bits, no infinities, largest finite 448) bit pattern 0x00..0x7E."""
    byte = np.asarray(byte, dtype=np.int64)
    e = byte >> 3
    m = byte & 7
    sub = m * 2.0 ** -9
    nor = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    return np.where(e == 0, sub, nor)


E4M3_POS = e4m3_value(np.arange(0, 127))      # 0, 2^-9, ..., 448 ascending


def quantize(x, g=1.0):
    """Quantize x[rows, cols] (cols % 16 == 0).  Returns (codes, scales)."""
    x = np.asarray(x, dtype=np.float64)
    rows, cols = x.shape
    assert cols % BLOCK == 0
    xb = x.reshape(rows, cols // BLOCK, BLOCK)
    amax = np.abs(xb).max(axis=2)
    # smallest E4M3 value s with 6*s*g >= amax: the scale rounds upward so the block maximum is covered (Sec. 2.3)
    cover = 6.0 * E4M3_POS * g
    sidx = np.searchsorted(cover, amax, side="left")
    sidx = np.minimum(sidx, 126)                    # saturate at 448
    step = (E4M3_POS[sidx] * g)[:, :, None]         # s*g: at most 4 significant bits
    a = np.abs(xb)
    mag = np.zeros(xb.shape, dtype=np.int64)
    for j, mid in enumerate(E2M1_MID):
        bound = mid * step                          # exact: at most 7 significant bits
        # a tie goes to the even code: boundary j separates codes j and j+1
        if (j + 1) % 2 == 0:
            mag += (a >= bound)
        else:
            mag += (a > bound)
    mag = np.where(step == 0, 0, mag)               # all-zero block: only the signs remain
    sign = np.signbit(xb).astype(np.int64)
    nib = (sign << 3) | mag
    nib = nib.reshape(rows, cols)
    codes = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return codes, sidx.astype(np.uint8)


STREAM_SR = 3          # Philox stream of the stochastic-rounding draws (row orientation)
STREAM_SR_T = 4        # ... of the transposed orientation


def quantize_sr(x, g, seed, stream=STREAM_SR, words=None):
    """Stochastically rounded variant (Sec. 4, FP4 Training: SR is the default of every FP4 run).

    The paper names the rounding mode and nothing else; readings of this build:
      * block scale exactly as in quantize(): chosen from the block's amax, rounded up;
      * a = min(|x| / (s*g), 6) in real arithmetic, as in quantize();
      * with lo <= a < hi the two neighbouring E2M1 magnitudes, the element goes to hi with
        probability t = (a - lo) / (hi - lo) and to lo otherwise (so its expectation is a);
        a value on the grid stays where it is;
      * the draw: u = (w >> 8) * 2^-24 with w the Philox4x32-10 word whose index is the
        element's row-major position in x, stream 3 (4 for a transposed copy); go up iff u < t.
        Evaluated without a division as (lo + u (hi - lo)) * s * g < |x|: the left side has at
        most 31 significant bits, so the comparison is exact in fp64 and the same everywhere.
    words (optional, uint32 of x's shape) replaces the Philox draws -- for tests.
    Returns (codes, scales) in the storage layout of quantize().
    """
    from . import rng
    x = np.asarray(x, dtype=np.float64)
    rows, cols = x.shape
    assert cols % BLOCK == 0
    xb = x.reshape(rows, cols // BLOCK, BLOCK)
    amax = np.abs(xb).max(axis=2)
    cover = 6.0 * E4M3_POS * g
    sidx = np.minimum(np.searchsorted(cover, amax, side="left"), 126)
    step = np.repeat(E4M3_POS[sidx] * g, BLOCK, axis=1)             # s*g per element, [rows, cols]
    a = np.abs(x)
    if words is None:
        words = rng.philox_words(seed, stream, 0, rows * cols).reshape(rows, cols)
    u = (np.asarray(words, dtype=np.uint64) >> np.uint64(8)).astype(np.float64) * 2.0 ** -24
    # lo = largest grid magnitude with lo * s * g <= |x| (products exact: at most 6 significant bits)
    lo_i = np.zeros(x.shape, dtype=np.int64)
    for j in range(1, 8):
        lo_i += (a >= E2M1_GRID[j] * step)
    hi_i = np.minimum(lo_i + 1, 7)
    lo, hi = E2M1_GRID[lo_i], E2M1_GRID[hi_i]
    up = (lo + u * (hi - lo)) * step < a                             # exact; never true at lo = hi = 6
    mag = np.where(up, hi_i, lo_i).astype(np.int64)
    mag = np.where(step == 0, 0, mag)
    sign = np.signbit(x).astype(np.int64)
    nib = (sign << 3) | mag
    codes = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return codes, sidx.astype(np.uint8)


# value of each nibble (sign << 3 | magnitude code), and of both nibbles of each code byte (low nibble first)
_NIBBLE_VALUE = E2M1_GRID[np.arange(16) & 7] * np.where(np.arange(16) & 8, -1.0, 1.0)
_BYTE_VALUES = np.stack([_NIBBLE_VALUE[np.arange(256) & 15], _NIBBLE_VALUE[np.arange(256) >> 4]], axis=1)


def dequantize(codes, scales, g=1.0):
    """Inverse map: fp64 matrix [rows, cols] of grid * s * g."""
    codes = np.asarray(codes).astype(np.uint8, copy=False)
    rows, half = codes.shape
    val = _BYTE_VALUES[codes].reshape(rows, half * 2 // BLOCK, BLOCK)    # element 2j = low nibble of byte j
    s = e4m3_value(scales) * g
    return (val * s[:, :, None]).reshape(rows, half * 2)


def tensor_scale_for(amax, headroom=1.0):
    """Smallest power of two g with 6*448*g >= amax*headroom (g <= 1 kept as is
    when amax is 0).  Power of two keeps every quantizer comparison exact."""
    amax = float(amax) * headroom
    if amax <= 0.0:
        return 1.0
    m, e = np.frexp(amax / (6.0 * 448.0))       # amax/2688 = m * 2^e, 0.5 <= m < 1
    return float(np.ldexp(1.0, e - 1 if m == 0.5 else e))
