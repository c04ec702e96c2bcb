"""Random draws of the scalable decomposition (Sec. 3.1) -- oracle side.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper asks for (i) a random subset of rows and (ii) a Gaussian test matrix
Omega with k+s columns, without fixing a generator.  Both are drawn here from
Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
as 1, 2, 3", SC'11), written from the published round function.

Stream convention (a reading of this build, the paper is silent):
  word w of stream t under a 64-bit seed is output lane (w mod 4) of the Philox
  block with counter (w div 4 low 32 bits, w div 4 high 32 bits, t, 0) and key
  (seed low 32 bits, seed high 32 bits).
  stream 1 -> row sample, stream 2 -> Omega.
"""
import numpy as np

PHILOX_M0 = 0xD2511F53
PHILOX_M1 = 0xCD9E8D57
PHILOX_W0 = 0x9E3779B9
PHILOX_W1 = 0xBB67AE85
MASK32 = 0xFFFFFFFF

STREAM_ROWS = 1
STREAM_OMEGA = 2


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds.

    counter: uint array [..., 4], key: uint array [..., 2] (broadcastable).
    Returns uint32 array [..., 4].
    """
    c = np.asarray(counter, dtype=np.uint64) & MASK32
    k = np.asarray(key, dtype=np.uint64) & MASK32
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = k[..., 0], k[..., 1]
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + PHILOX_W0) & MASK32
            k1 = (k1 + PHILOX_W1) & MASK32
        p0 = c0 * np.uint64(PHILOX_M0)      # 32x32 -> 64 bit, no overflow in uint64
        p1 = c2 * np.uint64(PHILOX_M1)
        hi0, lo0 = p0 >> np.uint64(32), p0 & MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def philox_words(seed, stream, first, count):
    """Words first .. first+count-1 of the given stream, as uint32[count]."""
    seed = int(seed)
    w = np.arange(first, first + count, dtype=np.uint64)
    blk = w >> np.uint64(2)
    lane = (w & np.uint64(3)).astype(np.int64)
    ctr = np.stack([blk & MASK32, blk >> np.uint64(32),
                    np.full_like(blk, stream), np.zeros_like(blk)], axis=-1)
    key = np.array([seed & MASK32, (seed >> 32) & MASK32], dtype=np.uint64)
    out = philox4x32_10(ctr, key)
    return out[np.arange(count), lane]


def sample_count(M, k, p, rho, group=1):
    """Number of sampled rows l_k.  group = 1: ceil(rho*M), at least k+p, at most M.
    group > 1 (whole sequences of `group` consecutive rows are drawn, Sec. 3.1 samples sequences; M % group == 0):
    ceil(rho * M/group) sequences, at least ceil((k+p)/group), at most M/group, times group."""
    r = k + p
    if group == 1:
        return int(min(M, max(r, int(np.ceil(rho * M - 1e-12)))))
    assert M % group == 0
    G = M // group
    return int(min(G, max(-(-r // group), int(np.ceil(rho * G - 1e-12))))) * group


def sample_rows(seed, M, Ms, group=1):
    """Random subset of Ms of the M rows (Sec. 3.1, sparse random sampling).

    Reading: one row drawn uniformly from each of Ms equal strata, so the rows
    are distinct, ascending, and every row has inclusion probability ~Ms/M.
      lo_j = floor(j*M/Ms), hi_j = floor((j+1)*M/Ms),
      idx_j = lo_j + (u_j mod (hi_j - lo_j)),  u_j = word j of stream 1.
    group > 1: the same draw over the M/group sequences (Ms/group of them), each chosen
    sequence contributing its `group` consecutive rows.
    """
    if group > 1:
        assert M % group == 0 and Ms % group == 0
        g = sample_rows(seed, M // group, Ms // group)
        return (g[:, None] * group + np.arange(group, dtype=np.int64)[None, :]).reshape(-1)
    j = np.arange(Ms, dtype=np.int64)
    lo = (j * M) // Ms
    hi = ((j + 1) * M) // Ms
    u = philox_words(seed, STREAM_ROWS, 0, Ms).astype(np.int64)
    return (lo + u % (hi - lo)).astype(np.int64)


def round_to_bf16(x):
    """Round fp64 values to the nearest bfloat16 (ties to even); returns fp64."""
    f = np.asarray(x, dtype=np.float64)
    out = np.zeros_like(f)
    nz = f != 0
    m, e = np.frexp(f[nz])              # f = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0      # 8 significant bits; rint = ties-to-even
    out[nz] = np.ldexp(q, e)
    return out


def gaussian_omega(seed, N, r):
    """Gaussian test matrix Omega in R^{N x r} (Sec. 3.1, random projection).

    Entry e = n*r + c uses words 2e and 2e+1 of stream 2:
      u1 = ((w0 >> 9) + 0.5) * 2^-23   in (0,1)
      u2 =  (w1 >> 8)        * 2^-24   in [0,1)
      z  = sqrt(-2 ln u1) * cos(2 pi u2)         (Box-Muller)
    and is then rounded to bfloat16 (the sketch multiplies bf16 by bf16).
    """
    cnt = N * r
    w = philox_words(seed, STREAM_OMEGA, 0, 2 * cnt).astype(np.float64)
    w0, w1 = w[0::2], w[1::2]
    u1 = (np.floor(w0 / 512.0) + 0.5) * 2.0 ** -23
    u2 = np.floor(w1 / 256.0) * 2.0 ** -24
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return round_to_bf16(z).reshape(N, r)
