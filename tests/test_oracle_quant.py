"""Pins for oracle/quant.py: the paper's value table, a library decode of E4M3,
an exact rational-arithmetic restatement of round(e/s)*s, ties, scale coverage."""
import os
from fractions import Fraction

import numpy as np
import torch

from oracle import quant
from oracle import quant as oq
from oracle import rng as orng


def test_grid_matches_paper_table(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "e2m1_grid.txt"))
            if l.strip() and not l.startswith("#")]
    assert [float(v) for _, v in rows] == list(quant.E2M1_GRID)
    # E2M1 bit semantics: code = e(2 bits) m(1 bit), bias 1, subnormal at e = 0
    for c in range(8):
        e, m = c >> 1, c & 1
        v = m * 0.5 if e == 0 else (1 + m / 2) * 2.0 ** (e - 1)
        assert v == quant.E2M1_GRID[c]


def test_e4m3_table_matches_library_decode():
    ref = torch.arange(0, 127, dtype=torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    assert np.array_equal(ref, quant.E4M3_POS)
    assert quant.E4M3_POS[126] == 448.0 and quant.E4M3_POS[1] == 2.0 ** -9
    assert np.all(np.diff(quant.E4M3_POS) > 0)
    assert np.count_nonzero(quant.E4M3_POS) == 126


def _exact_quantize_block(block, g):
    """round(e/s)*s with exact rationals: scale = smallest E4M3 covering amax/6,
    nearest grid value, ties to the even code."""
    fr = [Fraction(float(v)) for v in block]
    amax = max(abs(v) for v in fr)
    gq = Fraction(float(g))
    sidx = 126
    for i in range(127):
        if 6 * Fraction(float(quant.E4M3_POS[i])) * gq >= amax:
            sidx = i
            break
    step = Fraction(float(quant.E4M3_POS[sidx])) * gq
    grid = [Fraction(float(v)) for v in quant.E2M1_GRID]
    codes = []
    for v in fr:
        if step == 0:
            codes.append(0)
            continue
        t = abs(v) / step
        best = min(range(8), key=lambda c: (abs(t - grid[c]), c % 2))
        codes.append(best)
    return sidx, codes


def _nibbles(codes):
    n = np.empty((codes.shape[0], codes.shape[1] * 2), dtype=np.int64)
    n[:, 0::2] = codes & 15
    n[:, 1::2] = codes >> 4
    return n


def test_against_exact_rational_rounding_random():
    rs = np.random.default_rng(1)
    for g in (1.0, 2.0 ** -11, 2.0 ** 3):
        x = rs.standard_normal((40, 32)) * np.exp(rs.uniform(-8, 8, (40, 1))) * g
        x = x.astype(np.float32).astype(np.float64)
        codes, scales = quant.quantize(x, g)
        nib = _nibbles(codes)
        for i in range(x.shape[0]):
            for b in range(2):
                blk = x[i, 16 * b:16 * b + 16]
                sidx, mags = _exact_quantize_block(blk, g)
                assert scales[i, b] == sidx
                assert list(nib[i, 16 * b:16 * b + 16] & 7) == mags
        assert np.array_equal(nib >> 3, np.signbit(x).astype(np.int64))


def test_against_exact_rational_all_scales_bf16_inputs():
    # every E4M3 scale is exercised; inputs are bf16 values (what the path feeds)
    rs = np.random.default_rng(2)
    for sidx in range(1, 127):
        s = quant.E4M3_POS[sidx]
        blk = rs.uniform(-6.2, 6.2, 16) * s
        blk[0] = 5.9 * s * rs.choice([-1, 1])       # pins the scale to >= this index region
        blk = torch.from_numpy(blk).to(torch.bfloat16).double().numpy()
        codes, scales = quant.quantize(blk[None, :])
        ref_s, ref_c = _exact_quantize_block(blk, 1.0)
        assert scales[0, 0] == ref_s
        assert list(_nibbles(codes)[0] & 7) == ref_c


def test_ties_go_to_even_code():
    # with scale 1.0 (byte 0x38) and the block max at 6, midpoints map as RNE demands
    blk = np.zeros(16)
    blk[0] = 6.0
    mids = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    blk[1:8] = mids
    blk[8:15] = [-m for m in mids]
    codes, scales = quant.quantize(blk[None, :])
    assert scales[0, 0] == 0x38 and quant.E4M3_POS[0x38] == 1.0
    d = quant.dequantize(codes, scales)[0]
    assert list(d[1:8]) == [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0]
    assert list(d[8:15]) == [-0.0, -1.0, -1.0, -2.0, -2.0, -4.0, -4.0]
    assert d[0] == 6.0
    # just above / below a midpoint
    blk[1:3] = [np.nextafter(np.float32(0.25), np.float32(1)), np.nextafter(np.float32(0.75), np.float32(0))]
    d = quant.dequantize(*quant.quantize(blk[None, :]))[0]
    assert list(d[1:3]) == [0.5, 0.5]


def test_scale_covers_block_max_and_is_minimal():
    rs = np.random.default_rng(3)
    x = (rs.standard_normal((64, 64)) * np.exp(rs.uniform(-6, 4, (64, 4)).repeat(16, axis=1)))
    for g in (1.0, 0.25):
        codes, scales = quant.quantize(x, g)
        amax = np.abs(x.reshape(64, 4, 16)).max(axis=2)
        s = quant.E4M3_POS[scales] * g
        assert np.all(6 * s >= amax)
        below = quant.E4M3_POS[np.maximum(scales.astype(int) - 1, 0)] * g
        assert np.all((6 * below < amax) | (scales == 0))
        # for normal-range scales the block max lands on +-6
        d = quant.dequantize(codes, scales, g).reshape(64, 4, 16)
        normal = scales >= 8
        assert np.all(np.abs(d).max(axis=2)[normal] == 6 * s[normal])


def test_error_bound_and_idempotence():
    rs = np.random.default_rng(4)
    x = rs.standard_normal((32, 128))
    codes, scales = quant.quantize(x)
    d = quant.dequantize(codes, scales)
    s = np.repeat(quant.E4M3_POS[scales], 16, axis=1)
    # widest grid gap is 2 (between 4 and 6): error <= 1 step everywhere, <= 0.25 step below 2
    assert np.all(np.abs(x - d) <= 1.0 * s + 1e-15)
    small = np.abs(x) <= 2 * s
    assert np.all(np.abs(x - d)[small] <= 0.25 * s[small] + 1e-15)
    c2, s2 = quant.quantize(d)
    assert np.array_equal(c2, codes) and np.array_equal(s2, scales)


def test_zero_block_saturation_and_signs():
    blk = np.zeros((1, 32))
    blk[0, 3] = -0.0
    blk[0, 16:] = 1e9
    blk[0, 17] = -1e9
    codes, scales = quant.quantize(blk)
    assert scales[0, 0] == 0 and scales[0, 1] == 126
    nib = _nibbles(codes)[0]
    assert nib[3] == 8 and np.all(np.delete(nib[:16], 3) == 0)
    assert nib[16] == 7 and nib[17] == 15
    d = quant.dequantize(codes, scales)
    assert np.all(d[0, :16] == 0) and d[0, 16] == 6 * 448 and d[0, 17] == -6 * 448


def test_tiny_values_flush_without_tensor_scale():
    # paper-literal g = 1: a block below 6*2^-9 cannot be covered finer than 2^-9 steps
    blk = np.full((1, 16), 2.0 ** -13)
    d1 = quant.dequantize(*quant.quantize(blk, 1.0), 1.0)
    assert np.all(d1 == 0)
    g = 2.0 ** -11
    d2 = quant.dequantize(*quant.quantize(blk, g), g)
    # the scale is rounded up, so the block max maps to 6*s*g >= amax (within one E4M3 step)
    assert np.all(d2 >= blk) and np.all(d2 <= blk * 1.125)


def test_tensor_scale_for():
    assert quant.tensor_scale_for(6 * 448.0) == 1.0
    assert quant.tensor_scale_for(6 * 448.0 + 1) == 2.0
    assert quant.tensor_scale_for(1.0) == 2.0 ** -11
    assert quant.tensor_scale_for(0.0) == 1.0


def test_packing_layout():
    blk = np.zeros((1, 16))
    blk[0, 0], blk[0, 1] = 6.0, -3.0       # codes 7 and 8|5
    codes, _ = quant.quantize(blk)
    assert codes[0, 0] == (7 | (13 << 4))


def test_ties_to_even_with_every_scale_mantissa():
    # values exactly on a midpoint stay there under the fp32 quotient, for any scale mantissa
    for sidx in (0x38, 0x39, 0x3B, 0x3F, 0x45, 0x12, 0x05):
        s = quant.E4M3_POS[sidx]
        blk = np.zeros(16)
        blk[0] = 6.0 * s
        blk[1:8] = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]) * s
        codes, scales = quant.quantize(blk[None, :])
        assert scales[0, 0] == sidx
        d = quant.dequantize(codes, scales)[0] / s
        assert list(d[:8]) == [6.0, 0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0]


def test_one_ulp_either_side_of_every_midpoint_every_scale():
    # round(e/s) in real arithmetic: an fp32 input one ulp below / on / one ulp above midpoint * s * g decides by its
    # true side, for every E4M3 scale (with and without mantissa bits) -- checked against exact rationals
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    below = [0, 1, 2, 3, 4, 5, 6]            # code just below each midpoint
    even = [0, 2, 2, 4, 4, 6, 6]             # where a tie goes
    for g in (1.0, 2.0 ** -11, 2.0 ** 5):
        for sidx in range(1, 127):
            s = quant.E4M3_POS[sidx] * g
            t = (mids * s).astype(np.float32)
            assert np.array_equal(t.astype(np.float64), mids * s)      # thresholds are fp32 values
            for delta, want in ((-1, below), (0, even), (1, [b + 1 for b in below])):
                blk = np.zeros(16)
                blk[0] = 6.0 * s
                v = t if delta == 0 else np.nextafter(t, np.float32(np.inf if delta > 0 else 0))
                blk[1:8] = v.astype(np.float64)
                blk[8:15] = -blk[1:8]
                codes, scales = quant.quantize(blk[None, :], g)
                assert scales[0, 0] == sidx
                nib = _nibbles(codes)[0]
                assert list(nib[1:8]) == want and list(nib[8:15] & 7) == want and np.all(nib[8:15] >> 3 == 1)
                ref_s, ref_c = _exact_quantize_block(blk, g)
                assert ref_s == sidx and list(nib & 7) == ref_c


def test_correctly_rounded_fp32_quotient_never_changes_a_decision():
    # Property the GPU quantizer relies on: for fp32 inputs, rounding the IEEE fp32 quotient x / (s g) to the E2M1 grid
    # (ties to even) takes the same decisions as the exact rule.  fl32(x/step) can equal a midpoint m with x != m step
    # only if two fp32 neighbours of m step are closer than m's own half-ulp relative spacing, which would need
    # significand(m step) >= 2 significand(m).  Checked here on the fp32 neighbours of every threshold and at random.
    rs = np.random.default_rng(7)
    mids32 = quant.E2M1_MID.astype(np.float32)

    def by_quotient(x32, step32):
        y = np.abs(x32 / step32).astype(np.float32)
        mag = np.zeros(y.shape, dtype=np.int64)
        for j, m in enumerate(mids32):
            mag += (y >= m) if (j + 1) % 2 == 0 else (y > m)
        return mag

    for g in (1.0, 2.0 ** -11):
        for sidx in range(1, 127):
            step = np.float32(quant.E4M3_POS[sidx] * g)
            t = mids32 * step
            x = np.concatenate([t, np.nextafter(t, np.float32(0)), np.nextafter(t, np.float32(np.inf)),
                                (rs.uniform(0, 6, 57) * float(step)).astype(np.float32)])
            x[0] = np.float32(6) * step
            got = by_quotient(x, step)
            for i in range(0, x.size, 16):
                blk = x[i:i + 16].astype(np.float64).copy()
                blk[0] = 6.0 * float(step)
                ref_s, ref_c = _exact_quantize_block(blk, g)
                assert ref_s == sidx
                assert list(got[i + 1:i + 16]) == ref_c[1:]


# ---------------------------------------------------------------------------------------------
# Stochastic rounding (Sec. 4, FP4 Training): pins of oracle.quant.quantize_sr
# ---------------------------------------------------------------------------------------------
def _deq_mag(codes, scales, g):
    return np.abs(oq.dequantize(codes, scales, g))


def test_sr_scale_choice_is_the_rne_quantizers_and_signs_kept():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((8, 64)) * np.exp(rng.uniform(-6, 6, (8, 1)))
    x[0, :16] = 0.0
    x[1, 3] = -0.0
    c0, s0 = oq.quantize(x, 0.25)
    c1, s1 = oq.quantize_sr(x, 0.25, seed=11)
    assert np.array_equal(s0, s1)
    assert np.array_equal((c0 & 0x88), (c1 & 0x88))          # sign bits of both nibbles


def test_sr_result_is_one_of_the_two_neighbours_and_grid_points_stay():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((16, 128)).astype(np.float32).astype(np.float64)
    g = 2.0 ** -3
    codes, scales = oq.quantize_sr(x, g, seed=3)
    step = np.repeat(oq.e4m3_value(scales) * g, 16, axis=1)
    y = np.minimum(np.abs(x) / step, 6.0)            # fp64 quotient: off by 1e-16, far from any grid point here
    q = _deq_mag(codes, scales, g) / step
    lo = oq.E2M1_GRID[np.searchsorted(oq.E2M1_GRID, y, side="right") - 1]
    hi = oq.E2M1_GRID[np.minimum(np.searchsorted(oq.E2M1_GRID, y, side="left"), 7)]
    assert np.all((q == lo) | (q == hi))
    # values that already sit on the grid never move, whatever the draw
    grid_vals = np.tile(np.concatenate([oq.E2M1_GRID, -oq.E2M1_GRID]), (4, 1))     # amax 6 -> scale 1
    for seed in range(5):
        c, s = oq.quantize_sr(grid_vals, 1.0, seed=seed)
        assert np.array_equal(oq.dequantize(c, s, 1.0), grid_vals)


def test_sr_threshold_is_exact():
    # one block with amax 6 (scale 1): element 1 is 2.25 -> between 2 and 3, t = 0.25 exactly
    x = np.zeros((1, 16)); x[0, 0] = 6.0; x[0, 1] = 2.25; x[0, 2] = -0.125; x[0, 3] = 5.0
    def run(word):
        w = np.full((1, 16), word, dtype=np.uint32)
        c, s = oq.quantize_sr(x, 1.0, seed=0, words=w)
        return oq.dequantize(c, s, 1.0)[0]
    t_quarter = int(0.25 * 2 ** 24)
    assert run((t_quarter - 1) << 8)[1] == 3.0          # u just below t: up
    assert run(t_quarter << 8)[1] == 2.0                # u == t: down (strict comparison)
    assert run((t_quarter << 8) | 0xFF)[1] == 2.0       # the low 8 bits of the word are not used
    assert run(0)[2] == -0.5 and run(0)[3] == 6.0       # u = 0 < t: up, sign kept
    assert run(0xFFFFFFFF)[2] == -0.0 and run(0xFFFFFFFF)[3] == 4.0
    assert run(0)[0] == 6.0 and run(0xFFFFFFFF)[0] == 6.0


def test_sr_is_unbiased_and_uses_the_pinned_philox_stream():
    # the same value in every position: the mean over 2^16 independent draws approaches the value
    val = 2.6
    x = np.full((4096, 16), val); x[:, 0] = 6.0          # keeps every block's scale at 1
    codes, scales = oq.quantize_sr(x, 1.0, seed=2024)
    d = oq.dequantize(codes, scales, 1.0)[:, 1:]
    n = d.size
    p = 0.6                                              # (2.6 - 2) / (3 - 2)
    assert set(np.unique(d)) == {2.0, 3.0}
    assert abs(d.mean() - val) < 5 * np.sqrt(p * (1 - p) / n)
    # draws are the words of stream 3 at the elements' row-major positions
    w = orng.philox_words(2024, oq.STREAM_SR, 0, x.size).reshape(x.shape)
    u = (w >> 8) * 2.0 ** -24
    assert np.array_equal(d == 3.0, (2.0 + u < val)[:, 1:])
    # another seed or the transposed copy's stream gives other draws
    c2, _ = oq.quantize_sr(x, 1.0, seed=2025)
    c3, _ = oq.quantize_sr(x, 1.0, seed=2024, stream=oq.STREAM_SR_T)
    assert not np.array_equal(c2, codes) and not np.array_equal(c3, codes)


def test_sr_expected_error_beats_rne_bias_on_a_constant():
    # RNE maps 2.4 to 2 every time (bias -0.4); SR's mean stays at 2.4
    x = np.full((2048, 16), 2.4); x[:, 0] = 6.0
    c_rne, s_rne = oq.quantize(x, 1.0)
    c_sr, s_sr = oq.quantize_sr(x, 1.0, seed=9)
    assert np.all(oq.dequantize(c_rne, s_rne, 1.0)[:, 1:] == 2.0)
    assert abs(oq.dequantize(c_sr, s_sr, 1.0)[:, 1:].mean() - 2.4) < 0.01


def _exact_sr_block(block, g, words):
    """Stochastic rounding with exact rationals: scale as for nearest rounding; a = |e|/(s g) clipped at 6;
    between grid neighbours lo <= a < hi go up iff u < (a - lo)/(hi - lo), u = (word >> 8) / 2^24."""
    fr = [Fraction(float(v)) for v in block]
    sidx, _ = _exact_quantize_block(block, g)
    step = Fraction(float(quant.E4M3_POS[sidx])) * Fraction(float(g))
    grid = [Fraction(float(v)) for v in quant.E2M1_GRID]
    mags = []
    for v, w in zip(fr, words):
        if step == 0:
            mags.append(0)
            continue
        a = min(abs(v) / step, Fraction(6))
        lo_i = max(i for i in range(8) if grid[i] <= a)
        if lo_i == 7:
            mags.append(7)
            continue
        t = (a - grid[lo_i]) / (grid[lo_i + 1] - grid[lo_i])
        u = Fraction(int(w) >> 8, 2 ** 24)
        mags.append(lo_i + 1 if u < t else lo_i)
    return sidx, mags


def test_sr_against_exact_rationals_random_and_at_the_threshold():
    rs = np.random.default_rng(8)
    for g in (1.0, 2.0 ** -11):
        x = (rs.standard_normal((24, 32)) * np.exp(rs.uniform(-6, 6, (24, 1))) * g).astype(np.float32).astype(np.float64)
        w = rs.integers(0, 2 ** 32, x.shape, dtype=np.uint64).astype(np.uint32)
        codes, scales = oq.quantize_sr(x, g, seed=0, words=w)
        nib = _nibbles(codes)
        for i in range(x.shape[0]):
            for b in range(2):
                sl = slice(16 * b, 16 * b + 16)
                sidx, mags = _exact_sr_block(x[i, sl], g, w[i, sl])
                assert scales[i, b] == sidx and list(nib[i, sl] & 7) == mags
    # draws placed on the threshold of each element: floor(t 2^24) is the last u that does not go up ... unless t 2^24
    # is an integer, in which case u == t does not go up either (strict comparison); one below always goes up
    for sidx in (0x38, 0x3B, 0x45, 0x1D):
        s = float(quant.E4M3_POS[sidx])
        blk = (rs.uniform(0.01, 5.99, 16) * s).astype(np.float32).astype(np.float64)
        blk[0] = 6.0 * s
        step = Fraction(s)
        grid = [Fraction(float(v)) for v in quant.E2M1_GRID]
        words_hi, words_lo = [], []
        for v in blk:
            a = min(Fraction(float(v)) / step, Fraction(6))
            lo_i = max(i for i in range(8) if grid[i] <= a)
            t = (a - grid[lo_i]) / (grid[min(lo_i + 1, 7)] - grid[lo_i]) if lo_i < 7 else Fraction(0)
            n = (t * 2 ** 24).__ceil__()                       # smallest integer n with n / 2^24 >= t
            words_lo.append((max(n - 1, 0) << 8) & 0xFFFFFFFF)  # u < t (when t > 0): up
            words_hi.append((min(n, 2 ** 24 - 1) << 8) | 0xFF)  # u >= t: stays (unless clipped at the top draw)
        for words in (words_lo, words_hi):
            wa = np.array(words, dtype=np.uint32)[None, :]
            c, sc = oq.quantize_sr(blk[None, :], 1.0, seed=0, words=wa)
            ref_s, ref_m = _exact_sr_block(blk, 1.0, wa[0])
            assert sc[0, 0] == ref_s == sidx and list(_nibbles(c)[0] & 7) == ref_m
