"""Pins of the MXFP4 oracle quantizer against the published conversion rule and against the
NVFP4 oracle where the two formats coincide (no GPU)."""
import math

import numpy as np

from oracle import mx
from oracle import quant

GRID = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def _nibbles(codes):
    out = np.empty((codes.shape[0], codes.shape[1] * 2), dtype=np.int64)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


def test_scale_rule_worked_values():
    # amax in [4, 8) * 2^e -> X = 2^e: 5 -> 1, 7.9 -> 1 (and 7.9 saturates to 6), 8 -> 2, 0.3 -> 2^-4
    for amax, want_x, want_top in [(5.0, 1.0, 4.0), (7.9, 1.0, 6.0), (8.0, 2.0, 8.0), (0.3, 2.0 ** -4, 0.25),
                                   (6.0, 1.0, 6.0), (3.999, 0.5, 3.0)]:     # 3.999 / 0.5 = 7.998 saturates to 6
        x = np.zeros((1, 32))
        x[0, 5] = -amax
        c, s = mx.quantize_mx(x)
        assert 2.0 ** (int(s[0, 0]) - 127) == want_x, amax
        assert mx.dequantize_mx(c, s)[0, 5] == -want_top, amax


def test_values_on_the_grid_round_trip_for_every_exponent():
    rs = np.random.default_rng(0)
    for e in (-126, -40, -3, 0, 7, 100, 125):
        v = np.array(GRID)[rs.integers(0, 8, (4, 64))] * rs.choice([-1.0, 1.0], (4, 64))
        v[:, 0] = 6.0
        v[:, 32] = -4.0                       # amax 4 also selects X = 2^e
        x = v * 2.0 ** e
        c, s = mx.quantize_mx(x)
        assert np.all(s == e + 127)
        assert np.array_equal(mx.dequantize_mx(c, s), x)


def test_brute_force_nearest_with_ties_to_even_and_saturation():
    rs = np.random.default_rng(1)
    x = rs.standard_normal((6, 96)) * np.exp(rs.standard_normal((6, 96)))
    x[0, :8] = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 7.0]     # midpoints of the grid at X = 1 (7 saturates) ...
    x[0, 8] = 7.5                                               # ... and amax in [4, 8) keeps X = 1
    x[0, 9:32] = 0.0
    c, s = mx.quantize_mx(x)
    nib = _nibbles(c)
    signed = [(m, g) for m, g in enumerate(GRID)]
    for r in range(x.shape[0]):
        for b in range(x.shape[1] // 32):
            blk = x[r, 32 * b:32 * b + 32]
            amax = np.abs(blk).max()
            m_, ex = math.frexp(amax)
            X = 2.0 ** (ex - 1 - 2)
            assert int(s[r, b]) - 127 == ex - 3
            for i, v in enumerate(blk):
                q = abs(v) / X
                best = min(signed, key=lambda t: (abs(t[1] - q), t[0] & 1))    # nearest; on a tie the even code
                got = nib[r, 32 * b + i]
                assert (got & 7) == best[0], (r, b, i, v)
                assert (got >> 3) == (1 if np.signbit(v) else 0)
    assert list(nib[0, :9] & 7) == [0, 2, 2, 4, 4, 6, 6, 7, 7]


def test_error_bound():
    rs = np.random.default_rng(2)
    x = rs.standard_normal((16, 256)) * 10.0 ** rs.uniform(-3, 3, (16, 1))
    c, s = mx.quantize_mx(x)
    X = 2.0 ** (s.astype(np.float64) - 127)
    err = np.abs(mx.dequantize_mx(c, s) - x).reshape(16, 8, 32)
    q = np.abs(x).reshape(16, 8, 32) / X[:, :, None]
    # half the local grid spacing below 6, plus the saturated range (6, 8)
    bound = np.where(q <= 2, 0.25, np.where(q <= 4, 0.5, np.where(q <= 6, 1.0, 2.0))) * X[:, :, None]
    assert np.all(err <= bound)


def test_zero_block_and_signs():
    x = np.zeros((2, 64))
    x[1, 40] = -0.0
    c, s = mx.quantize_mx(x)
    assert np.all(s == 0)
    nib = _nibbles(c)
    assert nib[1, 40] == 8 and nib.sum() == 8
    assert np.all(mx.dequantize_mx(c, s) == 0.0)


def test_coincides_with_nvfp4_when_the_block_maximum_is_six_times_a_power_of_two():
    # amax = 6 * 2^e in both 16-element halves: NVFP4 (g = 1) picks the E4M3 scale 2^e, MX picks X = 2^e
    rs = np.random.default_rng(3)
    x = rs.uniform(-6, 6, (8, 64))
    x[:, 3::16] = 6.0
    x *= 0.25
    c_mx, s_mx = mx.quantize_mx(x)
    c_nv, s_nv = quant.quantize(x, 1.0)
    assert np.array_equal(c_mx, c_nv)
    assert np.all(quant.e4m3_value(s_nv) == 0.25) and np.all(s_mx == 125)


def test_gemm_of_lossless_operands_is_the_plain_product():
    rs = np.random.default_rng(4)
    def lossless(m, n):
        a = np.array(GRID)[rs.integers(0, 8, (m, n))] * rs.choice([-1.0, 1.0], (m, n))
        a[:, ::32] = 6.0
        return a * 0.5
    A, B = lossless(24, 96), lossless(40, 96)
    assert np.array_equal(mx.mx_gemm_nt(mx.quantize_mx(A), mx.quantize_mx(B)), A @ B.T)
