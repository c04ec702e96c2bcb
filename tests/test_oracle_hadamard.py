"""Pins for oracle/hadamard.py: a library Hadamard matrix, orthogonality, the inverse, product preservation."""
import numpy as np
from scipy.linalg import hadamard

from oracle import hadamard as had
from oracle import quant as oq
from oracle import rng as orng


def test_butterfly_is_the_sylvester_matrix_product():
    rs = np.random.default_rng(0)
    x = rs.standard_normal((7, 64))
    d = had.sign_vector(11)
    H = hadamard(16).astype(np.float64)
    assert np.array_equal(H @ H.T, 16 * np.eye(16))
    ref = ((x.reshape(7, 4, 16) * d) @ H / 4).reshape(7, 64)
    assert np.allclose(had.rht16(x, 11, np.float64), ref, rtol=1e-14, atol=1e-14)
    # in fp32 (the precision the quantizer sees) it is the same rotation to rounding
    assert np.allclose(had.rht16(x, 11), ref, rtol=0, atol=4 * 2.0 ** -24 * np.abs(x).max() * 4)


def test_signs_come_from_philox_stream_5_and_are_mixed():
    d = had.sign_vector(5)
    w = orng.philox_words(5, 5, 0, 16)
    assert np.array_equal(d < 0, (w >> 31).astype(bool))
    assert set(np.unique(np.concatenate([had.sign_vector(s) for s in range(8)]))) == {-1.0, 1.0}
    assert not np.array_equal(had.sign_vector(1), had.sign_vector(2))


def test_rotation_is_orthogonal_invertible_and_preserves_products():
    rs = np.random.default_rng(1)
    x, w = rs.standard_normal((5, 48)), rs.standard_normal((6, 48))
    zx, zw = had.rht16(x, 3, np.float64), had.rht16(w, 3, np.float64)
    assert np.allclose(np.linalg.norm(zx, axis=1), np.linalg.norm(x, axis=1))
    assert np.allclose(zx @ zw.T, x @ w.T, atol=1e-12)                  # both operands rotated along the contraction
    H = hadamard(16)
    back = ((zx.reshape(5, 3, 16) @ H.T / 4) * had.sign_vector(3)).reshape(5, 48)   # H symmetric, d its own inverse
    assert np.allclose(back, x, atol=1e-13)


def test_an_outlier_is_spread_over_its_block():
    x = np.zeros((1, 32))
    x[0, 5] = 8.0
    z = had.rht16(x, 9)
    assert np.all(np.abs(z[0, :16]) == 2.0) and np.all(z[0, 16:] == 0)


def test_quantize_rht_sr_is_the_sr_quantizer_of_the_rotated_values():
    rs = np.random.default_rng(2)
    x = rs.standard_normal((8, 64)).astype(np.float32).astype(np.float64)
    c, s = had.quantize_rht_sr(x, 2.0 ** -9, 17)
    c2, s2 = oq.quantize_sr(had.rht16(x, 17), 2.0 ** -9, 17)
    assert np.array_equal(c, c2) and np.array_equal(s, s2)
    # rotating back the dequantized values recovers x to quantization accuracy (block max step: amax / 6 * 1)
    d = oq.dequantize(c, s, 2.0 ** -9)
    H = hadamard(16)
    back = ((d.reshape(8, 4, 16) @ H.T / 4) * had.sign_vector(17)).reshape(8, 64)
    assert np.linalg.norm(back - x) / np.linalg.norm(x) < 0.25
