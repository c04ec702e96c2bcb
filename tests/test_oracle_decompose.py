"""Pins for oracle/decompose.py: planted low-rank recovery, the full-rank
special case against a brute-force Jacobi SVD, and the invariants that hold
for any input (Sec. 3.2: A = U S V^T + R with orthonormal factors)."""
import numpy as np
import pytest

from oracle import decompose as dec
from oracle import rng


def _haar(rs, n, q):
    q_, _ = np.linalg.qr(rs.standard_normal((n, q)))
    return q_


def _planted(rs, M, N, s):
    return (_haar(rs, M, len(s)) * s) @ _haar(rs, N, len(s)).T


def _jacobi_singular_values(A, sweeps=30):
    """Brute force: one-sided Jacobi (Hestenes) written out with scalar loops."""
    W = np.array(A, dtype=np.float64)
    n = W.shape[1]
    for _ in range(sweeps):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                a, b, c = W[:, p] @ W[:, p], W[:, q] @ W[:, q], W[:, p] @ W[:, q]
                if abs(c) <= 1e-300:
                    continue
                off = max(off, abs(c) / np.sqrt(a * b))
                z = (b - a) / (2 * c)
                t = np.sign(z) / (abs(z) + np.sqrt(1 + z * z)) if z != 0 else 1.0
                cs = 1 / np.sqrt(1 + t * t)
                sn = cs * t
                wp = cs * W[:, p] - sn * W[:, q]
                W[:, q] = sn * W[:, p] + cs * W[:, q]
                W[:, p] = wp
        if off < 1e-15:
            break
    return np.sort(np.linalg.norm(W, axis=0))[::-1]


def test_exact_recovery_of_planted_low_rank():
    rs = np.random.default_rng(0)
    s = np.array([50.0, 20.0, 7.0, 3.0, 1.0, 0.5])
    A = _planted(rs, 300, 120, s)
    U, S, V = dec.decompose(A, k=8, p=4, rho=0.25, seed=3)
    assert np.allclose(S[:6], s, rtol=1e-10)
    assert np.all(S[6:] < 1e-10)
    R = dec.residual(A, U, S, V)
    assert np.abs(R).max() < 1e-10
    # the recovered right space contains the planted one
    Vp = np.linalg.svd(A, full_matrices=False)[2][:6].T
    assert np.linalg.norm(Vp - V @ (V.T @ Vp)) < 1e-10


def test_full_rank_special_case_is_the_exact_svd():
    rs = np.random.default_rng(1)
    A = rs.standard_normal((40, 24))
    # rho = 1 and k + p = min(M, N): the sketch spans everything, result = thin SVD
    U, S, V = dec.decompose(A, k=24, p=0, rho=1.0, seed=9)
    assert np.allclose(S, _jacobi_singular_values(A), rtol=1e-11)
    assert np.abs(dec.residual(A, U, S, V)).max() < 1e-11
    # k < r: top-k of the exact SVD
    U, S, V = dec.decompose(A, k=5, p=19, rho=1.0, seed=9)
    sv = _jacobi_singular_values(A)
    assert np.allclose(S, sv[:5], rtol=1e-11)
    ev = np.linalg.eigvalsh(A.T @ A)[::-1]
    assert np.allclose(S ** 2, ev[:5], rtol=1e-10)
    # right singular vectors satisfy A^T A v = s^2 v
    assert np.abs(A.T @ (A @ V) - V * S ** 2).max() < 1e-10


@pytest.mark.parametrize("M,N,k,p,rho", [(256, 512, 8, 8, 0.25), (200, 96, 12, 4, 0.5), (64, 80, 4, 4, 1.0)])
def test_invariants_for_any_input(M, N, k, p, rho):
    rs = np.random.default_rng(2)
    s = 100.0 * np.arange(1, min(M, N) + 1) ** -1.5 + 0.01
    A = _planted(rs, M, N, s)
    U, S, V = dec.decompose(A, k, p, rho, seed=77)
    assert U.shape == (M, k) and S.shape == (k,) and V.shape == (N, k)
    I = np.eye(k)
    assert np.abs(U.T @ U - I).max() < 1e-12
    assert np.abs(V.T @ V - I).max() < 1e-12
    assert np.all(np.diff(S) <= 0) and np.all(S > 0)
    assert np.allclose(np.linalg.norm(A @ V, axis=0), S, rtol=1e-12)
    R = dec.residual(A, U, S, V)
    assert np.abs(R @ V).max() < 1e-10 * s[0]
    assert np.isclose((S ** 2).sum() + (R ** 2).sum(), (A ** 2).sum(), rtol=1e-12)
    assert np.abs((U * S) @ V.T + R - A).max() < 1e-12 * s[0]
    sv = np.linalg.svd(A, compute_uv=False)
    assert np.all(S <= sv[:k] * (1 + 1e-12))                 # Ritz values interlace
    # U diag(S) V^T is A projected on span(V)
    assert np.abs((U * S) @ V.T - A @ V @ V.T).max() < 1e-10 * s[0]
    # with a decaying spectrum the leading values are close to the true ones
    assert abs(S[0] - sv[0]) / sv[0] < 1e-3


def test_only_sampled_rows_decide_the_subspace():
    rs = np.random.default_rng(3)
    A = _planted(rs, 128, 64, 10.0 * np.arange(1, 65) ** -1.0)
    Ms = rng.sample_count(128, 4, 4, 0.25)
    idx = rng.sample_rows(5, 128, Ms)
    U1, S1, V1 = dec.decompose(A, 4, 4, 0.25, seed=5)
    A2 = A.copy()
    mask = np.ones(128, bool)
    mask[idx] = False
    A2[mask] *= 3.0                                           # change only unsampled rows
    U2, S2, V2 = dec.decompose(A2, 4, 4, 0.25, seed=5)
    assert dec.principal_angle(V1, V2) < 1e-7                 # same right subspace
    assert not np.allclose(S1, S2)                            # but the broadcast sees all rows


def test_explicit_draws_equal_seeded_draws():
    rs = np.random.default_rng(4)
    A = rs.standard_normal((96, 48))
    idx = rng.sample_rows(8, 96, rng.sample_count(96, 6, 2, 0.5))
    om = rng.gaussian_omega(8, 48, 8)
    a = dec.decompose(A, 6, 2, 0.5, seed=8)
    b = dec.decompose(A, 6, 2, 0.5, seed=0, idx=idx, omega=om)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_angle_and_alignment_metrics():
    e = np.eye(6)
    assert dec.principal_angle(e[:, :2], e[:, :2]) < 1e-12
    assert abs(dec.principal_angle(e[:, :2], e[:, 2:4]) - np.pi / 2) < 1e-7
    t = 0.3
    q = np.stack([np.cos(t) * e[:, 0] + np.sin(t) * e[:, 2], e[:, 1]], axis=1)
    assert abs(dec.principal_angle(e[:, :2], q) - t) < 1e-12
    assert np.isclose(dec.subspace_alignment(e[:, :2], q), (np.cos(t) ** 2 + 1) / 2)


def test_fix_signs():
    rs = np.random.default_rng(5)
    U, V = rs.standard_normal((10, 3)), rs.standard_normal((7, 3))
    U2, V2 = dec.fix_signs(U, V)
    assert np.all(V2[np.abs(V2).argmax(axis=0), np.arange(3)] > 0)
    assert np.allclose(U2 @ V2.T, U @ V.T)


def test_reduced_spectrum_report():
    # rho = 1 and k + p = min(M, N): the reduced matrix has the singular values of A itself
    rs = np.random.default_rng(21)
    A = _planted(rs, 40, 24, np.linspace(5.0, 0.1, 24))
    d = {}
    dec.decompose(A, 16, 8, 1.0, seed=3, details=d)
    assert np.allclose(d["sigma_reduced"], np.linalg.svd(A, compute_uv=False), rtol=1e-10)
    # in general they are r values, descending, bounded by the singular values of the sampled rows (interlacing)
    d = {}
    idx = np.arange(0, 40, 2)
    dec.decompose(A, 6, 4, 0.5, seed=4, idx=idx, details=d)
    sB = d["sigma_reduced"]
    sv = np.linalg.svd(A[idx], compute_uv=False)
    assert sB.shape == (10,) and np.all(np.diff(sB) <= 0) and np.all(sB <= sv[:10] * (1 + 1e-12))
