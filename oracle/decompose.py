"""Scalable spectral decomposition and split (Sec. 3.1, Sec. 3.2) -- oracle side.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

decompose() follows the paper's two-step procedure in its order: sample a few
rows, sketch them with a Gaussian test matrix, thin QR, top-k eigenspace in the
reduced space (randomized SVD of Halko et al., which the paper cites), then
"broadcast" that hidden-dimension subspace to all rows.  The factors are
finally put in singular-value form so that A = U diag(S) V^T + R with U, V
orthonormal and S descending, as Sec. 3.2 writes every split.

Readings (the paper gives two sentences and no algorithm for the composition
of sampling and projection; its dimensions in the projection paragraph are
inconsistent): the sample gives the RIGHT (hidden-dimension) subspace V0; the
broadcast is C = A V0 over all rows; no power iteration.
"""
import numpy as np
from . import rng


def decompose(A, k, p, rho, seed, idx=None, omega=None, details=None, group=1):
    """A[M,N] fp64 -> U[M,k], S[k], V[N,k].

    idx / omega override the seeded draws (used to feed identical draws to two
    implementations).  details (optional dict) receives by-products for reports:
    'sigma_reduced' = all k+p singular values of the reduced matrix B, whose gap
    between positions k and k+1 says how well defined the selected subspace is.
    group > 1: whole sequences of `group` consecutive rows are sampled (Sec. 3.1)."""
    A = np.asarray(A, dtype=np.float64)
    M, N = A.shape
    r = k + p
    if idx is None:
        Ms = rng.sample_count(M, k, p, rho, group)
        idx = rng.sample_rows(seed, M, Ms, group)
    if omega is None:
        omega = rng.gaussian_omega(seed, N, r)
    As = A[idx, :]                        # sparse random sampling of rows
    Z = As @ omega                        # sketch Z = X Omega
    H, _ = np.linalg.qr(Z)                # thin QR, Z = H R
    B = H.T @ As                          # reduced matrix  (r x N)
    _, sB, Vt = np.linalg.svd(B, full_matrices=False)
    if details is not None:
        details["sigma_reduced"] = sB
    V0 = Vt[:k, :].T                      # top-k subspace in the reduced space
    C = A @ V0                            # broadcast to the full batch
    U, S, Wt = np.linalg.svd(C, full_matrices=False)
    V = V0 @ Wt.T
    return U, S, V


def residual(A, U, S, V):
    """R = A - U diag(S) V^T (Sec. 3.2: W_R = W - U_k S_k V_k^T)."""
    return np.asarray(A, dtype=np.float64) - (U * S) @ V.T


def fix_signs(U, V):
    """Make each pair (u_i, v_i) unique: largest-magnitude entry of v_i > 0."""
    j = np.abs(V).argmax(axis=0)
    sg = np.sign(V[j, np.arange(V.shape[1])])
    sg[sg == 0] = 1.0
    return U * sg, V * sg


def principal_angle(Qa, Qb):
    """Largest principal angle (rad) between the column spaces of two
    orthonormal bases, via sin(theta_max) = ||(I - Qa Qa^T) Qb||_2."""
    Qa, _ = np.linalg.qr(Qa)
    Qb, _ = np.linalg.qr(Qb)
    D = Qb - Qa @ (Qa.T @ Qb)
    s = np.linalg.svd(D, compute_uv=False)
    return float(np.arcsin(min(1.0, s[0])))


def subspace_alignment(Qa, Qb):
    """Mean squared canonical correlation of two orthonormal bases (Sec. 3.1,
    the alignment measure of the sampling figure)."""
    return float(np.linalg.norm(Qa.T @ Qb, "fro") ** 2 / Qa.shape[1])
