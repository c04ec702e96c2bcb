"""fprop / dgrad / wgrad on split-quantized operands (Sec. 3.2) -- oracle side.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Layout (PyTorch convention): X[L,K] activations, W[N,K] weight (out x in, the
transpose of the paper's W), Y = X W^T [L,N], G = dL/dY [L,N].
A split operand holds Q(U), S (unquantized, Sec. 3.2: singular values are kept
in high precision), Q(V) and Q(R).  The quantized operand is
    Abar = deq(Q(U)) diag(S) deq(Q(V))^T + deq(Q(R))
and the three products are plain fp64 matmuls of those (the paper's own
emulation is dequantize-then-multiply, App. C.1):
    fwd   Y  = Xbar Wbar^T      (Eq. 2)
    dgrad dX = Gbar Wbar        (Eq. 3)
    wgrad dW = Gbar^T Xbar      (the dL/dW_R line after Eq. 3, transposed)

Blocks of 16 lie along the contraction axis of the consuming GEMM (a reading:
the paper does not say).  A residual used by two GEMMs is therefore quantized
twice from the same unquantized residual, once along each axis; `R` below is
quantized along the columns of A, `Rt` is the transpose quantized along the
rows of A.  Factors are quantized along their long axis (each singular vector
contiguous).
"""
import numpy as np
from . import quant


class SplitQ:
    """Quantized split of one matrix A[M,N]; every member is plain numpy.

    Ut: (codes, scales, g) of U^T [k,M];  Vt: of V^T [k,N];
    R : of R [M,N] (blocks along N);      Rt: of R^T [N,M] (blocks along M);
    S : fp64 [k].  k == 0 means "not split": R holds Q(A)."""

    def __init__(self, Ut, S, Vt, R, Rt):
        self.Ut, self.S, self.Vt, self.R, self.Rt = Ut, S, Vt, R, Rt


def split_quantize(A, U, S, V, g_u, g_v, g_r, want_t=True):
    """Q_b applied separately to U, V and R, not to S (Sec. 3.2 before Eq. 2)."""
    from .decompose import residual
    A = np.asarray(A, dtype=np.float64)
    if U is None or U.shape[1] == 0:
        R = A
        Ut = Vt = None
        S = np.zeros(0)
    else:
        R = residual(A, U, S, V)
        Ut = quant.quantize(U.T, g_u) + (g_u,)
        Vt = quant.quantize(V.T, g_v) + (g_v,)
    Rq = quant.quantize(R, g_r) + (g_r,)
    Rtq = quant.quantize(R.T, g_r) + (g_r,) if want_t else None
    return SplitQ(Ut, np.asarray(S, dtype=np.float64), Vt, Rq, Rtq)


def split_quantize_sr(A, U, S, V, g_u, g_v, g_r, seed, want_t=True):
    """split_quantize with the stochastically rounded quantizer (Sec. 4: SR is the default of the FP4
    runs).  Readings of this build: the residual draws from `seed` (stream 3 for R, stream 4 for the
    transposed copy), Q(U^T) from `seed + 1` and Q(V^T) from `seed + 2` (both transposed copies, stream 4),
    so that no two tensors share draws."""
    from .decompose import residual
    A = np.asarray(A, dtype=np.float64)
    if U is None or U.shape[1] == 0:
        R = A
        Ut = Vt = None
        S = np.zeros(0)
    else:
        R = residual(A, U, S, V)
        Ut = quant.quantize_sr(np.ascontiguousarray(U.T), g_u, seed + 1, quant.STREAM_SR_T) + (g_u,)
        Vt = quant.quantize_sr(np.ascontiguousarray(V.T), g_v, seed + 2, quant.STREAM_SR_T) + (g_v,)
    Rq = quant.quantize_sr(R, g_r, seed, quant.STREAM_SR) + (g_r,)
    Rtq = quant.quantize_sr(np.ascontiguousarray(R.T), g_r, seed, quant.STREAM_SR_T) + (g_r,) if want_t else None
    return SplitQ(Ut, np.asarray(S, dtype=np.float64), Vt, Rq, Rtq)


def split_from_parts(W_R, U, S, V, g_u, g_v, g_r, want_t=True, seed=None):
    """Quantized split of a weight whose parts are stored, not recomputed (Sec. 3.2: for parameters the
    low-rank factors and the residual are separate trainable variables): Q_b on U, V and the given W_R,
    S untouched.  No subtraction happens here, W_R is taken as it is.  seed = None rounds to nearest;
    otherwise the stochastic quantizer with the same keys as split_quantize_sr."""
    W_R = np.asarray(W_R, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    if seed is None:
        Ut = quant.quantize(U.T, g_u) + (g_u,)
        Vt = quant.quantize(V.T, g_v) + (g_v,)
        Rq = quant.quantize(W_R, g_r) + (g_r,)
        Rtq = quant.quantize(W_R.T, g_r) + (g_r,) if want_t else None
    else:
        Ut = quant.quantize_sr(np.ascontiguousarray(U.T), g_u, seed + 1, quant.STREAM_SR_T) + (g_u,)
        Vt = quant.quantize_sr(np.ascontiguousarray(V.T), g_v, seed + 2, quant.STREAM_SR_T) + (g_v,)
        Rq = quant.quantize_sr(W_R, g_r, seed, quant.STREAM_SR) + (g_r,)
        Rtq = quant.quantize_sr(np.ascontiguousarray(W_R.T), g_r, seed, quant.STREAM_SR_T) + (g_r,) if want_t else None
    return SplitQ(Ut, np.asarray(S, dtype=np.float64), Vt, Rq, Rtq)


def assemble(sq, transposed_residual=False):
    """Abar [M,N] from a SplitQ, using R (blocks along N) or Rt (blocks along M)."""
    if transposed_residual:
        Rb = quant.dequantize(*sq.Rt).T
    else:
        Rb = quant.dequantize(*sq.R)
    if sq.Ut is None:
        return Rb
    Ub = quant.dequantize(*sq.Ut).T
    Vb = quant.dequantize(*sq.Vt).T
    return (Ub * sq.S) @ Vb.T + Rb


def _take(M, rows):
    return M if rows is None else M[np.asarray(rows)]


def linear_fwd(xq, wq, rows=None):
    """Y = Xbar Wbar^T; contraction over K: X_R and W_R blocked along K.
    rows (optional): only these rows of Y (the same product, fewer output rows)."""
    return _take(assemble(xq), rows) @ assemble(wq).T


def linear_dgrad(gq, wq, rows=None):
    """dX = Gbar Wbar; contraction over N: G_R blocked along N (its columns),
    W_R blocked along N (its rows -> Rt).  rows: only these rows of dX."""
    return _take(assemble(gq), rows) @ assemble(wq, transposed_residual=True)


def linear_wgrad(gq, xq, rows=None):
    """dW = Gbar^T Xbar; contraction over L: both residuals blocked along rows.
    rows: only these rows of dW."""
    return _take(assemble(gq, transposed_residual=True).T, rows) @ assemble(xq, transposed_residual=True)


def factor_grads(dW, wq):
    """Gradients of the weight's low-rank factors (Sec. 3.2, backward pass, the formulas after Eq. 3).

    Layout of this build: W[N,K] = U S V^T + W_R with U [N,k], V [K,k] (the paper writes Y = X W with
    W [m,n], so its U_k is this V and its V_k is this U), dW[N,K] = dL/dW = Gbar^T Xbar as returned
    by linear_wgrad.  With the quantized factors Ubar, Vbar and the unquantized S:
        dL/dU = dW Vbar S          [N,k]
        dL/dS = Ubar^T dW Vbar     [k,k]   (the paper's k x k expression, transposed to this layout)
        dL/dV = dW^T Ubar S        [K,k]
    which are the paper's four-term sums with Xbar^T (P T Q^T + D_R) collected into dW.
    Returns (dU, dS, dV) in fp64.
    """
    dW = np.asarray(dW, dtype=np.float64)
    Ub = quant.dequantize(*wq.Ut).T          # [N,k]
    Vb = quant.dequantize(*wq.Vt).T          # [K,k]
    S = np.asarray(wq.S, dtype=np.float64)
    T = dW @ Vb
    return T * S, Ub.T @ T, (dW.T @ Ub) * S


def linear_fwd_expanded(xq, wq):
    """Eq. 2 written out term by term (used only to pin linear_fwd)."""
    XR = quant.dequantize(*xq.R)
    WR = quant.dequantize(*wq.R)
    Y = XR @ WR.T
    have_x, have_w = xq.Ut is not None, wq.Ut is not None
    if have_x:
        Ax = quant.dequantize(*xq.Ut).T
        Bx = quant.dequantize(*xq.Vt).T
    if have_w:
        Uw = quant.dequantize(*wq.Ut).T      # [N,k]: left factor of W[N,K]
        Vw = quant.dequantize(*wq.Vt).T      # [K,k]
    if have_w:
        Y = Y + ((XR @ Vw) * wq.S) @ Uw.T
    if have_x:
        Y = Y + (Ax * xq.S) @ (Bx.T @ WR.T)
    if have_x and have_w:
        Y = Y + ((Ax * xq.S) @ (Bx.T @ Vw) * wq.S) @ Uw.T
    return Y
