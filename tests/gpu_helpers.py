"""Helpers shared by the GPU parity tests: move quantized operands to the oracle's types."""
import numpy as np
import torch

from oracle import linear as olin
from oracle import quant as oq


def fp4_to_oracle(t):
    """metis.Fp4Tensor -> (codes, scales, g) numpy triple of the oracle."""
    return (t.codes.cpu().numpy(), t.scales.cpu().numpy(), t.tscale)


def split_to_oracle(sp):
    """metis.SplitTensor -> oracle SplitQ holding the SAME codes, scales and S."""
    Ut = fp4_to_oracle(sp.Ut) if sp.k else None
    Vt = fp4_to_oracle(sp.Vt) if sp.k else None
    S = sp.S[:sp.k].double().cpu().numpy() if sp.k else np.zeros(0)
    return olin.SplitQ(Ut, S, Vt, fp4_to_oracle(sp.R), fp4_to_oracle(sp.Rt) if sp.Rt is not None else None)


def make_split(metis, A, k, p, rho, seed, want_t=True, headroom=1.0):
    """decompose + split_quantize on the GPU; returns (SplitTensor, U, S, V, R_debug)."""
    Ad = A.cuda()
    M, N = A.shape
    g_r = oq.tensor_scale_for(float(A.abs().max()), headroom)
    if k == 0:
        sp = metis.SplitTensor(M, N, 0, 1.0, 1.0, g_r, want_t)
        metis.quantize(Ad, sp.R, sp.Rt)
        return sp, None, None, None, None
    U, S, V = metis.decompose(Ad, k, p, rho, seed)
    sp = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g_r, want_t)
    Rd = torch.empty((M, N), dtype=torch.float32, device="cuda")
    metis.split_quantize(Ad, U, S, V, sp, R_debug=Rd)
    torch.cuda.synchronize()
    return sp, U, S, V, Rd


def rel_fro(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


# ---- element-wise bound for the split GEMMs ---------------------------------------------------------
# The kernels compute Abar Bbar^T as R_a R_b^T + E1 U_b^T + U_a (E2 S_a)^T with fp32 accumulation, where
# E1 = (R_a V_b + U_a S_a V_a^T V_b) S_b and E2 S_a = (R_b V_a) S_a are rounded once to bf16 (2^-9) and the
# result is rounded to the output type.  With |.| taken element-wise,
#   |got - ref| <= 2 ulp_out |ref| + 2 * 2^-9 L1 + (K + 2k) 2^-24 (|R_a| |R_b|^T + L1),
#   L1 = |E1| |U_b|^T + |U_a| |E2 S_a|^T,
# the last term being the worst-case bound of an fp32 sum of K + 2k exact products.

def operand_parts(sq, transposed=False):
    """Dense fp64 parts of an oracle SplitQ seen as a [rows, contraction] GEMM operand:
    R [rows, K], U [rows, k], S [k], V [K, k] (U, S, V None when the operand is not split)."""
    if transposed:
        R = oq.dequantize(*sq.Rt)
        U, V = sq.Vt, sq.Ut
    else:
        R = oq.dequantize(*sq.R)
        U, V = sq.Ut, sq.Vt
    if sq.Ut is None:
        return R, None, None, None
    return R, oq.dequantize(*U).T, np.asarray(sq.S, dtype=np.float64), oq.dequantize(*V).T


def elementwise_bound(a_parts, b_parts, ref, out_dtype):
    Ra, Ua, Sa, Va = a_parts
    Rb, Ub, Sb, Vb = b_parts
    K = Ra.shape[1]
    kk = 0
    L1 = np.zeros_like(ref)
    if Ub is not None:
        E1 = Ra @ Vb
        if Ua is not None:
            E1 = E1 + (Ua * Sa) @ (Va.T @ Vb)
        L1 += np.abs(E1 * Sb) @ np.abs(Ub).T
        kk += Ub.shape[1]
    if Ua is not None:
        L1 += np.abs(Ua) @ np.abs((Rb @ Va) * Sa).T
        kk += Ua.shape[1]
    ulp_out = 2.0 ** -9 if out_dtype == torch.bfloat16 else 2.0 ** -24
    bound = 2 * ulp_out * np.abs(ref) + 2 * 2.0 ** -9 * L1 + (K + kk) * 2.0 ** -24 * (np.abs(Ra) @ np.abs(Rb).T + L1)
    return bound + np.finfo(np.float64).tiny              # an all-zero row stays comparable (0 <= tiny)


def take_row_groups(sq, groups):
    """Oracle SplitQ of the rows 16 g .. 16 g + 15 (g in groups) of a split matrix: rows of R and, because U^T is
    blocked along those rows in groups of 16, whole blocks of U^T (8 code bytes + 1 scale byte per factor row).
    Pure data selection; Rt is dropped."""
    groups = np.asarray(groups)
    rows = (16 * groups[:, None] + np.arange(16)[None, :]).ravel()
    R = (sq.R[0][rows], sq.R[1][rows], sq.R[2])
    Ut = None
    if sq.Ut is not None:
        cb = (8 * groups[:, None] + np.arange(8)[None, :]).ravel()
        Ut = (sq.Ut[0][:, cb], sq.Ut[1][:, groups], sq.Ut[2])
    return olin.SplitQ(Ut, sq.S, sq.Vt, R, None), rows
