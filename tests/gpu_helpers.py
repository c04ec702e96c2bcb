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
