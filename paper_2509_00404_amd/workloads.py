"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds none of the method's arithmetic: only matrices with a planted singular
spectrum, shaped like the LLaMA-3-8B linears the paper trains (Sec. 4), which
stand in for the paper's DCLM-trained tensors (few dominant singular values,
Sec. 2.1; activation outlier channels).  Everything is generated on the CPU
with numpy's PCG64 so the same seed gives the same matrix everywhere, and is
returned as a torch bfloat16 CPU tensor.
"""
import numpy as np
import torch

BASE_SEED = 250900404


def _orth(rng, n, q):
    g = rng.standard_normal((n, q), dtype=np.float32)
    qmat, _ = np.linalg.qr(g)
    return qmat


def planted(M, N, spectrum, seed, noise_top=0.0, rms=None, outlier_cols=0, outlier_gain=20.0):
    """A = U0 diag(spectrum) V0^T (+ iid Gaussian noise whose largest singular
    value is ~noise_top), rescaled to the requested RMS, then `outlier_cols`
    randomly chosen columns multiplied by `outlier_gain`; cast to bf16."""
    rng = np.random.default_rng(seed)
    s = np.asarray(spectrum, dtype=np.float32)
    q = s.shape[0]
    U0 = _orth(rng, M, q)
    V0 = _orth(rng, N, q)
    A = torch.from_numpy(U0 * s) @ torch.from_numpy(V0).T
    if noise_top > 0.0:
        sigma = noise_top / (np.sqrt(M) + np.sqrt(N))
        A += torch.from_numpy(rng.standard_normal((M, N), dtype=np.float32)) * float(sigma)
    if rms is not None:
        A *= float(rms) / float(A.pow(2).mean().sqrt())
    if outlier_cols > 0:
        cols = rng.choice(N, size=outlier_cols, replace=False)
        A[:, torch.from_numpy(cols)] *= outlier_gain
    return A.to(torch.bfloat16)


def power_law(q, alpha, head=0, head_gain=1.0):
    i = np.arange(1, q + 1, dtype=np.float64)
    s = i ** (-alpha)
    s[:head] *= head_gain
    return s


def weight(N, K, seed, alpha=1.0):
    """Weight W[N,K]: s_i = i^-alpha, RMS 0.02, Gaussian noise floor at 1% of s_1."""
    q = min(N, K, 1024)
    s = power_law(q, alpha)
    return planted(N, K, s, seed, noise_top=0.01 * s[0], rms=0.02)


def activation(L, K, seed, alpha=1.2):
    """Activations X[L,K]: s_i = i^-alpha, RMS 1, 0.1% outlier channels at 20x."""
    q = min(L, K, 1024)
    return planted(L, K, power_law(q, alpha), seed, rms=1.0,
                   outlier_cols=max(1, round(K / 1000)), outlier_gain=20.0)


def gradient(L, N, seed, alpha=2.0):
    """Output gradient G[L,N]: steep spectrum, top-4 singular values 100x, RMS 1e-3."""
    q = min(L, N, 1024)
    return planted(L, N, power_law(q, alpha, head=4, head_gain=100.0), seed, rms=1e-3)


def tiny_planted(seed, M=256, N=512):
    """Config 1: s_i = 100 i^-1.5 + 0.01, full rank."""
    q = min(M, N)
    i = np.arange(1, q + 1, dtype=np.float64)
    return planted(M, N, 100.0 * i ** -1.5 + 0.01, seed)


def gaussian(L, K, seed):
    rng = np.random.default_rng(seed)
    return torch.from_numpy(rng.standard_normal((L, K), dtype=np.float32)).to(torch.bfloat16)


def seed_for(config, tensor_id):
    return BASE_SEED + 100 * config + tensor_id


# k, p, sample rates per config
PARAMS = {
    1: dict(k=8, p=8, rho_w=0.25, rho_x=0.25),
    2: dict(k=64, p=16, rho_w=1.0, rho_x=1.0 / 16),
    3: dict(k=64, p=16, rho_w=1.0, rho_x=1.0 / 16),
    4: dict(k=64, p=16, rho_w=1.0, rho_x=1.0 / 16),
    5: dict(k=64, p=16, rho_w=1.0, rho_x=1.0 / 16),
}


def config(c):
    """Tensors of benchmark configuration c (1..4) as a dict of bf16 CPU tensors.

    1: A 256x512 planted (decomposed, used as the weight), X 128x512 N(0,1)
    2: W 4096x4096, X 8192x4096
    3: W 14336x4096, X 8192x4096
    4: W 4096x14336, X 8192x14336, G 8192x4096
    """
    if c == 1:
        return dict(W=tiny_planted(seed_for(1, 0)), X=gaussian(128, 512, seed_for(1, 1)))
    if c == 2:
        return dict(W=weight(4096, 4096, seed_for(2, 0)), X=activation(8192, 4096, seed_for(2, 1)))
    if c == 3:
        return dict(W=weight(14336, 4096, seed_for(3, 0)), X=activation(8192, 4096, seed_for(3, 1)))
    if c == 4:
        return dict(W=weight(4096, 14336, seed_for(4, 0)), X=activation(8192, 14336, seed_for(4, 1)),
                    G=gradient(8192, 4096, seed_for(4, 2)))
    raise ValueError("config must be 1..4 (config 5 is built per linear by layer_linear)")


# Config 5: (name, N, K) of one LLaMA-3-8B layer's seven linears (k and v are 1024 wide under GQA)
LAYER_LINEARS = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                 ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]
LAYER_TOKENS = 16384


def layer_linear(name, L=LAYER_TOKENS):
    """One linear of config 5 as an independent (X, W, G) triple with its own seeds:
    W[N,K] (alpha = 1.0), X[L,K] (alpha = 1.2, outlier channels), G[L,N] (alpha = 2.0, top-4 x100).
    Tensor ids 10 i + {0: W, 1: X, 2: G} for the i-th linear, so seed_for(5, id) + 7 is its library seed."""
    i = [n for n, _, _ in LAYER_LINEARS].index(name)
    _, N, K = LAYER_LINEARS[i]
    return dict(W=weight(N, K, seed_for(5, 10 * i)), X=activation(L, K, seed_for(5, 10 * i + 1)),
                G=gradient(L, N, seed_for(5, 10 * i + 2)))


def layer_seed(name, tensor):
    """Library seed of tensor 'W' / 'X' / 'G' of config 5's linear `name`."""
    i = [n for n, _, _ in LAYER_LINEARS].index(name)
    return seed_for(5, 10 * i + "WXG".index(tensor)) + 7
