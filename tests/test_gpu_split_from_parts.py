"""GPU parity: the split of a weight from its stored parts (Sec. 3.2: for parameters the factors and
the residual are separate variables).  Codes and scales bit-exact against the oracle on the same
fp32 / bf16 inputs, for both rounding modes; then one pass of the persistent-weight path
(parts -> forward -> wgrad -> factor gradients) against the oracle end to end."""
import numpy as np
import pytest
import torch

from oracle import linear as olin
from oracle import quant as oq
from gpu_helpers import make_split, rel_fro, split_to_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def _parts(N, K, k, seed, dtype):
    g = torch.Generator().manual_seed(seed)
    U = torch.linalg.qr(torch.randn((N, k), generator=g, dtype=torch.float64))[0].float().contiguous()
    V = torch.linalg.qr(torch.randn((K, k), generator=g, dtype=torch.float64))[0].float().contiguous()
    S = (3.0 * torch.arange(1, k + 1, dtype=torch.float32) ** -1.0)
    WR = (0.02 * torch.randn((N, K), generator=g, dtype=torch.float32)
          * torch.exp(0.5 * torch.randn((1, K), generator=g, dtype=torch.float32))).to(dtype)
    return WR, U, S, V


def _same(a, b):
    return np.array_equal(a.codes.cpu().numpy(), b[0]) and np.array_equal(a.scales.cpu().numpy(), b[1])


@pytest.mark.parametrize("N,K,k,want_t", [(256, 512, 8, True), (144, 272, 5, True), (1040, 208, 64, True),
                                          (80, 96, 3, False), (2064, 144, 128, True)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("seed", [None, 77])
def test_split_from_parts_bit_exact(metis, N, K, k, want_t, dtype, seed):
    WR, U, S, V = _parts(N, K, k, N + K + k, dtype)
    g_r = oq.tensor_scale_for(float(WR.abs().max()))
    sp = metis.SplitTensor(N, K, k, 2.0 ** -11, 2.0 ** -11, g_r, want_t)
    sp.S.fill_(float("nan"))
    metis.split_from_parts(WR.cuda(), U.cuda(), S.cuda(), V.cuda(), sp, seed=seed)
    torch.cuda.synchronize()
    ref = olin.split_from_parts(WR.double().numpy(), U.double().numpy(), S.double().numpy(), V.double().numpy(),
                                2.0 ** -11, 2.0 ** -11, g_r, want_t=want_t, seed=seed)
    assert _same(sp.Ut, ref.Ut) and _same(sp.Vt, ref.Vt) and _same(sp.R, ref.R)
    if want_t:
        assert _same(sp.Rt, ref.Rt)
    assert np.array_equal(sp.S[:k].cpu().numpy(), S.numpy())


def test_persistent_weight_step(metis):
    """parts -> fwd -> wgrad -> factor gradients, each stage against the oracle on the same quantized operands."""
    from paper_2509_00404_amd import workloads
    L, N, K, k = 256, 384, 512, 16
    WR, U, S, V = _parts(N, K, k, 5, torch.bfloat16)
    g_r = oq.tensor_scale_for(float(WR.abs().max()))
    wsp = metis.SplitTensor(N, K, k, 2.0 ** -11, 2.0 ** -11, g_r, True)
    metis.split_from_parts(WR.cuda(), U.cuda(), S.cuda(), V.cuda(), wsp)
    X = workloads.planted(L, K, workloads.power_law(min(L, K), 1.2), 1, rms=1.0, outlier_cols=1)
    G = workloads.planted(L, N, workloads.power_law(min(L, N), 2.0, head=4, head_gain=100.0), 3, rms=1e-3)
    xs = make_split(metis, X, 0, 0, 1.0, 0)[0]
    gs = make_split(metis, G, 8, 8, 0.5, 9)[0]
    wsb = torch.empty((metis.linear_workspace_bytes(L, N, K, 16),), dtype=torch.uint8, device="cuda")
    Y = torch.empty((L, N), dtype=torch.float32, device="cuda")
    dW = torch.empty((N, K), dtype=torch.float32, device="cuda")
    metis.fp4_linear_fwd(xs, wsp, Y, wsb)
    metis.fp4_linear_wgrad(gs, xs, dW, wsb)
    dU = torch.empty((N, k), dtype=torch.float32, device="cuda")
    dS = torch.empty((k, k), dtype=torch.float32, device="cuda")
    dV = torch.empty((K, k), dtype=torch.float32, device="cuda")
    metis.fp4_factor_grads(dW, wsp, dU, dS, dV)
    torch.cuda.synchronize()
    xo, wo, go = split_to_oracle(xs), split_to_oracle(wsp), split_to_oracle(gs)
    assert rel_fro(Y.double().cpu().numpy(), olin.linear_fwd(xo, wo)) < 5e-3
    dWo = olin.linear_wgrad(go, xo)
    assert rel_fro(dW.double().cpu().numpy(), dWo) < 5e-3
    # factor gradients from the oracle's own dW: the GEMM's fp16-operand error carries through linearly
    for a, b in zip((dU, dS, dV), olin.factor_grads(dWo, wo)):
        assert rel_fro(a.double().cpu().numpy(), b) < 5e-3


def test_rejects_mismatched_parts(metis):
    WR, U, S, V = _parts(64, 96, 4, 1, torch.float32)
    sp = metis.SplitTensor(64, 112, 4, 2.0 ** -11, 2.0 ** -11, 2.0 ** -6, True)     # built for another width
    with pytest.raises(metis.MetisError):
        metis.split_from_parts(WR.cuda(), U.cuda(), S.cuda(), V.cuda(), sp)
