"""GPU parity of the MXFP4 variant: quantizer codes and scales bit-exact against the oracle, and the
block-scaled matrix-instruction GEMM against the oracle's fp64 product of the same quantized operands
(every product is exact and only the fp32 accumulation rounds: 1e-5 relative Frobenius)."""
import numpy as np
import pytest
import torch

from oracle import mx as omx
from gpu_helpers import rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def _data(M, K, seed, dtype):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn((M, K), generator=g) * torch.exp(1.5 * torch.randn((M, 1), generator=g))
    x[0, :8] = torch.tensor([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 7.0])      # grid midpoints and a saturating value
    x[0, 8:32] = 0.0
    x[0, 9] = 7.5
    if M > 2:
        x[1, 32:64] = 0.0                                                      # an all-zero block with a negative zero
        x[1, 40] = -0.0
        x[2, :32] = 2.0 ** -130                                               # below the fp32 normal range
    return x.to(dtype)


@pytest.mark.parametrize("M,K", [(128, 256), (77, 96), (1, 32), (513, 4096)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_quantize_mx_bit_exact(metis, M, K, dtype):
    x = _data(M, K, M + K, dtype)
    out = metis.MxTensor(M, K)
    metis.quantize_mx(x.cuda(), out)
    torch.cuda.synchronize()
    c, s = omx.quantize_mx(x.double().numpy())
    assert np.array_equal(out.scales.cpu().numpy(), s)
    assert np.array_equal(out.codes.cpu().numpy(), c)


@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (300, 200, 768), (1040, 528, 1024), (64, 1100, 512),
                                   # K not a multiple of the 256-deep stage: the tail variant (whole blocks of 32 only)
                                   (256, 256, 128), (300, 200, 384), (130, 70, 96), (520, 264, 1248)])
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_mxfp4_gemm_against_oracle(metis, M, N, K, out_dtype):
    a, b = _data(M, K, 1, torch.bfloat16), _data(N, K, 2, torch.bfloat16)
    qa, qb = metis.MxTensor(M, K), metis.MxTensor(N, K)
    metis.quantize_mx(a.cuda(), qa)
    metis.quantize_mx(b.cuda(), qb)
    Cm = torch.full((M, N), float("nan"), dtype=out_dtype, device="cuda")
    metis.mxfp4_gemm_nt(qa, qb, Cm)
    torch.cuda.synchronize()
    ref = omx.mx_gemm_nt((qa.codes.cpu().numpy(), qa.scales.cpu().numpy()), (qb.codes.cpu().numpy(), qb.scales.cpu().numpy()))
    got = Cm.double().cpu().numpy()
    assert np.isfinite(got).all()
    assert rel_fro(got, ref) < (1e-5 if out_dtype == torch.float32 else 4e-3)
    # and the quantized product approximates the unquantized one as FP4 does (~10 %)
    assert rel_fro(ref, a.double().numpy() @ b.double().numpy().T) < 0.25


def test_rejects_bad_arguments(metis):
    Cm = torch.empty((64, 64), dtype=torch.float32, device="cuda")
    qc = metis.MxTensor(64, 256)
    with pytest.raises(metis.MetisError):
        metis.mxfp4_gemm_nt(qc, metis.MxTensor(32, 512), Cm)
    with pytest.raises(metis.MetisError):
        metis.quantize_mx(torch.zeros((64, 64), dtype=torch.float32, device="cuda"), qc)
