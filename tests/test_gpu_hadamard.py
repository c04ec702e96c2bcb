"""GPU parity: random Hadamard rotation + stochastically rounded NVFP4 quantization, bit-exact against the oracle."""
import numpy as np
import pytest
import torch

from oracle import hadamard as ohad
from oracle import quant as oq

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


@pytest.mark.parametrize("M,N", [(1, 16), (37, 48), (300, 1040), (1024, 4096)])
def test_rotated_sr_codes_and_scales_bit_exact(metis, M, N):
    rs = np.random.default_rng(M + N)
    x = rs.standard_normal((M, N)) * np.exp(rs.uniform(-6, 4, (M, 1)))
    x[:, ::97] *= 20.0                                         # outlier channels
    x = torch.from_numpy(x).to(torch.bfloat16)
    for seed, g in ((5, 1.0), ((1 << 41) + 9, oq.tensor_scale_for(float(x.abs().max()) * 4))):
        out = metis.Fp4Tensor(M, N, g)
        metis.quantize_rht_sr(x.cuda(), seed, out)
        torch.cuda.synchronize()
        c, s = ohad.quantize_rht_sr(x.double().numpy(), g, seed)
        assert np.array_equal(out.scales.cpu().numpy(), s) and np.array_equal(out.codes.cpu().numpy(), c)


def test_rotation_keeps_the_product_and_spreads_outliers(metis):
    rs = np.random.default_rng(3)
    X = torch.from_numpy(rs.standard_normal((64, 256))).to(torch.bfloat16)
    W = torch.from_numpy(rs.standard_normal((32, 256)) * 0.05).to(torch.bfloat16)
    X[:, 7] *= 30.0
    qx, qw = metis.Fp4Tensor(64, 256, 2.0 ** -4), metis.Fp4Tensor(32, 256, 2.0 ** -8)
    metis.quantize_rht_sr(X.cuda(), 21, qx)
    metis.quantize_rht_sr(W.cuda(), 21, qw)
    torch.cuda.synchronize()
    dx = oq.dequantize(qx.codes.cpu().numpy(), qx.scales.cpu().numpy(), qx.tscale)
    dw = oq.dequantize(qw.codes.cpu().numpy(), qw.scales.cpu().numpy(), qw.tscale)
    ref = X.double().numpy() @ W.double().numpy().T
    err = np.linalg.norm(dx @ dw.T - ref) / np.linalg.norm(ref)
    assert err < 0.5                                   # same seed on both operands: the product survives (FP4 + SR noise)
    metis.quantize_rht_sr(W.cuda(), 22, qw)            # another sign vector on one operand: a different rotation
    torch.cuda.synchronize()
    dw2 = oq.dequantize(qw.codes.cpu().numpy(), qw.scales.cpu().numpy(), qw.tscale)
    assert np.linalg.norm(dx @ dw2.T - ref) / np.linalg.norm(ref) > 2 * err
    with pytest.raises(metis.MetisError):
        metis.quantize_rht_sr(X.float().cuda(), 1, qx)                       # bf16 input only
