"""GPU parity: stochastically rounded NVFP4 codes and scales bit-exact against the oracle
(same inputs, same seed: both sides draw the same Philox words)."""
import numpy as np
import pytest
import torch

from oracle import quant as oq

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def _check(metis, x, g, seed, transposed=False, both=False):
    M, N = x.shape
    out = metis.Fp4Tensor(M, N, g) if (not transposed or both) else None
    out_t = metis.Fp4Tensor(N, M, g) if (transposed or both) else None
    metis.quantize_sr(x.cuda(), seed, out, out_t)
    torch.cuda.synchronize()
    xn = x.double().numpy()
    if out is not None:
        c, s = oq.quantize_sr(xn, g, seed, oq.STREAM_SR)
        assert np.array_equal(out.scales.cpu().numpy(), s)
        assert np.array_equal(out.codes.cpu().numpy(), c)
    if out_t is not None:
        c, s = oq.quantize_sr(np.ascontiguousarray(xn.T), g, seed, oq.STREAM_SR_T)
        assert np.array_equal(out_t.scales.cpu().numpy(), s)
        assert np.array_equal(out_t.codes.cpu().numpy(), c)


@pytest.mark.parametrize("M,N", [(128, 512), (1, 16), (37, 48), (300, 1040), (1024, 4096)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_rows_random(metis, M, N, dtype):
    rs = np.random.default_rng(M * 11 + N)
    x = rs.standard_normal((M, N)) * np.exp(rs.uniform(-12, 6, (M, 1)))
    x = torch.from_numpy(x).to(dtype)
    g = oq.tensor_scale_for(float(x.abs().max()))
    _check(metis, x, g, seed=M + 17 * N)
    _check(metis, x, 1.0, seed=(1 << 40) + 5)


@pytest.mark.parametrize("M,N", [(64, 64), (16, 48), (144, 80), (512, 1040)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_transposed_and_both(metis, M, N, dtype):
    rs = np.random.default_rng(M + 3 * N)
    x = torch.from_numpy(rs.standard_normal((M, N)) * np.exp(rs.uniform(-4, 4, (M, N)))).to(dtype)
    g = oq.tensor_scale_for(float(x.abs().max()))
    _check(metis, x, g, seed=77, transposed=True)
    _check(metis, x, g, seed=78, both=True)


def test_draws_at_the_threshold_and_inputs_next_to_grid_points(metis):
    # probability t = (|x|/(s g) - lo)/(hi - lo) in real arithmetic: fp32 inputs with full significands (t is not
    # an fp32-rounded value) and inputs a few ulp around every grid point * s, many seeds' worth of draws
    rs = np.random.default_rng(5)
    rows = []
    for sidx in range(9, 120, 3):
        step = oq.E4M3_POS[sidx]
        gridp = (oq.E2M1_GRID[1:] * step).astype(np.float32)
        for k in (-2, -1, 0, 1, 2):
            v = np.minimum((gridp.view(np.int32) + k).view(np.float32), np.float32(6 * step))
            fill = (rs.uniform(0.0, 6.0, 8) * step).astype(np.float32)
            rows.append(np.concatenate([[6 * step], v, -fill]).astype(np.float32))
    x = torch.from_numpy(np.array(rows).repeat(16, axis=0))     # the same row under 16 different word offsets
    for seed in (1, 2, 3):
        _check(metis, x, 1.0, seed)
    big = (rs.uniform(-6, 6, (2048, 1024)) * np.exp(rs.uniform(-2, 2, (2048, 64)).repeat(16, axis=1))).astype(np.float32)
    _check(metis, torch.from_numpy(big), oq.tensor_scale_for(float(np.abs(big).max())), seed=123456789, both=True)


def test_degenerate_blocks(metis):
    # all-zero blocks, signed zeros, grid points, saturated blocks (amax above 6*448*g)
    x = torch.zeros(16, 64)
    x[1, 5] = -0.0
    x[2, :16] = torch.tensor([0, .5, 1, 1.5, 2, 3, 4, 6, -0.5, -1, -1.5, -2, -3, -4, -6, 6.0])
    x[3, 16:32] = 1e6
    x[3, 17] = -3e5
    x[4, :] = torch.linspace(-6, 6, 64)
    for seed in (0, 1, 2):
        _check(metis, x, 1.0, seed)
        _check(metis, x.to(torch.bfloat16), 2.0 ** -4, seed, both=True)


def test_unbiased_and_seed_dependent(metis):
    x = torch.full((4096, 64), 2.4)
    x[:, ::16] = 6.0
    out = metis.Fp4Tensor(4096, 64, 1.0)
    out2 = metis.Fp4Tensor(4096, 64, 1.0)
    metis.quantize_sr(x.cuda(), 5, out)
    metis.quantize_sr(x.cuda(), 6, out2)
    torch.cuda.synchronize()
    d = oq.dequantize(out.codes.cpu().numpy(), out.scales.cpu().numpy(), 1.0)
    keep = np.ones(64, bool); keep[::16] = False
    assert abs(d[:, keep].mean() - np.float32(2.4)) < 5e-3
    assert not np.array_equal(out.codes.cpu().numpy(), out2.codes.cpu().numpy())
