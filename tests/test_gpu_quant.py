"""GPU parity: NVFP4 codes and scales bit-exact against the oracle on identical inputs."""
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


def _check(metis, x, g, transposed=False, both=False):
    M, N = x.shape
    xd = x.cuda()
    out = metis.Fp4Tensor(M, N, g) if (not transposed or both) else None
    out_t = metis.Fp4Tensor(N, M, g) if (transposed or both) else None
    metis.quantize(xd, out, out_t)
    torch.cuda.synchronize()
    xn = x.double().numpy()
    if out is not None:
        c, s = oq.quantize(xn, g)
        assert np.array_equal(out.scales.cpu().numpy(), s)
        assert np.array_equal(out.codes.cpu().numpy(), c)
    if out_t is not None:
        c, s = oq.quantize(xn.T, g)
        assert np.array_equal(out_t.scales.cpu().numpy(), s)
        assert np.array_equal(out_t.codes.cpu().numpy(), c)


@pytest.mark.parametrize("M,N", [(128, 512), (1, 16), (37, 48), (300, 1040), (2048, 4096)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_rows_random(metis, M, N, dtype):
    rs = np.random.default_rng(M * 7 + N)
    x = rs.standard_normal((M, N)) * np.exp(rs.uniform(-12, 6, (M, 1)))
    x = torch.from_numpy(x).to(dtype)
    g = oq.tensor_scale_for(float(x.abs().max()))
    _check(metis, x, g)
    _check(metis, x, 1.0)


@pytest.mark.parametrize("M,N", [(64, 64), (16, 48), (144, 80), (1024, 2064)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_transposed_and_both(metis, M, N, dtype):
    rs = np.random.default_rng(M + N)
    x = torch.from_numpy(rs.standard_normal((M, N)) * np.exp(rs.uniform(-4, 4, (M, N)))).to(dtype)
    g = oq.tensor_scale_for(float(x.abs().max()))
    _check(metis, x, g, transposed=True)
    _check(metis, x, g, both=True)


def test_every_scale_and_every_tie(metis):
    # row b: block scale index b (1..126); elements sit on the rounding midpoints and next to them
    rows = []
    for sidx in range(1, 127):
        s = oq.E4M3_POS[sidx]
        mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]) * s
        blk = np.concatenate([[6 * s], mids, -mids, [0.0]])
        near = np.concatenate([[-6 * s], np.nextafter(mids.astype(np.float32), np.float32(0)),
                               np.nextafter(mids.astype(np.float32), np.float32(np.inf)), [-0.0]])
        rows.append(np.concatenate([blk, near]))
    x = torch.from_numpy(np.array(rows)).to(torch.float32)
    _check(metis, x, 1.0)
    _check(metis, x * 2.0 ** -11, 2.0 ** -11)


def test_fp32_inputs_within_a_few_ulp_of_every_threshold(metis):
    # real-arithmetic round(e / (s g)): fp32 inputs k ulp (k = -3..3) from midpoint * s * g for every scale, with
    # and without mantissa bits; the kernel's fp32 quotient must decide every one of them as exact arithmetic does
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    for g in (1.0, 2.0 ** -11):
        rows = []
        for sidx in range(1, 127):
            step = oq.E4M3_POS[sidx] * g
            t = (mids * step).astype(np.float32)
            for k in range(-3, 4):
                v = (t.view(np.int32) + k).view(np.float32)
                sign = -1.0 if (k + sidx) % 2 else 1.0
                rows.append(np.concatenate([[6 * step], v * sign, -v * sign, [step]]).astype(np.float32))
        x = torch.from_numpy(np.array(rows))
        _check(metis, x, g)


def test_fp32_random_mantissas_large(metis):
    # two million fp32 values with full 24-bit significands spread over many block scales
    rs = np.random.default_rng(99)
    x = (rs.standard_normal((1024, 2048)) * np.exp(rs.uniform(-3, 3, (1024, 128)).repeat(16, axis=1))).astype(np.float32)
    _check(metis, torch.from_numpy(x), oq.tensor_scale_for(float(np.abs(x).max())))


def test_all_bf16_magnitudes(metis):
    # every finite non-negative bf16 pattern, shuffled into blocks
    bits = np.arange(0, 0x7F80, dtype=np.uint32)
    vals = (bits << 16).view(np.float32)
    vals = vals[(vals < 2.0 ** 14) & (vals > 2.0 ** -30)]
    n = (len(vals) // 512) * 512
    rs = np.random.default_rng(0)
    v = rs.permutation(vals[:n]) * rs.choice([-1.0, 1.0], n).astype(np.float32)
    x = torch.from_numpy(v.reshape(-1, 512)).to(torch.bfloat16)
    _check(metis, x, 1.0)
    _check(metis, x, 2.0 ** -3)


def test_zero_saturation_and_strided_input(metis):
    x = torch.zeros((32, 64), dtype=torch.bfloat16)
    x[0, 3] = -0.0
    x[1, :16] = 1e9
    x[1, 5] = -1e9
    x[2, 16:32] = 2.0 ** -20
    _check(metis, x, 1.0)
    big = torch.randn((64, 256), dtype=torch.bfloat16)
    view = big[:, 64:192]                       # ld != cols
    out = metis.Fp4Tensor(64, 128, 2.0 ** -9)
    metis.quantize(view.cuda()[:, :], out) if False else None
    vd = big.cuda()[:, 64:192]
    metis.quantize(vd, out)
    torch.cuda.synchronize()
    c, s = oq.quantize(view.double().numpy(), 2.0 ** -9)
    assert np.array_equal(out.codes.cpu().numpy(), c) and np.array_equal(out.scales.cpu().numpy(), s)


def test_argument_errors(metis):
    x = torch.zeros((16, 24), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(metis.MetisError):
        metis.quantize(x, metis.Fp4Tensor(16, 32, 1.0))            # cols not a multiple of 16 / mismatch
    y = torch.zeros((16, 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(metis.MetisError):
        metis.quantize(y, metis.Fp4Tensor(16, 32, 3.0))            # tensor scale not a power of two
    with pytest.raises(metis.MetisError):
        metis.quantize(y[:8], None, metis.Fp4Tensor(32, 8, 1.0))   # rows not a multiple of 16
