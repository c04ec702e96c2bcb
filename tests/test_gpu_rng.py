"""GPU parity: Philox row sample (bit-exact) and Gaussian test matrix vs the oracle."""
import numpy as np
import pytest
import torch

from oracle import rng as orng

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


@pytest.mark.parametrize("M,Ms,seed", [(256, 64, 1), (8192, 512, 250900611), (1000, 77, 3), (97, 97, 4),
                                       (14336, 14336, 5), (16384, 1024, (1 << 40) + 17)])
def test_sample_rows_bit_exact(metis, M, Ms, seed):
    idx = metis.sample_rows(seed, M, Ms).cpu().numpy().view(np.uint32).astype(np.int64)
    assert np.array_equal(idx, orng.sample_rows(seed, M, Ms))


def test_sample_count_matches(metis):
    for M, k, p, rho in [(256, 8, 8, 0.25), (8192, 64, 16, 1 / 16), (8192, 64, 16, 0.01), (4096, 64, 16, 1.0),
                         (16384, 64, 16, 1 / 16), (1000, 3, 2, 0.333)]:
        assert metis.sample_count(M, k, p, rho) == orng.sample_count(M, k, p, rho)


@pytest.mark.parametrize("N,r,seed", [(512, 16, 7), (4096, 80, 250900611), (333, 7, (1 << 33) + 5)])
def test_omega_matches_oracle(metis, N, r, seed):
    # the oracle evaluates Box-Muller in fp64, the kernel in fp32: after rounding to bf16 the two
    # may differ by one bf16 ulp where the fp64 value sits next to a rounding boundary
    om = metis.gaussian_omega(seed, N, r).float().cpu().numpy().astype(np.float64)
    ref = orng.gaussian_omega(seed, N, r)
    diff = om != ref
    assert diff.mean() <= 1e-3
    ulp = np.maximum(np.abs(ref), 2.0 ** -126) * 2.0 ** -7
    # near the zero crossings of the cosine the fp32 argument reduction adds an absolute error
    assert np.all(np.abs(om - ref) <= ulp + 4e-6)


@pytest.mark.parametrize("M,group,k,p,rho", [(4096, 64, 8, 8, 1.0 / 16), (8192, 512, 64, 16, 1.0 / 16),
                                             (1024, 16, 64, 16, 0.01), (960, 32, 4, 4, 0.5), (256, 256, 8, 8, 0.1),
                                             (8192, 1, 64, 16, 1.0 / 16)])
def test_sequence_granular_sample_bit_exact(metis, M, group, k, p, rho):
    Ms = metis.sample_count(M, k, p, rho, group)
    assert Ms == orng.sample_count(M, k, p, rho, group)
    for seed in (3, (1 << 45) + 17):
        got = metis.sample_rows(seed, M, Ms, group=group).cpu().numpy().astype(np.int64) & 0xFFFFFFFF
        assert np.array_equal(got, orng.sample_rows(seed, M, Ms, group))
    with pytest.raises(metis.MetisError):
        metis.sample_rows(1, M + 1, Ms, group=2 if group == 1 else group)      # M not a multiple of the group
