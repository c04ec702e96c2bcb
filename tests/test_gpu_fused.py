"""GPU parity of the fused decomposition + split (metis_decompose_split_quantize): one pass over A in HBM, the
residual taken as A - (A V0) V0^T band by band.  Checked against the oracle exactly as the two-call path is:
singular values and subspaces of U, S, V, the residual against fp64 from the returned factors, codes and scales
bit-exact on the kernel's own quantizer input (both orientations), and against the two-call path's outputs."""
import numpy as np
import pytest
import torch

from oracle import decompose as odec
from oracle import quant as oq

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def _run(metis, A, k, p, rho, seed, want_t):
    M, N = A.shape
    Ad = A.cuda()
    g = metis.tensor_scale(float(A.abs().max()))
    fused = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, want_t)
    Rd = torch.empty((M, N), dtype=torch.float32, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    U, S, V = metis.decompose_split_quantize(Ad, k, p, rho, seed, fused, R_debug=Rd, info=info)
    two = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, want_t)
    U2, S2, V2 = metis.decompose(Ad, k, p, rho, seed)
    metis.split_quantize(Ad, U2, S2, V2, two)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    return fused, two, (U, S, V), (U2, S2, V2), Rd, g


@pytest.mark.parametrize("M,N,k,p,rho,want_t", [(1168, 2096, 40, 8, 0.5, True),       # one band, ragged tiles
                                                (256, 512, 8, 8, 0.25, False),         # config 1's shape
                                                (4992, 14336, 64, 16, 1.0 / 16, True)])  # three bands (2304 rows each)
def test_fused_split_matches_oracle_and_two_call_path(metis, M, N, k, p, rho, want_t):
    from paper_2509_00404_amd import workloads
    A = workloads.planted(M, N, workloads.power_law(min(M, N, 512), 1.2), M + N, rms=1.0, outlier_cols=2)
    seed = 77
    fused, two, (U, S, V), (U2, S2, V2), Rd, g = _run(metis, A, k, p, rho, seed, want_t)
    An = A.double().numpy()
    Un, Sn, Vn = (t.double().cpu().numpy() for t in (U, S, V))
    # factors against the oracle (its own seeded draws: the two Gaussian matrices differ in < 1e-3 of entries by an ulp)
    Ur, Sr, Vr = odec.decompose(An, k, p, rho, seed)
    assert np.max(np.abs(Sn - Sr) / Sr) < 1e-3
    assert odec.principal_angle(Vn, Vr) < 1e-2 and odec.principal_angle(Un, Ur) < 1e-2
    # same factors as the two-call path (same kernels; a band's broadcast may cut its contraction differently)
    assert np.max(np.abs(Sn - S2.double().cpu().numpy()) / Sn) < 1e-5
    # the quantizer's input is the residual of the returned factors
    R = Rd.double().cpu().numpy()
    assert np.linalg.norm(R - (An - (Un * Sn) @ Vn.T)) <= 1e-4 * np.linalg.norm(An)
    # codes and scales bit-exact on that input, every row and (transposed copy) every column
    c, s = oq.quantize(R, g)
    assert np.array_equal(fused.R.codes.cpu().numpy(), c) and np.array_equal(fused.R.scales.cpu().numpy(), s)
    if want_t:
        c, s = oq.quantize(np.ascontiguousarray(R.T), g)
        assert np.array_equal(fused.Rt.codes.cpu().numpy(), c) and np.array_equal(fused.Rt.scales.cpu().numpy(), s)
    for fac, q in ((Un, fused.Ut), (Vn, fused.Vt)):
        c, s = oq.quantize(np.ascontiguousarray(fac.T), q.tscale)
        assert np.array_equal(q.codes.cpu().numpy(), c) and np.array_equal(q.scales.cpu().numpy(), s)
    assert torch.equal(fused.S[:k], S)
    # against the two-call path: the same residual up to fp32 rounding, so almost all code bytes agree
    # (a value or a block maximum within ~2^-16 of the low-rank part's magnitude of a threshold may fall either way)
    diff = (fused.R.codes != two.R.codes).float().mean().item()
    sdiff = (fused.R.scales != two.R.scales).float().mean().item()
    print("fused vs two-call: differing code bytes %.2e, scale bytes %.2e" % (diff, sdiff))
    assert diff < 2e-3 and sdiff < 2e-3


def test_fused_split_in_a_batch_and_argument_errors(metis):
    from paper_2509_00404_amd import workloads
    jobs, refs = [], []
    for i, (M, N, k, p, rho) in enumerate([(512, 1024, 16, 8, 0.5), (768, 512, 64, 16, 1.0)]):
        A = workloads.planted(M, N, workloads.power_law(min(M, N), 1.1), 50 + i, rms=1.0).cuda()
        g = metis.tensor_scale(float(A.abs().max()))
        sp = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, True)
        ws = torch.empty((metis.decompose_split_workspace_bytes(M, N, k, p, rho),), dtype=torch.uint8, device="cuda")
        jobs.append(dict(A=A, k=k, p=p, rho=rho, seed=5 + i, workspace=ws, split=sp,
                         U=torch.empty((M, k), device="cuda"), S=torch.empty((k,), device="cuda"),
                         V=torch.empty((N, k), device="cuda")))
        ref = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, True)
        metis.decompose_split_quantize(A, k, p, rho, 5 + i, ref)
        refs.append(ref)
    metis.DecomposeBatch(jobs).run()
    torch.cuda.synchronize()
    for j, ref in zip(jobs, refs):
        assert (j["split"].R.codes != ref.R.codes).float().mean().item() < 2e-3
        assert (j["split"].Rt.codes != ref.Rt.codes).float().mean().item() < 2e-3
        assert (j["split"].Ut.codes != ref.Ut.codes).float().mean().item() < 2e-2
    # a workspace sized for the plain decomposition is refused
    A = jobs[0]["A"]
    small = torch.empty((metis.decompose_workspace_bytes(512, 1024, 16, 8, 0.5),), dtype=torch.uint8, device="cuda")
    with pytest.raises(metis.MetisError):
        metis.decompose_split_quantize(A, 16, 8, 0.5, 1, jobs[0]["split"], workspace=small)
    with pytest.raises(metis.MetisError):                                  # split of another shape
        metis.decompose_split_quantize(A, 16, 8, 0.5, 1, jobs[1]["split"])
