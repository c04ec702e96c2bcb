"""GPU: the measurement kernels the bench quotes its ceilings from run, report their work, and reject bad arguments.
(No oracle here: they compute nothing of the method; the copy is checked byte for byte.)"""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def test_copy_and_read(metis):
    src = torch.randint(0, 256, (1 << 22,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    metis.ceiling_copy(src, dst)
    sink = torch.zeros(256 * 8, dtype=torch.int32, device="cuda")
    metis.ceiling_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_matrix_loops_report_their_flops(metis):
    sink = torch.zeros(512 * 256, dtype=torch.float32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    per_mfma = 2.0 * 32 * 32 * 16
    assert metis.ceiling_mfma(3, sink) == 512 * 4 * 3 * 8 * per_mfma
    for wps in (1, 2):
        for nv in (0, 2, 4, 5, 6, 8):
            assert metis.ceiling_mfma_mix(5, nv, wps, sink) == cus * wps * 4 * 5 * 4 * per_mfma
    # the GEMM's stage loop on registers: steps come in pairs, 16 matrix instructions each
    assert metis.ceiling_mfma_mix(5, metis.MIX_GEMM_EXPANSION, 1, sink) == cus * 4 * 6 * 16 * per_mfma
    assert metis.ceiling_mfma_mix(5, metis.MIX_GEMM_EXPANSION_FP6, 1, sink) == cus * 4 * 6 * 16 * per_mfma
    torch.cuda.synchronize()
    assert float(sink.abs().max()) == 0.0          # the sink is only there to keep the work alive


def test_bad_arguments(metis):
    sink = torch.zeros(512 * 256, dtype=torch.float32, device="cuda")
    for args in ((0, 4, 1), (5, 3, 1), (5, 4, 3), (5, metis.MIX_GEMM_EXPANSION, 2),
                 (5, metis.MIX_GEMM_EXPANSION_FP6, 2), (5, -3, 1)):
        with pytest.raises(metis.MetisError):
            metis.ceiling_mfma_mix(*args, sink)
