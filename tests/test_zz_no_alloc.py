"""The entry point that allocates nothing: metis_split_quantize_static against metis_split_quantize, through
the C ABI, two calls in a row, the second on a smaller input (the shared scratch keeps the first call's bytes)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def metis():
    from paper_2509_00404_amd import metis as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def _factors(M, N, k, seed):
    gen = torch.Generator().manual_seed(seed)
    A = (torch.randn((M, k), generator=gen) @ torch.randn((k, N), generator=gen) * 0.1
         + torch.randn((M, N), generator=gen) * 0.05).to(torch.bfloat16)
    U, _ = torch.linalg.qr(torch.randn((M, k), generator=gen))
    V, _ = torch.linalg.qr(torch.randn((N, k), generator=gen))
    S = torch.sort(torch.rand((k,), generator=gen) * 3 + 0.1, descending=True).values
    return A.cuda(), U.contiguous().cuda(), S.cuda(), V.contiguous().cuda()


def _both(metis, M, N, k, seed, want_t):
    A, U, S, V = _factors(M, N, k, seed)
    g = metis.tensor_scale(float(A.abs().max()))
    ref = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, want_t)
    got = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, want_t)
    Rr = torch.empty((M, N), dtype=torch.float32, device="cuda")
    Rg = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    for t in (got.R, got.Ut, got.Vt) + ((got.Rt,) if want_t else ()):
        t.codes.fill_(0xA5)
        t.scales.fill_(0xA5)
    metis.split_quantize(A, U, S, V, ref, R_debug=Rr)
    metis.split_quantize_static(A, U, S, V, got, R_debug=Rg)
    torch.cuda.synchronize()
    return ref, got, Rr, Rg


def _same(ref, got, Rr, Rg, want_t):
    assert torch.equal(Rr, Rg)                       # the exact quantizer input, bit for bit
    pairs = [(ref.R, got.R), (ref.Ut, got.Ut), (ref.Vt, got.Vt)] + ([(ref.Rt, got.Rt)] if want_t else [])
    for a, b in pairs:
        assert torch.equal(a.codes, b.codes) and torch.equal(a.scales, b.scales)
    assert torch.equal(ref.S, got.S)


def test_static_scratch_matches_workspace_call_twice_second_smaller(metis):
    # first call: several tiles and ragged tails, rank padded 40 -> 64; second: smaller matrix, smaller padded rank
    first = _both(metis, 1168, 2096, 40, 1, True)
    _same(*first, True)
    second = _both(metis, 272, 336, 8, 2, True)
    _same(*second, True)
    # and without the debug dump (the whole-workgroup path), again smaller after larger
    for (M, N, k, seed) in ((2048, 4096, 64, 3), (256, 512, 16, 4)):
        A, U, S, V = _factors(M, N, k, seed)
        g = metis.tensor_scale(float(A.abs().max()))
        ref = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, False)
        got = metis.SplitTensor(M, N, k, 2.0 ** -11, 2.0 ** -11, g, False)
        metis.split_quantize(A, U, S, V, ref)
        metis.split_quantize_static(A, U, S, V, got)
        torch.cuda.synchronize()
        assert torch.equal(ref.R.codes, got.R.codes) and torch.equal(ref.R.scales, got.R.scales)
        assert torch.equal(ref.Ut.codes, got.Ut.codes) and torch.equal(ref.Vt.codes, got.Vt.codes)


def test_static_scratch_rejects_oversize_input_before_enqueueing(metis):
    M, N, k = 32768, 32768, 128                      # (M + N) * 4 * 128 = 32 MiB > 8 MiB
    assert metis.split_workspace_bytes(M, N, k) > metis.SPLIT_STATIC_SCRATCH_BYTES
    import ctypes as C
    a = metis.Mat(1, M, N, N, metis.BF16)            # never dereferenced: the size check comes first
    s = metis.Split()
    st = metis.lib().metis_split_quantize_static(None, C.byref(a), 1, 1, 1, k, C.byref(s), None)
    assert st == -6 and b"scratch" in metis.lib().metis_status_string(st)
