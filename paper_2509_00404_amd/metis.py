"""ctypes binding of libmetis_hip.so (declared in include/metis.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream, every step of the path runs in the library's kernels.  There is no CPU
fallback: a missing library or a non-zero status raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmetis_hip.so")

BF16, F32 = 0, 1


class Mat(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("dtype", C.c_int)]


class Fp4(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scales", C.c_void_p), ("tscale", C.c_float),
                ("rows", C.c_int64), ("cols", C.c_int64)]


class Split(C.Structure):
    _fields_ = [("Ut", Fp4), ("Vt", Fp4), ("R", Fp4), ("Rt", Fp4), ("S", C.c_void_p), ("k", C.c_int)]


class MxFp4(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scales", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64)]


class DecomposeJob(C.Structure):
    _fields_ = [("A", C.POINTER(Mat)), ("k", C.c_int), ("oversample", C.c_int), ("sample_rate", C.c_double),
                ("seed", C.c_uint64), ("U", C.c_void_p), ("S", C.c_void_p), ("V", C.c_void_p), ("amax_out", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("idx", C.c_void_p), ("n_idx", C.c_int64),
                ("omega", C.c_void_p), ("info", C.c_void_p), ("split", C.POINTER(Split)), ("R_debug", C.c_void_p), ("sample_group", C.c_int64)]


class MetisError(RuntimeError):
    pass


_lib = None

_SIGNATURES = {
    "metis_status_string": (C.c_char_p, [C.c_int]),
    "metis_version": (C.c_int, []),
    "metis_tensor_scale": (C.c_float, [C.c_float]),
    "metis_sample_count": (C.c_int64, [C.c_int64, C.c_int, C.c_int, C.c_double]),
    "metis_sample_rows": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int64, C.c_int64, C.c_void_p]),
    "metis_sample_count_sequences": (C.c_int64, [C.c_int64, C.c_int, C.c_int, C.c_double, C.c_int64]),
    "metis_sample_sequences": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int64, C.c_int64, C.c_int64, C.c_void_p]),
    "metis_gaussian_omega": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int64, C.c_int, C.c_void_p]),
    "metis_decompose_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_double]),
    "metis_decompose": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_int, C.c_int, C.c_double, C.c_uint64,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                  C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]),
    "metis_decompose_split_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_double]),
    "metis_decompose_split_quantize": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_int, C.c_int, C.c_double, C.c_uint64,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Split),
                                                 C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_int64, C.c_void_p,
                                                 C.c_void_p]),
    "metis_decompose_batch": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(DecomposeJob)]),
    "metis_quantize": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.POINTER(Fp4), C.POINTER(Fp4)]),
    "metis_quantize_sr": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_uint64, C.POINTER(Fp4), C.POINTER(Fp4)]),
    "metis_quantize_rht_sr": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_uint64, C.POINTER(Fp4)]),
    "metis_split_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int]),
    "metis_split_quantize": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_int, C.POINTER(Split), C.c_void_p, C.c_void_p, C.c_size_t]),
    "metis_split_quantize_static": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_int, C.POINTER(Split), C.c_void_p]),
    "metis_split_quantize_sr": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_int, C.c_uint64, C.POINTER(Split), C.c_void_p, C.c_void_p, C.c_size_t]),
    "metis_split_from_parts": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                         C.POINTER(Split)]),
    "metis_split_from_parts_sr": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                            C.c_uint64, C.POINTER(Split)]),
    "metis_profile_events": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.c_int]),
    "metis_ceiling_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
    "metis_ceiling_read": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "metis_ceiling_mfma": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.POINTER(C.c_double)]),
    "metis_ceiling_mfma_mix": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double)]),
    "metis_linear_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int64, C.c_int]),
    "metis_fp4_linear_fwd": (C.c_int, [C.c_void_p, C.POINTER(Split), C.POINTER(Split), C.POINTER(Mat),
                                       C.c_void_p, C.c_size_t]),
    "metis_fp4_linear_dgrad": (C.c_int, [C.c_void_p, C.POINTER(Split), C.POINTER(Split), C.POINTER(Mat),
                                         C.c_void_p, C.c_size_t]),
    "metis_fp4_linear_wgrad": (C.c_int, [C.c_void_p, C.POINTER(Split), C.POINTER(Split), C.POINTER(Mat),
                                         C.c_void_p, C.c_size_t]),
    "metis_fp4_linear_phase": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(Split), C.POINTER(Split), C.POINTER(Mat),
                                        C.c_void_p, C.c_size_t]),
    "metis_quantize_mx": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.POINTER(MxFp4)]),
    "metis_mxfp4_gemm_nt": (C.c_int, [C.c_void_p, C.POINTER(MxFp4), C.POINTER(MxFp4), C.POINTER(Mat)]),
    "metis_factor_grads_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int]),
    "metis_fp4_factor_grads": (C.c_int, [C.c_void_p, C.POINTER(Mat), C.POINTER(Split), C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_size_t]),
}


def exported_symbols():
    """Names include/metis.h declares (the library must export every one)."""
    return sorted(_SIGNATURES)


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MetisError(f"{LIB_PATH} is not built; run: python -c 'import __graft_entry__ as g; g.build()'")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)          # AttributeError if the symbol is missing: fail loudly
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise MetisError(f"metis status {status}: {lib().metis_status_string(status).decode()}")


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _mat(t):
    assert t.is_cuda and t.dim() == 2 and t.stride(1) == 1
    dt = {torch.bfloat16: BF16, torch.float32: F32}[t.dtype]
    return Mat(t.data_ptr(), t.shape[0], t.shape[1], t.stride(0), dt)


class Fp4Tensor:
    """Device NVFP4 matrix: codes [rows, cols/2] u8, scales [rows, cols/16] u8, tscale."""

    def __init__(self, rows, cols, tscale, device="cuda"):
        self.rows, self.cols, self.tscale = rows, cols, float(tscale)
        self.codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=device)
        self.scales = torch.empty((rows, cols // 16), dtype=torch.uint8, device=device)

    def c(self):
        return Fp4(self.codes.data_ptr(), self.scales.data_ptr(), self.tscale, self.rows, self.cols)


def _null_fp4():
    return Fp4(None, None, 1.0, 0, 0)


class MxTensor:
    """Device MXFP4 matrix: codes [rows, cols/2] u8, scales [rows, cols/32] u8 (E8M0)."""

    def __init__(self, rows, cols, device="cuda"):
        self.rows, self.cols = rows, cols
        self.codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=device)
        self.scales = torch.empty((rows, cols // 32), dtype=torch.uint8, device=device)

    def c(self):
        return MxFp4(self.codes.data_ptr(), self.scales.data_ptr(), self.rows, self.cols)


class SplitTensor:
    """Device split-quantized operand of A[M,N] (see metis_split in include/metis.h)."""

    def __init__(self, M, N, k, g_u, g_v, g_r, want_t=True, device="cuda"):
        self.M, self.N, self.k = M, N, k
        self.Ut = Fp4Tensor(k, M, g_u, device) if k else None
        self.Vt = Fp4Tensor(k, N, g_v, device) if k else None
        self.R = Fp4Tensor(M, N, g_r, device)
        self.Rt = Fp4Tensor(N, M, g_r, device) if want_t else None
        self.S = torch.empty((max(k, 1),), dtype=torch.float32, device=device)

    def c(self):
        return Split(self.Ut.c() if self.Ut else _null_fp4(), self.Vt.c() if self.Vt else _null_fp4(),
                     self.R.c(), self.Rt.c() if self.Rt else _null_fp4(), self.S.data_ptr(), self.k)


def tensor_scale(amax):
    """Smallest power of two g with 6 * 448 * g >= amax (host helper of the library)."""
    return float(lib().metis_tensor_scale(float(amax)))


def sample_count(M, k, p, rho, group=1):
    return int(lib().metis_sample_count_sequences(M, k, p, rho, group))


def sample_rows(seed, M, Ms, device="cuda", group=1):
    """Row sample; group > 1 draws whole sequences of that many consecutive rows."""
    idx = torch.empty((Ms,), dtype=torch.int32, device=device)      # uint32 bits
    _check(lib().metis_sample_sequences(_stream(), seed, M, Ms, group, idx.data_ptr()))
    return idx


def gaussian_omega(seed, N, r, device="cuda"):
    om = torch.empty((N, r), dtype=torch.bfloat16, device=device)
    _check(lib().metis_gaussian_omega(_stream(), seed, N, r, om.data_ptr()))
    return om


def decompose_workspace_bytes(M, N, k, p, rho):
    return int(lib().metis_decompose_workspace_bytes(M, N, k, p, rho))


def decompose(A, k, oversample, sample_rate, seed, idx=None, omega=None, workspace=None,
              out=None, want_amax=False, info=None):
    """A[M,N] bf16 cuda -> (U[M,k], S[k], V[N,k]) fp32 (+ amax tensor when asked)."""
    M, N = A.shape
    if out is None:
        U = torch.empty((M, k), dtype=torch.float32, device=A.device)
        S = torch.empty((k,), dtype=torch.float32, device=A.device)
        V = torch.empty((N, k), dtype=torch.float32, device=A.device)
    else:
        U, S, V = out
    if workspace is None:
        nbytes = decompose_workspace_bytes(M, N, k, oversample, sample_rate)
        workspace = torch.empty((nbytes,), dtype=torch.uint8, device=A.device)
    amax = torch.empty((1,), dtype=torch.float32, device=A.device) if want_amax else None
    a = _mat(A)
    _check(lib().metis_decompose(
        _stream(), C.byref(a), k, oversample, sample_rate, seed, U.data_ptr(), S.data_ptr(), V.data_ptr(),
        amax.data_ptr() if want_amax else None, workspace.data_ptr(), workspace.numel(),
        idx.data_ptr() if idx is not None else None, idx.numel() if idx is not None else 0,
        omega.data_ptr() if omega is not None else None, info.data_ptr() if info is not None else None))
    return (U, S, V, amax) if want_amax else (U, S, V)


class DecomposeBatch:
    """Argument block of metis_decompose_batch, built once and reused: jobs = list of dicts with keys
    A, k, p, rho, seed, U, S, V, workspace and optionally amax, idx, omega, info (all tensors on the GPU)."""

    def __init__(self, jobs):
        self.keep = jobs                                   # the tensors stay alive with the block
        self.mats = [_mat(j["A"]) for j in jobs]
        self.splits = [j["split"].c() if j.get("split") is not None else None for j in jobs]
        self.arr = (DecomposeJob * len(jobs))()
        for a, m, sp, j in zip(self.arr, self.mats, self.splits, jobs):
            if sp is not None:                             # optional keys: split (SplitTensor), R_debug
                a.split = C.pointer(sp)
                a.R_debug = j["R_debug"].data_ptr() if j.get("R_debug") is not None else None
            ptr = lambda key: j[key].data_ptr() if j.get(key) is not None else None
            a.A = C.pointer(m)
            a.k, a.oversample, a.sample_rate, a.seed = j["k"], j["p"], j["rho"], j["seed"]
            a.U, a.S, a.V, a.amax_out = ptr("U"), ptr("S"), ptr("V"), ptr("amax")
            a.workspace, a.workspace_bytes = ptr("workspace"), j["workspace"].numel()
            a.idx, a.n_idx = ptr("idx"), (j["idx"].numel() if j.get("idx") is not None else 0)
            a.omega, a.info = ptr("omega"), ptr("info")
            a.sample_group = j.get("group", 1)

    def run(self):
        _check(lib().metis_decompose_batch(_stream(), len(self.arr), self.arr))


def decompose_split_workspace_bytes(M, N, k, p, rho):
    return int(lib().metis_decompose_split_workspace_bytes(M, N, k, p, rho))


def decompose_split_quantize(A, k, oversample, sample_rate, seed, out, R_debug=None, workspace=None, factors=None,
                             idx=None, omega=None, info=None):
    """Fused decomposition + split of A into `out` (SplitTensor); returns (U, S, V)."""
    M, N = A.shape
    if factors is None:
        U = torch.empty((M, k), dtype=torch.float32, device=A.device)
        S = torch.empty((k,), dtype=torch.float32, device=A.device)
        V = torch.empty((N, k), dtype=torch.float32, device=A.device)
    else:
        U, S, V = factors
    if workspace is None:
        workspace = torch.empty((decompose_split_workspace_bytes(M, N, k, oversample, sample_rate),), dtype=torch.uint8,
                                device=A.device)
    a, s = _mat(A), out.c()
    _check(lib().metis_decompose_split_quantize(
        _stream(), C.byref(a), k, oversample, sample_rate, seed, U.data_ptr(), S.data_ptr(), V.data_ptr(), None,
        C.byref(s), R_debug.data_ptr() if R_debug is not None else None, workspace.data_ptr(), workspace.numel(),
        idx.data_ptr() if idx is not None else None, idx.numel() if idx is not None else 0,
        omega.data_ptr() if omega is not None else None, info.data_ptr() if info is not None else None))
    return U, S, V


def quantize(A, out=None, out_t=None):
    """Plain NVFP4 quantization into out (blocks along cols) and/or out_t (A^T)."""
    a = _mat(A)
    o = out.c() if out is not None else None
    ot = out_t.c() if out_t is not None else None
    _check(lib().metis_quantize(_stream(), C.byref(a), C.byref(o) if o else None, C.byref(ot) if ot else None))


def quantize_sr(A, seed, out=None, out_t=None):
    """Stochastically rounded NVFP4 quantization (draws from Philox under `seed`)."""
    a = _mat(A)
    o = out.c() if out is not None else None
    ot = out_t.c() if out_t is not None else None
    _check(lib().metis_quantize_sr(_stream(), C.byref(a), int(seed), C.byref(o) if o else None,
                                   C.byref(ot) if ot else None))


def quantize_rht_sr(A, seed, out):
    """Random 16-point Hadamard rotation of every block, then stochastically rounded NVFP4 quantization."""
    a, o = _mat(A), out.c()
    _check(lib().metis_quantize_rht_sr(_stream(), C.byref(a), int(seed), C.byref(o)))


def split_workspace_bytes(M, N, k):
    return int(lib().metis_split_workspace_bytes(M, N, k))


def split_quantize(A, U, S, V, out, R_debug=None, workspace=None):
    a = _mat(A)
    s = out.c()
    if workspace is None:
        workspace = torch.empty((split_workspace_bytes(A.shape[0], A.shape[1], out.k),), dtype=torch.uint8,
                                device=A.device)
    _check(lib().metis_split_quantize(_stream(), C.byref(a), U.data_ptr(), S.data_ptr(), V.data_ptr(),
                                      out.k, C.byref(s), R_debug.data_ptr() if R_debug is not None else None,
                                      workspace.data_ptr(), workspace.numel()))


SPLIT_STATIC_SCRATCH_BYTES = 8 << 20


def split_quantize_static(A, U, S, V, out, R_debug=None):
    """split_quantize on the library's built-in scratch array (no workspace, no allocation)."""
    a = _mat(A)
    s = out.c()
    _check(lib().metis_split_quantize_static(_stream(), C.byref(a), U.data_ptr(), S.data_ptr(), V.data_ptr(),
                                             out.k, C.byref(s), R_debug.data_ptr() if R_debug is not None else None))


def split_quantize_sr(A, U, S, V, seed, out, R_debug=None, workspace=None):
    """split_quantize with stochastically rounded quantizers (draws from Philox under `seed`)."""
    a = _mat(A)
    s = out.c()
    if workspace is None:
        workspace = torch.empty((split_workspace_bytes(A.shape[0], A.shape[1], out.k),), dtype=torch.uint8,
                                device=A.device)
    _check(lib().metis_split_quantize_sr(_stream(), C.byref(a), U.data_ptr(), S.data_ptr(), V.data_ptr(),
                                         out.k, int(seed), C.byref(s),
                                         R_debug.data_ptr() if R_debug is not None else None,
                                         workspace.data_ptr(), workspace.numel()))


def split_from_parts(W_R, U, S, V, out, seed=None):
    """Quantize a weight's stored parts (factors U, V, residual W_R; S copied) into the split `out`;
    seed = None rounds to nearest, otherwise stochastically under that key."""
    a = _mat(W_R)
    s = out.c()
    assert all(t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 for t in (U, S, V))
    if seed is None:
        _check(lib().metis_split_from_parts(_stream(), C.byref(a), U.data_ptr(), S.data_ptr(), V.data_ptr(),
                                            out.k, C.byref(s)))
    else:
        _check(lib().metis_split_from_parts_sr(_stream(), C.byref(a), U.data_ptr(), S.data_ptr(), V.data_ptr(),
                                               out.k, int(seed), C.byref(s)))


def quantize_mx(A, out):
    a, o = _mat(A), out.c()
    _check(lib().metis_quantize_mx(_stream(), C.byref(a), C.byref(o)))
    return out


def mxfp4_gemm_nt(A, B, Cmat):
    """Cmat[M,N] = A[M,K] B[N,K]^T of two MxTensors."""
    a, b, c = A.c(), B.c(), _mat(Cmat)
    _check(lib().metis_mxfp4_gemm_nt(_stream(), C.byref(a), C.byref(b), C.byref(c)))
    return Cmat


def linear_workspace_bytes(L, N, K, k):
    return int(lib().metis_linear_workspace_bytes(L, N, K, k))


def _linear(fn, a, b, out, workspace):
    sa, sb, o = a.c(), b.c(), _mat(out)
    _check(fn(_stream(), C.byref(sa), C.byref(sb), C.byref(o),
              workspace.data_ptr() if workspace is not None else None,
              workspace.numel() if workspace is not None else 0))
    return out


LINEAR_FWD, LINEAR_DGRAD, LINEAR_WGRAD = 0, 1, 2
LINEAR_ALL, LINEAR_PREPARE, LINEAR_APPLY = 0, 1, 2


def fp4_linear_phase(product, phase, a, b, out, workspace):
    """One of the three products, whole or one of its two phases (see metis_fp4_linear_phase)."""
    sa, sb = a.c(), b.c()
    o = _mat(out) if out is not None else None
    _check(lib().metis_fp4_linear_phase(_stream(), product, phase, C.byref(sa), C.byref(sb), C.byref(o) if o is not None else None,
                                        workspace.data_ptr() if workspace is not None else None,
                                        workspace.numel() if workspace is not None else 0))
    return out


def fp4_linear_fwd(X, W, Y, workspace):
    return _linear(lib().metis_fp4_linear_fwd, X, W, Y, workspace)


def fp4_linear_dgrad(G, W, dX, workspace):
    return _linear(lib().metis_fp4_linear_dgrad, G, W, dX, workspace)


def fp4_linear_wgrad(G, X, dW, workspace):
    return _linear(lib().metis_fp4_linear_wgrad, G, X, dW, workspace)


def factor_grads_workspace_bytes(N, K, k):
    return int(lib().metis_factor_grads_workspace_bytes(N, K, k))


def fp4_factor_grads(dW, W, dU, dS, dV, workspace=None):
    """dU [N,k], dS [k,k], dV [K,k] (fp32, overwritten) from dW [N,K] and the quantized factors of W."""
    m, w = _mat(dW), W.c()
    assert all(t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 for t in (dU, dS, dV))
    if workspace is None:
        workspace = torch.empty((factor_grads_workspace_bytes(dW.shape[0], dW.shape[1], W.k),), dtype=torch.uint8,
                                device=dW.device)
    _check(lib().metis_fp4_factor_grads(_stream(), C.byref(m), C.byref(w), dU.data_ptr(), dS.data_ptr(),
                                        dV.data_ptr(), workspace.data_ptr(), workspace.numel()))
    return dU, dS, dV


def ceiling_copy(src, dst):
    _check(lib().metis_ceiling_copy(_stream(), src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size()))


def ceiling_read(src, sink):
    _check(lib().metis_ceiling_read(_stream(), src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr()))


def ceiling_mfma(iters, sink):
    """Launches the register-resident fp16 matrix-instruction loop; returns the launch's flop count."""
    fl = C.c_double()
    _check(lib().metis_ceiling_mfma(_stream(), iters, sink.data_ptr(), C.byref(fl)))
    return fl.value


MIX_GEMM_EXPANSION = -1      # valu_per_mfma: run the GEMM's own expansion + matrix instructions on registers
MIX_GEMM_EXPANSION_FP6 = -2  # ... with the codes in 6-bit containers and the 32-wide FP6 converter


def ceiling_mfma_mix(iters, valu_per_mfma, waves_per_simd, sink):
    """Matrix instructions interleaved with vector instructions (see metis_ceiling_mfma_mix); returns the flop count."""
    fl = C.c_double()
    _check(lib().metis_ceiling_mfma_mix(_stream(), iters, valu_per_mfma, waves_per_simd, sink.data_ptr(), C.byref(fl)))
    return fl.value


PROF_GEMM, PROF_BROADCAST, PROF_RESIDUAL_QUANT, PROF_QUANTIZE = 0, 1, 2, 3


class KernelTimer:
    """HIP events around every launch of one hot kernel (metis_profile_events)."""

    def __init__(self, kernel_id, n):
        self.kernel_id, self.n = kernel_id, n
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.hip.hipEventCreate.restype = C.c_int
        self.hip.hipEventElapsedTime.restype = C.c_int
        self.hip.hipEventDestroy.restype = C.c_int
        self.hip.hipGetLastError.restype = C.c_int
        self.start = (C.c_void_p * n)()
        self.stop = (C.c_void_p * n)()
        for arr in (self.start, self.stop):
            for i in range(n):
                ev = C.c_void_p()
                if self.hip.hipEventCreate(C.byref(ev)) != 0:
                    raise MetisError("hipEventCreate failed")
                arr[i] = ev

    def __enter__(self):
        _check(lib().metis_profile_events(self.kernel_id, self.start, self.stop, self.n))
        return self

    def __exit__(self, *exc):
        _check(lib().metis_profile_events(self.kernel_id, None, None, 0))

    def close(self):
        """Destroy the events (after the last durations_ms call)."""
        for arr in (self.start, self.stop):
            for i in range(self.n):
                if arr[i]:
                    self.hip.hipEventDestroy(arr[i])
                    arr[i] = None
        self.n = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def durations_ms(self, count):
        """Durations of the first `count` (<= n) bracketed launches since the timer was switched on, stopping at
        the first pair that was never recorded; call after a device sync."""
        out = []
        for i in range(min(count, self.n)):
            ms = C.c_float()
            if self.hip.hipEventElapsedTime(C.byref(ms), self.start[i], self.stop[i]) != 0:
                self.hip.hipGetLastError()                  # an unrecorded pair: clear the error it left behind
                break
            out.append(ms.value)
        return out
