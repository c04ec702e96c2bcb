// metis_decompose: sampled randomized SVD + broadcast + singular-value form
// (Sec. 3.1 "Scalable Spectral Decomposition", Sec. 3.2 for the form of the split).
//
// Sample stage (touches only the l_k sampled rows and (k+p)-sized matrices) runs in fp64
// on the f64 matrix cores: the Gram-based steps (CholeskyQR2, eigen-decomposition of
// B B^T) square the condition number of the sketch.  The one pass over all rows
// (C = A V0) runs on the bf16 matrix cores with V0 split in two bf16 parts.
#include "broadcast.h"
#include "dgemm.h"
#include "dgemm_skinny.h"
#include "smallmat.h"
#include "rng_dev.h"

namespace {

struct Layout {
    int64_t M, N, Ms;
    int k, r;
    size_t off_zacc, off_g1, off_g1b, off_g2, off_g3, off_flag, off_c, off_b, zero_bytes;
    size_t off_idx, off_omega, off_linv, off_h1, off_h, off_lam, off_t, off_v0f, off_v0hi, off_v0lo,
        off_lam3, off_w3, off_t3, off_jscr, total;
};

Layout make_layout(int64_t M, int64_t N, int k, int p, int64_t Ms) {
    Layout L;
    L.M = M; L.N = N; L.Ms = Ms; L.k = k; L.r = k + p;
    const size_t r = (size_t)L.r, kk = (size_t)k;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.off_zacc = take((size_t)Ms * r * 8);
    L.off_g1 = take(r * r * 8);
    L.off_g1b = take(r * r * 8);
    L.off_g2 = take(r * r * 8);
    L.off_g3 = take(kk * kk * 8);
    L.off_flag = take(4);
    L.off_b = take(r * (size_t)N * 8);
    L.zero_bytes = o;
    L.off_c = take((size_t)broadcast_splits(M, N) * (size_t)M * kk * 4);
    L.off_idx = take((size_t)Ms * 4);
    L.off_omega = take((size_t)N * r * 2);
    L.off_linv = take(r * r * 8);
    L.off_h1 = take((size_t)Ms * r * 8);
    L.off_h = take((size_t)Ms * r * 8);
    L.off_lam = take(r * 8);
    L.off_t = take(r * kk * 8);
    L.off_v0f = take((size_t)N * kk * 4);
    L.off_v0hi = take((size_t)N * kk * 2);
    L.off_v0lo = take((size_t)N * kk * 2);
    L.off_lam3 = take(kk * 8);
    L.off_w3 = take(kk * kk * 8);
    L.off_t3 = take(kk * kk * 8);
    L.off_jscr = take(jacobi_scratch_doubles((int)r) * 8);
    L.total = o;
    return L;
}

// Everything the chain needs before its first product, in one launch: blocks [0, zero_blocks) clear the
// accumulators (a fill kernel, not a memset node, so the call can be graph-captured) and the two optional
// output words, the next idx_blocks blocks draw the row sample, the rest draw Omega (a null idx / omega means
// the caller supplied it).
__global__ void __launch_bounds__(256)
k_decomp_setup(uint32_t* __restrict__ zero, size_t nwords, uint32_t* __restrict__ amax_out, int32_t* __restrict__ info,
               int zero_blocks, int idx_blocks, uint64_t seed, int64_t M, int64_t Ms, uint32_t* __restrict__ idx,
               int64_t omega_count, bf16_t* __restrict__ omega) {
    const int b = blockIdx.x;
    if (b < zero_blocks) {
        size_t i = (size_t)b * 256 + threadIdx.x;
        const size_t st = (size_t)zero_blocks * 256;
        for (; i < nwords; i += st) zero[i] = 0u;
        if (b == 0 && threadIdx.x == 0) {
            if (amax_out) *amax_out = 0u;
            if (info) *info = 0;
        }
    } else if (b < zero_blocks + idx_blocks) {
        const int64_t j = (int64_t)(b - zero_blocks) * 256 + threadIdx.x;
        if (j < Ms) idx[j] = sample_row(seed, M, Ms, j);
    } else {
        gaussian_pair(seed, (int64_t)(b - zero_blocks - idx_blocks) * 256 + threadIdx.x, omega_count, omega);
    }
}

DOperand op(const void* p, int64_t s_outer, int64_t s_k, const uint32_t* map_outer = nullptr,
            const uint32_t* map_k = nullptr) {
    DOperand o;
    o.p = p; o.s_outer = s_outer; o.s_k = s_k; o.map_outer = map_outer; o.map_k = map_k;
    o.nparts = 1; o.part_stride = 0;
    return o;
}

DOperand op_parts(const void* p, int64_t s_outer, int64_t s_k, int nparts, int64_t part_stride) {
    DOperand o = op(p, s_outer, s_k);
    o.nparts = nparts; o.part_stride = part_stride;
    return o;
}

DEpilogue epi(void* c, int64_t ldc, bf16_t* hi_t = nullptr, bf16_t* lo_t = nullptr, int64_t ld_t = 0) {
    DEpilogue e;
    e.c = c; e.ldc = ldc; e.hi_t = hi_t; e.lo_t = lo_t; e.ld_t = ld_t; e.skip = nullptr;
    return e;
}
DEpilogue epi_skip(void* c, int64_t ldc, const int32_t* skip) {
    DEpilogue e = epi(c, ldc);
    e.skip = skip;
    return e;
}

// contraction chunks so that ~2048 workgroups exist: the generic kernel does not prefetch, so a workgroup
// should own one or two 32-deep stages and the grid, not the loop, should cover the contraction
int split_for(int64_t K, int64_t tiles) {
    int64_t s = 2048 / (tiles > 2048 ? 2048 : tiles);
    int64_t maxs = K / 32;
    if (s > maxs) s = maxs;
    return (int)(s < 1 ? 1 : s);
}

}  // namespace

extern "C" int metis_sample_rows(void* stream, uint64_t seed, int64_t M, int64_t Ms, uint32_t* idx);
extern "C" int metis_gaussian_omega(void* stream, uint64_t seed, int64_t N, int r, uint16_t* omega);

extern "C" size_t metis_decompose_workspace_bytes(int64_t M, int64_t N, int k, int p, double rho) {
    int64_t Ms = metis_sample_count(M, k, p, rho);
    if (Ms < 1 || N < 1 || k < 1) return 0;
    return make_layout(M, N, k, p, Ms).total;
}

extern "C" int metis_decompose(void* stream, const metis_mat* A, int k, int oversample, double sample_rate,
                               uint64_t seed, float* U, float* S, float* V, float* amax_out, void* workspace,
                               size_t workspace_bytes, const uint32_t* idx_in, int64_t n_idx,
                               const uint16_t* omega_in, int32_t* info) {
    if (!A || !A->ptr || !U || !S || !V || !workspace) return METIS_INVALID_ARG;
    if (k < 1 || oversample < 0 || !(sample_rate > 0.0) || sample_rate > 1.0) return METIS_INVALID_ARG;
    if (A->dtype != METIS_BF16) return METIS_UNSUPPORTED;
    const int64_t M = A->rows, N = A->cols, lda = A->ld;
    if (M < 1 || N < 1 || lda < N) return METIS_BAD_SHAPE;
    if (N % 8 || lda % 8 || reinterpret_cast<uintptr_t>(A->ptr) % 16) return METIS_BAD_SHAPE;  // 16-byte row loads
    const int r = k + oversample;
    int64_t Ms = idx_in ? n_idx : metis_sample_count(M, k, oversample, sample_rate);
    if (Ms < 1 || Ms > M) return METIS_BAD_SHAPE;
    if (r > Ms || r > N) return METIS_BAD_SHAPE;
    if (r > SM_MAX_CHOL || k > 128) return METIS_UNSUPPORTED;
    const Layout L = make_layout(M, N, k, oversample, Ms);
    if (workspace_bytes < L.total) return METIS_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16) return METIS_INVALID_ARG;

    hipStream_t s = (hipStream_t)stream;
    char* ws = (char*)workspace;
    double* Zacc = (double*)(ws + L.off_zacc);
    double* G1 = (double*)(ws + L.off_g1);
    double* G1b = (double*)(ws + L.off_g1b);
    double* G2 = (double*)(ws + L.off_g2);
    double* G3 = (double*)(ws + L.off_g3);
    float* C = (float*)(ws + L.off_c);
    uint32_t* idx = (uint32_t*)(ws + L.off_idx);
    bf16_t* omega = (bf16_t*)(ws + L.off_omega);
    double* Linv = (double*)(ws + L.off_linv);
    double* H1 = (double*)(ws + L.off_h1);
    double* H = (double*)(ws + L.off_h);
    double* B = (double*)(ws + L.off_b);
    double* lam = (double*)(ws + L.off_lam);
    double* T = (double*)(ws + L.off_t);
    float* V0f = (float*)(ws + L.off_v0f);
    bf16_t* V0hi = (bf16_t*)(ws + L.off_v0hi);
    bf16_t* V0lo = (bf16_t*)(ws + L.off_v0lo);
    double* lam3 = (double*)(ws + L.off_lam3);
    double* W3 = (double*)(ws + L.off_w3);
    double* T3 = (double*)(ws + L.off_t3);
    const bf16_t* Ap = (const bf16_t*)A->ptr;
    int st;

    // accumulators start at zero; the draws the caller did not supply
    const uint32_t* idx_use = idx_in ? idx_in : idx;
    const bf16_t* om_use = omega_in ? omega_in : omega;
    {
        const int zero_blocks = 512, idx_blocks = idx_in ? 0 : (int)ceil_div64(Ms, 256);
        const int64_t omega_count = N * (int64_t)r;
        const int64_t omega_blocks = omega_in ? 0 : ceil_div64(ceil_div64(omega_count, 2), 256);
        if (zero_blocks + idx_blocks + omega_blocks > 0x7FFFFFFF) return METIS_UNSUPPORTED;
        hipLaunchKernelGGL(k_decomp_setup, dim3((unsigned)(zero_blocks + idx_blocks + omega_blocks)), dim3(256), 0, s,
                           (uint32_t*)ws, L.zero_bytes / 4, (uint32_t*)amax_out, info, zero_blocks, idx_blocks, seed, M, Ms,
                           idx_in ? nullptr : idx, omega_count, omega_in ? nullptr : omega);
        METIS_LAUNCH_CHECK();
    }

    const int64_t tiles_zr = ceil_div64(Ms, 32) * ceil_div64(r, 32);
    const int64_t tiles_rr = ceil_div64(r, 32) * ceil_div64(r, 32);
    // sketch Z = A_s Omega
    const bool fast = skinny_ok(Ap, lda, N, r) && reinterpret_cast<uintptr_t>(om_use) % 16 == 0;
    if (fast) {
        if ((st = launch_sketch(s, Ap, lda, idx_use, Ms, N, om_use, r, Zacc)) != METIS_OK) return st;
    } else {
        launch_dgemm<bf16_t, bf16_t, EPI_ATOMIC_F64>(s, op(Ap, lda, 1, idx_use), op(om_use, 1, r), Ms, r, N,
                                                      split_for(N, tiles_zr), epi(Zacc, r));
    }
    // CholeskyQR2: Z = H R
    launch_dgemm<double, double, EPI_ATOMIC_F64>(s, op(Zacc, 1, r), op(Zacc, 1, r), r, r, Ms,
                                                  split_for(Ms, tiles_rr), epi(G1, r));
    METIS_LAUNCH_CHECK();
    // The second pass only repairs the orthogonality the first one lost to cond(Z)^2 eps.  When the first
    // factor's diagonal shows a well-conditioned sketch the first pass's H1 is orthonormal to ~1e-10 already:
    // a device flag then turns the second pass's kernels into no-ops and the projection reads H1.
    int32_t* wellcond = fast ? (int32_t*)(ws + L.off_flag) : nullptr;
    if ((st = launch_chol_inv(s, G1, r, Linv, info, wellcond, nullptr)) != METIS_OK) return st;
    launch_dgemm<double, double, EPI_STORE_F64>(s, op(Zacc, r, 1), op(Linv, r, 1), Ms, r, r, 1, epi(H1, r));
    launch_dgemm<double, double, EPI_ATOMIC_F64>(s, op(H1, 1, r), op(H1, 1, r), r, r, Ms,
                                                  split_for(Ms, tiles_rr), epi_skip(G1b, r, wellcond));
    METIS_LAUNCH_CHECK();
    if ((st = launch_chol_inv(s, G1b, r, Linv, info, nullptr, wellcond)) != METIS_OK) return st;
    launch_dgemm<double, double, EPI_STORE_F64>(s, op(H1, r, 1), op(Linv, r, 1), Ms, r, r, 1, epi_skip(H, r, wellcond));
    // reduced matrix B = H^T A_s  (r x N)
    if (fast) {
        if ((st = launch_project(s, H, H1, wellcond, r, Ap, lda, idx_use, Ms, N, B)) != METIS_OK) return st;
    } else {
        launch_dgemm<double, bf16_t, EPI_ATOMIC_F64>(s, op(H, 1, r), op(Ap, 1, lda, nullptr, idx_use), r, N, Ms,
                                                      split_for(Ms, ceil_div64(r, 32) * ceil_div64(N, 32)), epi(B, N));
    }
    // top-k right singular vectors of B from the eigen-decomposition of B B^T
    launch_dgemm<double, double, EPI_ATOMIC_F64>(s, op(B, N, 1), op(B, N, 1), r, r, N, split_for(N, tiles_rr),
                                                  epi(G2, r));
    METIS_LAUNCH_CHECK();
    if ((st = launch_jacobi_eig(s, G2, r, k, lam, nullptr, T, nullptr, (double*)(ws + L.off_jscr))) != METIS_OK) return st;
    launch_dgemm<double, double, EPI_STORE_SPLIT_T>(s, op(B, 1, N), op(T, 1, k), N, k, r, 1,
                                                     epi(V0f, k, V0hi, V0lo, N));
    METIS_LAUNCH_CHECK();
    // broadcast to the full batch: C = A V0
    const int pi = metis_prof_begin(METIS_PROF_BROADCAST, s);
    st = launch_broadcast(s, Ap, lda, M, N, V0hi, V0lo, k, C, (uint32_t*)amax_out);
    metis_prof_end(METIS_PROF_BROADCAST, pi, s);
    if (st != METIS_OK) return st;
    // singular-value form: C = U S W^T, V = V0 W
    const int64_t tiles_kk = ceil_div64(k, 32) * ceil_div64(k, 32);
    const int cparts = broadcast_splits(M, N);
    const int64_t cstride = M * (int64_t)k;
    const bool gram_fast = k % 4 == 0;
    if (gram_fast) {
        // sums the broadcast's partial products into C (part 0) on the way
        if ((st = launch_gram_parts(s, C, k, M, cparts, cstride, C, G3)) != METIS_OK) return st;
    } else {
        launch_dgemm<float, float, EPI_ATOMIC_F64>(s, op_parts(C, 1, k, cparts, cstride), op_parts(C, 1, k, cparts, cstride),
                                                    k, k, M, split_for(M, tiles_kk), epi(G3, k));
    }
    METIS_LAUNCH_CHECK();
    if ((st = launch_jacobi_eig(s, G3, k, k, lam3, W3, T3, S)) != METIS_OK) return st;
    if (gram_fast)
        launch_dgemm<float, double, EPI_STORE_F32>(s, op(C, k, 1), op(T3, 1, k), M, k, k, 1, epi(U, k));
    else
        launch_dgemm<float, double, EPI_STORE_F32>(s, op_parts(C, k, 1, cparts, cstride), op(T3, 1, k), M, k, k, 1, epi(U, k));
    launch_dgemm<float, double, EPI_STORE_F32>(s, op(V0f, k, 1), op(W3, 1, k), N, k, k, 1, epi(V, k));
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
