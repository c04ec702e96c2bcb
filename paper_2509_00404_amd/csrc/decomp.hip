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
#include "splitq.h"
#include "rng_dev.h"
#include <algorithm>
#include <vector>

namespace {

// contraction chunks so that ~2048 workgroups exist: the generic kernel does not prefetch, so a workgroup
// should own one or two 32-deep stages and the grid, not the loop, should cover the contraction
int split_for(int64_t K, int64_t tiles) {
    int64_t s = 2048 / (tiles > 2048 ? 2048 : tiles);
    int64_t maxs = K / 32;
    if (s > maxs) s = maxs;
    return (int)(s < 1 ? 1 : s);
}

struct Layout {
    int64_t M, N, Ms;
    int k, r;
    size_t off_zacc, off_g1, off_g1b, off_g2, off_g3, off_flag, off_c, off_b, off_parts, zero_bytes;
    size_t off_idx, off_omega, off_linv, off_h1, off_h, off_lam, off_t, off_v0f, off_v0hi, off_v0lo,
        off_lam3, off_w3, off_t3, off_jscr, total;
};

Layout make_layout(int64_t M, int64_t N, int k, int p, int64_t Ms) {
    Layout L;
    L.M = M; L.N = N; L.Ms = Ms; L.k = k; L.r = k + p;
    const size_t r = (size_t)L.r, kk = (size_t)k;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.off_flag = take(4);
    L.zero_bytes = o;                      // cleared at the start of a decomposition: only the flag word
    L.off_zacc = take((size_t)Ms * r * 8);
    L.off_g1 = take(r * r * 8);
    L.off_g1b = take(r * r * 8);
    L.off_g2 = take(r * r * 8);
    L.off_g3 = take(kk * kk * 8);
    L.off_b = take(r * (size_t)N * 8);
    {
        // one region for the partial products of whichever split contraction is running (they run one after the
        // other): the sketch, the projection and the four Gram matrices; sized for the fast and the generic kernels
        const int64_t tiles_rr = ceil_div64(L.r, 32) * ceil_div64(L.r, 32), tiles_kk = ceil_div64(k, 32) * ceil_div64(k, 32);
        const size_t zp = std::max(sketch_parts(Ms, N), dgemm_parts<EPI_PART_F64>(Ms, L.r, N, split_for(N, ceil_div64(Ms, 32) * ceil_div64(L.r, 32))));
        const size_t bp = std::max(project_parts(Ms, N), dgemm_parts<EPI_PART_F64>(L.r, N, Ms, split_for(Ms, ceil_div64(L.r, 32) * ceil_div64(N, 32))));
        const size_t g1p = dgemm_parts<EPI_PART_F64>(L.r, L.r, Ms, split_for(Ms, tiles_rr));
        const size_t g2p = dgemm_parts<EPI_PART_F64>(L.r, L.r, N, split_for(N, tiles_rr));
        const size_t g3p = std::max((int)ceil_div64(M, GR_ROWS), dgemm_parts<EPI_PART_F64>(k, k, M, split_for(M, tiles_kk)));
        size_t need = zp * (size_t)Ms * r;
        need = std::max(need, bp * r * (size_t)N);
        need = std::max(need, std::max(g1p, g2p) * r * r);
        need = std::max(need, g3p * kk * kk);
        L.off_parts = take(need * 8);
    }
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

// Extra workspace of the fused decomposition + split (after the decomposition's own layout): the bf16 operands of
// R = A - C V0^T and the partial products of one band of rows.  A band is as many rows as stay resident in the
// last-level cache between the pass that forms C = A V0 and the pass that subtracts and quantizes (64 MiB of A).
struct FusedLayout {
    size_t off_us_hi, off_us_lo, off_v_hi, off_v_lo, off_band, total;
    int64_t band_rows;
    int kp;
};

FusedLayout make_fused_layout(size_t base, int64_t M, int64_t N, int k) {
    FusedLayout F;
    F.kp = padded_rank(k);
    int64_t rows = (((int64_t)64 << 20) / (2 * N)) / 256 * 256;
    if (rows < 256) rows = 256;
    if (rows >= M) rows = M;
    F.band_rows = rows;
    size_t o = align_up(base, 256);
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    F.off_us_hi = take((size_t)M * F.kp * 2);
    F.off_us_lo = take((size_t)M * F.kp * 2);
    F.off_v_hi = take((size_t)N * F.kp * 2);
    F.off_v_lo = take((size_t)N * F.kp * 2);
    F.off_band = take((size_t)16 * (size_t)rows * (size_t)k * 4);
    F.total = o;
    return F;
}

// Everything the chain needs before its first product, in one launch: blocks [0, zero_blocks) clear the
// flag word (a fill kernel, not a memset node, so the call can be graph-captured) and the two optional
// output words, the next idx_blocks blocks draw the row sample, the rest draw Omega (a null idx / omega means
// the caller supplied it).
__global__ void __launch_bounds__(256)
k_decomp_setup(uint32_t* __restrict__ zero, size_t nwords, uint32_t* __restrict__ amax_out, int32_t* __restrict__ info,
               int zero_blocks, int idx_blocks, uint64_t seed, int64_t M, int64_t Ms, int64_t group,
               uint32_t* __restrict__ idx, int64_t omega_count, bf16_t* __restrict__ omega) {
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
        if (j < Ms) idx[j] = sample_row_grouped(seed, M, Ms, group, j);
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
    e.c = c; e.ldc = ldc; e.hi_t = hi_t; e.lo_t = lo_t; e.ld_t = ld_t; e.skip = nullptr; e.part_stride = 0;
    return e;
}
// partial products of a split contraction, M x N each
DEpilogue epi_part(double* parts, int64_t M, int64_t N, const int32_t* skip = nullptr) {
    DEpilogue e = epi(parts, N);
    e.part_stride = M * N;
    e.skip = skip;
    return e;
}
DEpilogue epi_skip(void* c, int64_t ldc, const int32_t* skip) {
    DEpilogue e = epi(c, ldc);
    e.skip = skip;
    return e;
}

}  // namespace

extern "C" int metis_sample_rows(void* stream, uint64_t seed, int64_t M, int64_t Ms, uint32_t* idx);
extern "C" int metis_gaussian_omega(void* stream, uint64_t seed, int64_t N, int r, uint16_t* omega);

extern "C" size_t metis_decompose_workspace_bytes(int64_t M, int64_t N, int k, int p, double rho) {
    int64_t Ms = metis_sample_count(M, k, p, rho);
    if (Ms < 1 || N < 1 || k < 1) return 0;
    return make_layout(M, N, k, p, Ms).total;
}

namespace {

// One decomposition in flight: the caller's arguments plus the carved-up workspace.
struct Job {
    const bf16_t* A;
    int64_t M, N, lda, Ms, group;
    int k, r;
    uint64_t seed;
    float *U, *S, *V, *amax_out;
    const uint32_t *idx_in, *idx_use;
    const bf16_t *omega_in, *om_use;
    int32_t *info, *wellcond;
    bool fast, gram_fast;
    int cparts;
    char* ws;
    Layout L;
    double *Zacc, *G1, *G1b, *G2, *G3, *Linv, *H1, *H, *B, *lam, *T, *lam3, *W3, *T3, *jscr, *parts;
    float *C, *V0f;
    uint32_t* idx;
    bf16_t *omega, *V0hi, *V0lo;
    // fused split (split != nullptr): R = A - C V0^T is quantized band by band right after the band's C
    metis_split* split;
    float* R_debug;
    FusedLayout F;
};

int make_job(const metis_decompose_job& a, Job& j) {
    if (!a.A || !a.A->ptr || !a.U || !a.S || !a.V || !a.workspace) return METIS_INVALID_ARG;
    if (a.k < 1 || a.oversample < 0 || !(a.sample_rate > 0.0) || a.sample_rate > 1.0) return METIS_INVALID_ARG;
    if (a.A->dtype != METIS_BF16) return METIS_UNSUPPORTED;
    j.M = a.A->rows; j.N = a.A->cols; j.lda = a.A->ld;
    if (j.M < 1 || j.N < 1 || j.lda < j.N) return METIS_BAD_SHAPE;
    if (j.N % 8 || j.lda % 8 || reinterpret_cast<uintptr_t>(a.A->ptr) % 16) return METIS_BAD_SHAPE;  // 16-byte row loads
    j.k = a.k;
    j.r = a.k + a.oversample;
    j.group = a.sample_group > 1 ? a.sample_group : 1;
    if (j.group > 1 && (j.M % j.group || j.M >= ((int64_t)1 << 32))) return METIS_BAD_SHAPE;
    j.Ms = a.idx ? a.n_idx : metis_sample_count_sequences(j.M, a.k, a.oversample, a.sample_rate, j.group);
    if (j.Ms < 1 || j.Ms > j.M) return METIS_BAD_SHAPE;
    if (j.r > j.Ms || j.r > j.N) return METIS_BAD_SHAPE;
    if (j.r > SM_MAX_CHOL || j.k > 128) return METIS_UNSUPPORTED;
    j.L = make_layout(j.M, j.N, a.k, a.oversample, j.Ms);
    j.split = a.split;
    j.R_debug = a.R_debug;
    size_t need = j.L.total;
    if (a.split) {
        const int cs = check_split_out(j.M, j.N, a.k, a.split);
        if (cs != METIS_OK) return cs;
        j.F = make_fused_layout(j.L.total, j.M, j.N, a.k);
        need = j.F.total;
    }
    if (a.workspace_bytes < need) return METIS_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(a.workspace) % 16) return METIS_INVALID_ARG;
    const Layout& L = j.L;
    char* ws = (char*)a.workspace;
    j.ws = ws;
    j.A = (const bf16_t*)a.A->ptr;
    j.seed = a.seed;
    j.U = a.U; j.S = a.S; j.V = a.V; j.amax_out = a.amax_out; j.info = a.info;
    j.Zacc = (double*)(ws + L.off_zacc);
    j.G1 = (double*)(ws + L.off_g1);
    j.G1b = (double*)(ws + L.off_g1b);
    j.G2 = (double*)(ws + L.off_g2);
    j.G3 = (double*)(ws + L.off_g3);
    j.C = (float*)(ws + L.off_c);
    j.idx = (uint32_t*)(ws + L.off_idx);
    j.omega = (bf16_t*)(ws + L.off_omega);
    j.Linv = (double*)(ws + L.off_linv);
    j.H1 = (double*)(ws + L.off_h1);
    j.H = (double*)(ws + L.off_h);
    j.B = (double*)(ws + L.off_b);
    j.lam = (double*)(ws + L.off_lam);
    j.T = (double*)(ws + L.off_t);
    j.V0f = (float*)(ws + L.off_v0f);
    j.V0hi = (bf16_t*)(ws + L.off_v0hi);
    j.V0lo = (bf16_t*)(ws + L.off_v0lo);
    j.lam3 = (double*)(ws + L.off_lam3);
    j.W3 = (double*)(ws + L.off_w3);
    j.T3 = (double*)(ws + L.off_t3);
    j.jscr = (double*)(ws + L.off_jscr);
    j.parts = (double*)(ws + L.off_parts);
    j.idx_in = a.idx;
    j.omega_in = (const bf16_t*)a.omega;
    j.idx_use = a.idx ? a.idx : j.idx;
    j.om_use = a.omega ? (const bf16_t*)a.omega : j.omega;
    j.fast = skinny_ok(j.A, j.lda, j.N, j.r) && reinterpret_cast<uintptr_t>(j.om_use) % 16 == 0;
    // The second CholeskyQR pass only repairs the orthogonality the first one lost to cond(Z)^2 eps.  When the
    // first factor's diagonal shows a well-conditioned sketch the first pass's H1 is orthonormal to ~1e-10
    // already: a device flag then turns the second pass's kernels into no-ops and the projection reads H1.
    j.wellcond = j.fast ? (int32_t*)(ws + L.off_flag) : nullptr;
    j.gram_fast = a.k % 4 == 0;
    j.cparts = a.split ? 1 : broadcast_splits(j.M, j.N);      // the fused path sums each band's parts at once
    return METIS_OK;
}

// The single-workgroup factorizations of all jobs in one launch per distinct order (they are latency-bound on
// one CU each, so a batch costs what one problem costs).
template <class P, class F>
int launch_grouped(const std::vector<Job>& jobs, F order_of, int (*launch)(hipStream_t, const P*, int, int, int),
                   hipStream_t s, const std::vector<P>& probs, const std::vector<int>& kks) {
    std::vector<char> done(jobs.size(), 0);
    for (size_t i = 0; i < jobs.size(); ++i) {
        if (done[i]) continue;
        std::vector<P> grp;
        for (size_t t = i; t < jobs.size(); ++t)
            if (!done[t] && order_of(jobs[t]) == order_of(jobs[i]) && kks[t] == kks[i]) {
                grp.push_back(probs[t]);
                done[t] = 1;
            }
        const int st = launch(s, grp.data(), (int)grp.size(), order_of(jobs[i]), kks[i]);
        if (st != METIS_OK) return st;
    }
    return METIS_OK;
}

int chol_launch(hipStream_t s, const CholProblem* p, int count, int n, int) { return launch_chol_inv_batch(s, p, count, n); }

}  // namespace

extern "C" int metis_decompose_batch(void* stream, int n_jobs, const metis_decompose_job* args) {
    if (n_jobs < 0 || (n_jobs > 0 && !args)) return METIS_INVALID_ARG;
    if (n_jobs == 0) return METIS_OK;
    std::vector<Job> jobs((size_t)n_jobs);
    int st;
    // every argument error is found before anything is enqueued
    for (int i = 0; i < n_jobs; ++i)
        if ((st = make_job(args[i], jobs[(size_t)i])) != METIS_OK) return st;
    for (const Job& j : jobs) {
        const int64_t omega_blocks = j.omega_in ? 0 : ceil_div64(ceil_div64(j.N * (int64_t)j.r, 2), 256);
        if (512 + ceil_div64(j.Ms, 256) + omega_blocks > 0x7FFFFFFF) return METIS_UNSUPPORTED;
    }
    hipStream_t s = (hipStream_t)stream;
    const std::vector<int> zeros(jobs.size(), 0);

    // ---- flag and status words to zero, the draws the caller did not supply, sketch Z = A_s Omega, Gram of Z ----
    // (every split contraction writes its partial products to the job's `parts` region and a batched kernel adds
    // them in a fixed order: no floating-point atomics anywhere, so a decomposition is reproducible bit for bit)
    for (const Job& j : jobs) {
        const int zero_blocks = 1, idx_blocks = j.idx_in ? 0 : (int)ceil_div64(j.Ms, 256);
        const int64_t omega_count = j.N * (int64_t)j.r;
        const int64_t omega_blocks = j.omega_in ? 0 : ceil_div64(ceil_div64(omega_count, 2), 256);
        hipLaunchKernelGGL(k_decomp_setup, dim3((unsigned)(zero_blocks + idx_blocks + omega_blocks)), dim3(256), 0, s,
                           (uint32_t*)j.ws, j.L.zero_bytes / 4, (uint32_t*)j.amax_out, j.info, zero_blocks, idx_blocks, j.seed,
                           j.M, j.Ms, j.group, j.idx_in ? nullptr : j.idx, omega_count, j.omega_in ? nullptr : j.omega);
        METIS_LAUNCH_CHECK();
    }
    // products of the same kind and step of all jobs go out together (DgemmList): the small ones are latency-bound
    DgemmList<double, double, EPI_PART_F64> gram;
    DgemmList<double, double, EPI_STORE_F64> mul;
    DgemmList<double, double, EPI_STORE_SPLIT_T> v0mul;
    DgemmList<float, double, EPI_STORE_F32> outmul;
    SumList sums;
    auto tiles_rr = [](const Job& j) { return ceil_div64(j.r, 32) * ceil_div64(j.r, 32); };
    // Gram matrix of X (K x r, row-major, ld r) for every job: partial products, then their sum
    auto gram_of = [&](double* Job::*X, double* Job::*G, auto K_of, bool skippable) {
        for (const Job& j : jobs) {
            const int r = j.r;
            const int64_t K = K_of(j);
            const bool by_rows = X != &Job::B;           // Z, H1: contraction over rows; B (r x N): over columns
            const DOperand o = by_rows ? op(j.*X, 1, r) : op(j.*X, K, 1);
            const int32_t* skip = skippable ? j.wellcond : nullptr;
            gram.add(o, o, r, r, K, split_for(K, tiles_rr(j)), epi_part(j.parts, r, r, skip));
            sums.add(j.parts, dgemm_parts<EPI_PART_F64>(r, r, K, split_for(K, tiles_rr(j))), (int64_t)r * r, (int64_t)r * r,
                     j.*G, skip);
        }
        gram.launch(s);
        sums.launch(s);
    };
    for (const Job& j : jobs) {
        const int r = j.r;
        const int64_t tiles_zr = ceil_div64(j.Ms, 32) * ceil_div64(r, 32);
        int zp;
        if (j.fast) {
            if ((st = launch_sketch(s, j.A, j.lda, j.idx_use, j.Ms, j.N, j.om_use, r, j.parts)) != METIS_OK) return st;
            zp = sketch_parts(j.Ms, j.N);
        } else {
            launch_dgemm<bf16_t, bf16_t, EPI_PART_F64>(s, op(j.A, j.lda, 1, j.idx_use), op(j.om_use, 1, r), j.Ms, r, j.N,
                                                        split_for(j.N, tiles_zr), epi_part(j.parts, j.Ms, r));
            zp = dgemm_parts<EPI_PART_F64>(j.Ms, r, j.N, split_for(j.N, tiles_zr));
        }
        METIS_LAUNCH_CHECK();
        sums.add(j.parts, zp, j.Ms * (int64_t)r, j.Ms * (int64_t)r, j.Zacc);
    }
    sums.launch(s);
    METIS_LAUNCH_CHECK();
    gram_of(&Job::Zacc, &Job::G1, [](const Job& j) { return j.Ms; }, false);
    METIS_LAUNCH_CHECK();
    // ---- CholeskyQR2: Z = H R ----
    {
        std::vector<CholProblem> pr;
        for (const Job& j : jobs) pr.push_back({j.G1, j.Linv, j.info, j.wellcond, nullptr});
        if ((st = launch_grouped<CholProblem>(jobs, [](const Job& j) { return j.r; }, chol_launch, s, pr, zeros)) != METIS_OK)
            return st;
    }
    for (const Job& j : jobs) mul.add(op(j.Zacc, j.r, 1), op(j.Linv, j.r, 1), j.Ms, j.r, j.r, 1, epi(j.H1, j.r));
    mul.launch(s);
    gram_of(&Job::H1, &Job::G1b, [](const Job& j) { return j.Ms; }, true);
    METIS_LAUNCH_CHECK();
    {
        std::vector<CholProblem> pr;
        for (const Job& j : jobs) pr.push_back({j.G1b, j.Linv, j.info, nullptr, j.wellcond});
        if ((st = launch_grouped<CholProblem>(jobs, [](const Job& j) { return j.r; }, chol_launch, s, pr, zeros)) != METIS_OK)
            return st;
    }
    // ---- reduced matrix B = H^T A_s (r x N) and its Gram matrix ----
    for (const Job& j : jobs) mul.add(op(j.H1, j.r, 1), op(j.Linv, j.r, 1), j.Ms, j.r, j.r, 1, epi_skip(j.H, j.r, j.wellcond));
    mul.launch(s);
    METIS_LAUNCH_CHECK();
    for (const Job& j : jobs) {
        const int r = j.r;
        int bp;
        if (j.fast) {
            if ((st = launch_project(s, j.H, j.H1, j.wellcond, r, j.A, j.lda, j.idx_use, j.Ms, j.N, j.parts)) != METIS_OK) return st;
            bp = project_parts(j.Ms, j.N);
        } else {
            const int want = split_for(j.Ms, ceil_div64(r, 32) * ceil_div64(j.N, 32));
            launch_dgemm<double, bf16_t, EPI_PART_F64>(s, op(j.H, 1, r), op(j.A, 1, j.lda, nullptr, j.idx_use), r, j.N, j.Ms,
                                                        want, epi_part(j.parts, r, j.N));
            bp = dgemm_parts<EPI_PART_F64>(r, j.N, j.Ms, want);
        }
        METIS_LAUNCH_CHECK();
        sums.add(j.parts, bp, (int64_t)r * j.N, (int64_t)r * j.N, j.B);
    }
    sums.launch(s);
    METIS_LAUNCH_CHECK();
    gram_of(&Job::B, &Job::G2, [](const Job& j) { return j.N; }, false);
    METIS_LAUNCH_CHECK();
    // ---- top-k right singular vectors of B from the eigen-decomposition of B B^T ----
    {
        std::vector<JacobiProblem> pr;
        std::vector<int> kks;
        for (const Job& j : jobs) {
            pr.push_back({j.G2, j.lam, nullptr, j.T, nullptr, j.jscr});
            kks.push_back(j.k);
        }
        if ((st = launch_grouped<JacobiProblem>(jobs, [](const Job& j) { return j.r; }, launch_jacobi_eig_batch, s, pr, kks)) !=
            METIS_OK)
            return st;
    }
    // ---- broadcast to the full batch: C = A V0, and its Gram matrix ----
    for (const Job& j : jobs)
        v0mul.add(op(j.B, 1, j.N), op(j.T, 1, j.k), j.N, j.k, j.r, 1, epi(j.V0f, j.k, j.V0hi, j.V0lo, j.N));
    v0mul.launch(s);
    METIS_LAUNCH_CHECK();
    for (const Job& j : jobs) {
        const int k = j.k;
        if (j.split) {
            // Fused split (R = A - U S V^T = A - (A V0) V0^T needs only V0): band by band, C = A V0 for the band's
            // rows, then the band's residual and its quantization while the band is still in the last-level cache.
            const FusedLayout& F = j.F;
            bf16_t* us_hi = (bf16_t*)(j.ws + F.off_us_hi);
            bf16_t* us_lo = (bf16_t*)(j.ws + F.off_us_lo);
            bf16_t* v_hi = (bf16_t*)(j.ws + F.off_v_hi);
            bf16_t* v_lo = (bf16_t*)(j.ws + F.off_v_lo);
            float* band = (float*)(j.ws + F.off_band);
            metis_split* o = j.split;
            const bool want_t = o->Rt.codes != nullptr;
            if ((st = launch_v_factors(s, j.V0f, j.N, k, F.kp, v_hi, v_lo)) != METIS_OK) return st;
            for (int64_t r0 = 0; r0 < j.M; r0 += F.band_rows) {
                const int64_t rows = j.M - r0 < F.band_rows ? j.M - r0 : F.band_rows;
                const int parts = broadcast_splits(rows, j.N);
                const bf16_t* Ab = j.A + r0 * j.lda;
                const int pi = metis_prof_begin(METIS_PROF_BROADCAST, s);
                st = launch_broadcast(s, Ab, j.lda, rows, j.N, j.V0hi, j.V0lo, k, band, (uint32_t*)j.amax_out);
                metis_prof_end(METIS_PROF_BROADCAST, pi, s);
                if (st != METIS_OK) return st;
                if ((st = launch_band_factors(s, band, parts, rows * (int64_t)k, rows, k, F.kp, j.C + r0 * k,
                                              us_hi + r0 * F.kp, us_lo + r0 * F.kp)) != METIS_OK)
                    return st;
                if ((st = launch_residual_quant(s, Ab, j.lda, rows, j.N, j.M, r0, us_hi + r0 * F.kp, us_lo + r0 * F.kp, v_hi,
                                                v_lo, F.kp, o->R.tscale, o->R.codes + r0 * (j.N / 2),
                                                o->R.scales + r0 * (j.N / 16), want_t ? o->Rt.codes + r0 / 2 : nullptr,
                                                want_t ? o->Rt.scales + r0 / 16 : nullptr,
                                                j.R_debug ? j.R_debug + r0 * j.N : nullptr, false, 0)) != METIS_OK)
                    return st;
            }
        } else {
            const int pi = metis_prof_begin(METIS_PROF_BROADCAST, s);
            st = launch_broadcast(s, j.A, j.lda, j.M, j.N, j.V0hi, j.V0lo, k, j.C, (uint32_t*)j.amax_out);
            metis_prof_end(METIS_PROF_BROADCAST, pi, s);
            if (st != METIS_OK) return st;
        }
        const int64_t tiles_kk = ceil_div64(k, 32) * ceil_div64(k, 32);
        const int64_t cstride = j.M * (int64_t)k;
        if (j.gram_fast) {
            // sums the broadcast's partial products into C (part 0) on the way
            if ((st = launch_gram_parts(s, j.C, k, j.M, j.cparts, cstride, j.C, j.parts)) != METIS_OK) return st;
            sums.add(j.parts, (int)ceil_div64(j.M, GR_ROWS), (int64_t)k * k, (int64_t)k * k, j.G3);
        } else {
            const int want = split_for(j.M, tiles_kk);
            launch_dgemm<float, float, EPI_PART_F64>(s, op_parts(j.C, 1, k, j.cparts, cstride), op_parts(j.C, 1, k, j.cparts, cstride),
                                                      k, k, j.M, want, epi_part(j.parts, k, k));
            sums.add(j.parts, dgemm_parts<EPI_PART_F64>(k, k, j.M, want), (int64_t)k * k, (int64_t)k * k, j.G3);
        }
        METIS_LAUNCH_CHECK();
    }
    sums.launch(s);
    METIS_LAUNCH_CHECK();
    // ---- singular-value form: C = U S W^T, V = V0 W ----
    {
        std::vector<JacobiProblem> pr;
        std::vector<int> kks;
        for (const Job& j : jobs) {
            pr.push_back({j.G3, j.lam3, j.W3, j.T3, j.S, nullptr});
            kks.push_back(j.k);
        }
        if ((st = launch_grouped<JacobiProblem>(jobs, [](const Job& j) { return j.k; }, launch_jacobi_eig_batch, s, pr, kks)) !=
            METIS_OK)
            return st;
    }
    for (const Job& j : jobs) {
        const int k = j.k;
        const int64_t cstride = j.M * (int64_t)k;
        if (j.gram_fast)
            outmul.add(op(j.C, k, 1), op(j.T3, 1, k), j.M, k, k, 1, epi(j.U, k));
        else
            outmul.add(op_parts(j.C, k, 1, j.cparts, cstride), op(j.T3, 1, k), j.M, k, k, 1, epi(j.U, k));
        outmul.add(op(j.V0f, k, 1), op(j.W3, 1, k), j.N, k, k, 1, epi(j.V, k));
    }
    outmul.launch(s);
    METIS_LAUNCH_CHECK();
    for (const Job& j : jobs)
        if (j.split && (st = quantize_factors(s, j.U, j.S, j.V, j.M, j.N, j.k, j.split, false, 0)) != METIS_OK) return st;
    return METIS_OK;
}

extern "C" size_t metis_decompose_split_workspace_bytes(int64_t M, int64_t N, int k, int p, double rho) {
    const size_t base = metis_decompose_workspace_bytes(M, N, k, p, rho);
    if (base == 0 || k > 128) return 0;
    return make_fused_layout(base, M, N, k).total;
}

extern "C" int metis_decompose_split_quantize(void* stream, const metis_mat* A, int k, int oversample, double sample_rate,
                                              uint64_t seed, float* U, float* S, float* V, float* amax_out,
                                              metis_split* out, float* R_debug, void* workspace, size_t workspace_bytes,
                                              const uint32_t* idx_in, int64_t n_idx, const uint16_t* omega_in,
                                              int32_t* info) {
    if (!out) return METIS_INVALID_ARG;
    const metis_decompose_job job = {A, k, oversample, sample_rate, seed, U, S, V, amax_out, workspace, workspace_bytes,
                                     idx_in, n_idx, omega_in, info, out, R_debug, 1};
    return metis_decompose_batch(stream, 1, &job);
}

extern "C" int metis_decompose(void* stream, const metis_mat* A, int k, int oversample, double sample_rate,
                               uint64_t seed, float* U, float* S, float* V, float* amax_out, void* workspace,
                               size_t workspace_bytes, const uint32_t* idx_in, int64_t n_idx,
                               const uint16_t* omega_in, int32_t* info) {
    const metis_decompose_job job = {A, k, oversample, sample_rate, seed, U, S, V, amax_out, workspace, workspace_bytes,
                                     idx_in, n_idx, omega_in, info, nullptr, nullptr, 1};
    return metis_decompose_batch(stream, 1, &job);
}
