// One-workgroup fp64 factorizations of the small (k+p)x(k+p) matrices of the decomposition
// (Sec. 3.1): Cholesky + triangular inverse for CholeskyQR2 (thin QR Z = H R), and a
// one-sided Jacobi eigensolver for the Gram matrices of the reduced problem.
#include "smallmat.h"
#include <cstdlib>
#include <utility>

// ---------------------------------------------------------------------------------------
// Blocked Cholesky in LDS, shared by both kernels below.  On entry W holds the lower triangle of a
// symmetric matrix column-major (element (i, c), i >= c, at W[c*ld + i]); on exit the same places
// hold L, and rinv[c] = 1 / L[c][c].  Blocks of CB = 4 columns, two workgroup barriers per block:
//   1  one thread per row at or below the block reads the CB x CB diagonal block (LDS broadcast), factors
//      it on its own (every thread repeats the same ~30 operations: cheaper than a barrier and a round
//      trip through LDS) and solves its row's CB entries against it (the chain of dependent pivots is what a
//      block costs, and it grows faster than the block: CB = 8 measured slower than 4),
//   2  the trailing matrix takes the rank-CB update on the fp64 matrix cores: CB / 4
//      v_mfma_f64_16x16x4_f64 per 16x16 tile.
// BAD_PIVOT_ZEROES: a pivot <= floor zeroes its column (semi-definite input, eigensolver); otherwise it is
// replaced by 1e-300 and its 1-based index is written to *info (CholeskyQR2's rank check).
// ---------------------------------------------------------------------------------------
typedef double double4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double chol_rsqrt(double x) {
    double y = __builtin_amdgcn_rsq(x);
    y = y * (1.5 - 0.5 * x * y * y);
    y = y * (1.5 - 0.5 * x * y * y);
    return y;
}

template <bool BAD_PIVOT_ZEROES, int CB = 4>
__device__ void chol_blocked(double* __restrict__ W, int ld, int n, double* __restrict__ rinv, double floor_,
                             int32_t* __restrict__ info) {
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthr >> 6;
    static_assert(CB % 4 == 0, "the trailing update takes the block in chunks of the matrix instruction's depth");
    for (int k0 = 0; k0 < n; k0 += CB) {
        // ---- 1: diagonal block (entries past n act as an identity block) and the rows below ----
        double d[CB][CB];                                // lower triangle of the diagonal block
        double r[CB];
        if (tid < n - k0) {
            const int i = k0 + tid;
#pragma unroll
            for (int q = 0; q < CB; ++q)
#pragma unroll
                for (int c = 0; c <= q; ++c)
                    d[q][c] = (k0 + q < n) ? W[(size_t)(k0 + c) * ld + k0 + q] : (q == c ? 1.0 : 0.0);
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                double piv = d[c][c];
#pragma unroll
                for (int t = 0; t < c; ++t) piv -= d[c][t] * d[c][t];
                if (BAD_PIVOT_ZEROES) {
                    r[c] = piv > floor_ ? chol_rsqrt(piv) : 0.0;
                } else {
                    if (!(piv > 0.0)) {
                        if (tid == 0 && info && k0 + c < n) *info = k0 + c + 1;
                        piv = 1e-300;
                    }
                    r[c] = chol_rsqrt(piv);
                }
                d[c][c] = piv * r[c];                    // sqrt(pivot), or 0 for a zeroed column
#pragma unroll
                for (int q = c + 1; q < CB; ++q) {
                    double v = d[q][c];
#pragma unroll
                    for (int t = 0; t < c; ++t) v -= d[q][t] * d[c][t];
                    d[q][c] = v * r[c];
                }
            }
            if (tid >= CB) {
                double x[CB];
#pragma unroll
                for (int c = 0; c < CB; ++c) {
                    double v = W[(size_t)(k0 + c) * ld + i];
#pragma unroll
                    for (int t = 0; t < c; ++t) v -= x[t] * d[c][t];
                    x[c] = v * r[c];
                }
#pragma unroll
                for (int c = 0; c < CB; ++c) W[(size_t)(k0 + c) * ld + i] = x[c];
            }
        }
        __syncthreads();
        // the block's own rows are written once every thread has read the unfactored block; nothing
        // reads them again before the next barrier
        if (tid < CB && tid < n - k0) {
#pragma unroll
            for (int q = 0; q < CB; ++q)
                if (tid == q) {
                    rinv[k0 + q] = r[q];
#pragma unroll
                    for (int c = 0; c <= q; ++c) W[(size_t)(k0 + c) * ld + k0 + q] = d[q][c];
                }
        }
        if (n - k0 <= CB) break;
        // ---- 2: trailing update A22 -= L21 L21^T over the 16-aligned lower tiles that reach past k0 + CB ----
        const int t0 = (k0 + CB) & ~15;
        const int T = (n - t0 + 15) / 16, ntiles = T * (T + 1) / 2;
        for (int tile = wave; tile < ntiles; tile += nwaves) {
            int ti = 0, rem = tile;
            while (rem > ti) { rem -= ti + 1; ++ti; }       // tile -> (ti, tc), tc <= ti
            const int i0 = t0 + 16 * ti, c0 = t0 + 16 * rem;
            const int ia = i0 + (lane & 15), cb = c0 + (lane & 15);
            double av[CB / 4], bv[CB / 4];
#pragma unroll
            for (int kc = 0; kc < CB / 4; ++kc) {
                const size_t col = (size_t)(k0 + 4 * kc + (lane >> 4)) * ld;
                av[kc] = (ia < n && ia >= k0 + CB) ? W[col + ia] : 0.0;
                bv[kc] = (cb < n && cb >= k0 + CB) ? W[col + cb] : 0.0;
            }
            double4_t acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kc = 0; kc < CB / 4; ++kc) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av[kc], bv[kc], acc, 0, 0, 0);
            // D: lane l, element v -> (row 4 v + l / 16, column l % 16) of the tile
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + 4 * v + (lane >> 4), c = cb;
                if (i < n && c < n && c >= k0 + CB && i >= c) W[(size_t)c * ld + i] -= acc[v];
            }
        }
        __syncthreads();
    }
    __syncthreads();                                     // the last block's rows are visible to the caller
}

// ---------------------------------------------------------------------------------------
// Cholesky G = L L^T and Linv = L^-1 (lower triangular), n <= SM_MAX_N.
// LDS: L [n][n+1] doubles, X [n][n+1] doubles.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double chol_group8_sum(double x) {
    int lo, hi;
    double y;
    lo = __builtin_amdgcn_update_dpp(__double2loint(x), __double2loint(x), 0xB1, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(__double2hiint(x), __double2hiint(x), 0xB1, 0xF, 0xF, false);
    y = x + __hiloint2double(hi, lo);
    lo = __builtin_amdgcn_update_dpp(__double2loint(y), __double2loint(y), 0x4E, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(__double2hiint(y), __double2hiint(y), 0x4E, 0xF, 0xF, false);
    y = y + __hiloint2double(hi, lo);
    lo = __builtin_amdgcn_update_dpp(__double2loint(y), __double2loint(y), 0x141, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(__double2hiint(y), __double2hiint(y), 0x141, 0xF, 0xF, false);
    return y + __hiloint2double(hi, lo);
}

__global__ void __launch_bounds__(1024)
k_chol_inv(const CholBatch batch, int n) {
    extern __shared__ double sm[];
    const CholProblem& prob = batch.p[blockIdx.x];
    const double* __restrict__ G = prob.G;
    double* __restrict__ Linv = prob.Linv;
    int32_t* __restrict__ info = prob.info;
    int32_t* __restrict__ wellcond_out = prob.wellcond_out;
    const int32_t* __restrict__ skip_in = prob.skip_in;
    if (skip_in && *skip_in) {
        for (int e = threadIdx.x; e < n * n; e += 1024) Linv[e] = (e / n == e % n) ? 1.0 : 0.0;
        return;
    }
    const int ld = n + 1;
    double* L = sm;                              // column-major: L(i, c) at L[c*ld + i]
    double* X = sm + (size_t)n * ld;             // L^-1, row-major: X(t, c) at X[t*ld + c]
    __shared__ double dinv[SM_MAX_CHOL];
    const int tid = threadIdx.x;
    for (int e = tid; e < n * n; e += 1024) {
        int i = e / n, j = e - i * n;
        L[j * ld + i] = G[e];
        X[i * ld + j] = 0.0;
    }
    __syncthreads();
    chol_blocked<false>(L, ld, n, dinv, 0.0, info);
    if (wellcond_out && tid == 0) {
        double lo = dinv[0], hi = dinv[0];
        for (int j = 1; j < n; ++j) { lo = fmin(lo, dinv[j]); hi = fmax(hi, dinv[j]); }
        *wellcond_out = (hi <= 1e3 * lo) ? 1 : 0;        // a replaced pivot has dinv = 1e150 and fails this
    }
    // L^-1 by 16 x 16 blocks.  The diagonal blocks are inverted by substitution (one thread per column, 16 steps in
    // registers); then, one block sub-diagonal after the other, X_ij = -X_ii (sum_k L_ik X_kj) on the fp64 matrix
    // cores, one wave per block.  The inner sum leaves the matrix instruction in exactly the register layout that
    // the second product wants for its right operand (accumulator element v = contraction chunk v), so it never
    // touches memory.  Rows and columns past n act as an identity.
    {
        const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = 1024 >> 6;
        const int T = (n + 15) / 16;
        const bool whole = (n & 15) == 0;             // no padding: the accessors need no tests
        auto Lat = [&](int i, int c2) { return (whole || (i < n && c2 < n)) ? L[min(c2, n - 1) * ld + min(i, n - 1)] : (i == c2 ? 1.0 : 0.0); };
        auto Xat = [&](int t, int c2) { return (whole || (t < n && c2 < n)) ? X[min(t, n - 1) * ld + min(c2, n - 1)] : (t == c2 ? 1.0 : 0.0); };
        if (tid < 16 * T) {
            const int b0 = 16 * (tid >> 4), cc = tid & 15, c = b0 + cc;
            if (c < n) {
                double x[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int i = b0 + q;
                    double v = q == cc ? 1.0 : 0.0;
#pragma unroll
                    for (int u = 0; u < q; ++u) v -= Lat(i, b0 + u) * x[u];
                    x[q] = (q >= cc && i < n) ? v * dinv[i] : 0.0;
                }
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    if (b0 + q < n) X[(b0 + q) * ld + c] = x[q];
            }
        }
        __syncthreads();
        const int r16 = lane & 15, kq = lane >> 4;
        for (int d = 1; d < T; ++d) {
            for (int blk0 = 0; blk0 < T - d; blk0 += nwaves) {
                // block (ib, jb); surplus waves sit the round out (`wave` is a scalar: a uniform branch, and waves that
                // repeated a block would queue on the same matrix pipes)
                if (blk0 + wave >= T - d) continue;
                const int jb = blk0 + wave, ib = jb + d;
                double4_t P = {0.0, 0.0, 0.0, 0.0};
                double xa[4];                     // X_ii for the second product, loaded ahead
#pragma unroll
                for (int kc = 0; kc < 4; ++kc) xa[kc] = Xat(16 * ib + r16, 16 * ib + 4 * kc + kq);
                for (int k = jb; k < ib; ++k) {
                    double a[4], b[4];            // the operands of a whole block product before its four instructions
#pragma unroll
                    for (int kc = 0; kc < 4; ++kc) {
                        a[kc] = Lat(16 * ib + r16, 16 * k + 4 * kc + kq);
                        b[kc] = Xat(16 * k + 4 * kc + kq, 16 * jb + r16);
                    }
#pragma unroll
                    for (int kc = 0; kc < 4; ++kc) P = __builtin_amdgcn_mfma_f64_16x16x4f64(a[kc], b[kc], P, 0, 0, 0);
                }
                double4_t R = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int kc = 0; kc < 4; ++kc) R = __builtin_amdgcn_mfma_f64_16x16x4f64(xa[kc], P[kc], R, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = 16 * ib + 4 * v + kq, c2 = 16 * jb + r16;
                    if (i < n && c2 < n) X[i * ld + c2] = -R[v];
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();
    for (int e = tid; e < n * n; e += 1024) {
        int i = e / n, j = e - i * n;
        Linv[e] = X[i * ld + j];
    }
}

// ---------------------------------------------------------------------------------------
// One-sided Jacobi on a symmetric positive semi-definite G (n <= SM_MAX_N), applied to its
// Cholesky factor: rotate the columns of W = L until they are mutually orthogonal; then
// column j is sqrt(lambda_j) v_j.  1024 threads = 64 groups of 16 lanes, one column pair per group and
// step, round-robin ordering; dot products by 16-lane DPP rotations.
// Outputs (eigenvalues descending):
//   lam  [n]            eigenvalues
//   vec  [n][n]         vec[i*n + j] = component i of eigenvector j          (optional)
//   tmat [n][kk]        tmat[i*kk + c] = vec[i][c] / sqrt(lam_c), c < kk     (optional)
//   sval [kk]           (float) sqrt(lam_c)                                  (optional)
// ---------------------------------------------------------------------------------------
// ---- 8-lane all-reduce of a double with DPP (no LDS traffic) ----
template <int CTRL>
__device__ __forceinline__ double dpp_mov64(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xF, 0xF, true);
    hi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double group8_sum(double x) {
    x += dpp_mov64<0xB1>(x);      // quad_perm [1,0,3,2]
    x += dpp_mov64<0x4E>(x);      // quad_perm [2,3,0,1]
    x += dpp_mov64<0x141>(x);     // row_half_mirror: lane i <-> 7-i within each 8 lanes
    return x;
}

// 1/sqrt(x), 1/x for x > 0: hardware seed + one Newton step.  The rotation only has to be
// orthogonal to ~1e-13 (c and s come from the same t, so c^2 + s^2 = 1 up to the error of one rsqrt).
__device__ __forceinline__ double rsqrt_nr(double x) {
    double y = __builtin_amdgcn_rsq(x);
    return y * (1.5 - 0.5 * x * y * y);
}
__device__ __forceinline__ double rcp_nr(double x) {
    double y = __builtin_amdgcn_rcp(x);
    return y * (2.0 - x * y);
}

template <int JGL> __device__ __forceinline__ double group_sum(double x);
template <> __device__ __forceinline__ double group_sum<4>(double x) {
    x += dpp_mov64<0xB1>(x);      // quad_perm [1,0,3,2]
    x += dpp_mov64<0x4E>(x);      // quad_perm [2,3,0,1]
    return x;
}
template <> __device__ __forceinline__ double group_sum<8>(double x) { return group8_sum(x); }
template <> __device__ __forceinline__ double group_sum<16>(double x) {
    x = group8_sum(x);
    x += dpp_mov64<0x140>(x);     // row_mirror: lane i <-> 15-i within each 16 lanes
    return x;
}

// lanes per column pair: a step is bound by the latency of its chain of dependent operations, so the
// widest group (shortest per-lane column pieces) wins even though it needs the most waves
__host__ __device__ static inline int jacobi_lanes(int n) { (void)n; return 16; }
// Column stride in doubles: at least n rounded up to 16 (the rows from n up exist and stay zero, so the
// column loads and stores need no bounds checks), and = l (mod 2 l), which shifts neighbouring columns
// by one group's width in the banks.
__host__ __device__ static inline int jacobi_ld(int n, int l) {
    const int rows = (n + 15) / 16 * 16;
    return rows % (2 * l) == l ? rows : rows + l;
}

// ---------------------------------------------------------------------------------------
// Eigenvector preconditioner for the one-sided Jacobi below.
//
// The cyclic rotations need ~log n sweeps before their quadratic convergence sets in.  If the columns
// of the factor are first multiplied by an orthogonal P that is close to the eigenvector matrix of
// L^T L, the very first sweep already finds (nearly) orthogonal columns and the sweeps only confirm and
// refine: W0 = L P has W0 W0^T = L L^T = G for ANY orthogonal P, so the accuracy of P only affects the
// number of sweeps, never the result (a P orthogonal to 1e-10 perturbs G multiplicatively, i.e. every
// eigenvalue by 1e-10 relative).  P comes from the classical dense symmetric path, all inside this
// workgroup:
//   1  A = L^T L                                       (fp64 matrix cores)
//   2  Householder tridiagonalisation  Q^T A Q = T     (one row per 8 lanes, rows in registers)
//   3  eigenvalues of T by multisection on Sturm counts (8 probes per eigenvalue and round)
//   4  eigenvectors of T by twisted factorisation       (one thread per eigenvector)
//   5  back-transformation  P = Q Z                     (one column per 8 lanes, no barriers)
//   6  Newton-Schulz polish  P <- P (I - (P^T P - I) / 2)  until orthogonal to 1e-10; if the computed
//      vectors are far from orthogonal (coincident or tiny eigenvalues) the preconditioner is dropped
//   7  W0 = L P                                         (fp64 matrix cores)
// R1 holds L on entry (column-major, stride ld, (ne+1) columns); the result is left in R2 in the same
// layout.  gscr: (ne+1)*ld doubles of global scratch for L.  sa: 10*n + 40 doubles of LDS, 16-byte aligned.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_max(double x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmax(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

__device__ __forceinline__ double readlane64(double x, int l) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l), __builtin_amdgcn_readlane(__double2loint(x), l));
}
// x is the same in the 8 lanes of every group: the sum over the wave's 8 groups, in every lane
__device__ __forceinline__ double wave_sum_of_groups8(double x) {
    x += dpp_mov64<0x140>(x);     // row_mirror: the other group of this row of 16 lanes
    return (readlane64(x, 0) + readlane64(x, 16)) + (readlane64(x, 32) + readlane64(x, 48));
}
__device__ __forceinline__ double rcp_nr2(double x) {          // 1/x to ~1e-15 relative
    double y = __builtin_amdgcn_rcp(x);
    y = y * (2.0 - x * y);
    return y * (2.0 - x * y);
}

// 9^12 = 2.8e11 sections of the scaled spectrum: eigenvalues to ~1e-11 ||T||, eigenvectors orthogonal to
// ~1e-5 before the polish, which one Newton-Schulz step brings to ~1e-10
#define PRE_ROUNDS 12
#define PRE_MAX_ROUNDS 20

template <class F, int... I>
__device__ __forceinline__ void for_each_block_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a compile-time constant
template <int N, class F>
__device__ __forceinline__ void for_each_block(F&& f) {
    for_each_block_impl(f, std::make_integer_sequence<int, N>{});
}

// One 16x16 tile of sum_k a(i, k) b(k, j) on the fp64 matrix cores; lane supplies row/column (lane & 15) and the
// k offset lane >> 4.  fa / fb read in-bounds elements; out-of-range rows, columns and k contribute zero.
template <class FA, class FB>
__device__ __forceinline__ double4_t tile_mma(int n, int ia, int jb, int kq, FA fa, FB fb, bool batch = true) {
    const int ic = min(ia, n - 1), jc = min(jb, n - 1);
    const bool iok = ia < n, jok = jb < n;
    double4_t acc = {0.0, 0.0, 0.0, 0.0};
    if ((n & 15) == 0 && batch) {                 // whole tiles: no guards, operands of four steps loaded ahead
        for (int k0 = 0; k0 < n; k0 += 16) {
            double a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a[u] = fa(ia, k0 + 4 * u + kq);
                b[u] = fb(k0 + 4 * u + kq, jb);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u], b[u], acc, 0, 0, 0);
        }
        return acc;
    }
    for (int k0 = 0; k0 < n; k0 += 4) {
        const int k = k0 + kq, kc = min(k, n - 1);
        const double a = fa(ic, kc), b = fb(kc, jc);
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64((iok && k < n) ? a : 0.0, (jok && k < n) ? b : 0.0, acc, 0, 0, 0);
    }
    return acc;
}

// Reflectors j with (j+1)/8 == E0, highest first, applied to the column piece zr (rows q + 8 e); then the lower blocks.
template <int NR, int E0>
__device__ __forceinline__ void back_blocks(double (&zr)[NR], const double* __restrict__ V, int lda, int n, int q,
                                            const double* __restrict__ tauv) {
    const int jhi = min(8 * E0 + 6, n - 3), jlo = max(8 * E0 - 1, 0);
    for (int j = jhi; j >= jlo; --j) {
        const double tau = tauv[j];
        double v[NR], dot = 0.0;
#pragma unroll
        for (int e = E0; e < NR; ++e) {
            const int i = q + 8 * e;
            v[e] = i < n ? V[(size_t)i * lda + j] : 0.0;
            dot += v[e] * zr[e];
        }
        dot = tau * group8_sum(dot);
#pragma unroll
        for (int e = E0; e < NR; ++e) zr[e] -= dot * v[e];
    }
    if constexpr (E0 > 0) back_blocks<NR, E0 - 1>(zr, V, lda, n, q, tauv);
}

template <int NE>
__device__ void eig_precondition(double* __restrict__ R1, double* __restrict__ R2, int ld, int n, int ne,
                                 double* __restrict__ gscr, double* __restrict__ sa) {
    constexpr int NR = 2 * NE;                    // entries of a row (or column) per lane of an 8-lane group
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthr >> 6;
    const int T16 = (n + 15) / 16, ntiles = T16 * T16;
    const int lda = n | 1;                        // odd stride: rows and columns both walk all banks
    const size_t rsize = (size_t)(ne + 1) * ld;
    const int n8 = (n + 7) & ~7;
    double* dd = sa;            // [n] diagonal of T
    double* ee = dd + n;        // [n] ee[j] couples j and j+1
    double* de = ee + n;        // [2 n8] scaled T for the Sturm counts: d_k at [k], e_{k-1}^2 at [n8 + k]; padded with (4, 0): no sign change
    double* tauv = de + 2 * n8; // [n] Householder tau
    double* scl = tauv + n;     // [n] v_i = A[i][j] * scl[j] for i > j+1, v_{j+1} = 1
    double* lamv = scl + n;     // [n] eigenvalues of T, ascending
    const int n16 = (n + 15) & ~15;
    double* xx = lamv + n;      // [n16] current column below the diagonal, zero up to the current row and from n up
    double* pp = xx + n16;      // [n16] A v, zero up to the current row and from n up
    __shared__ double part_k[16], part_s[2][16];  // per-wave partial sums: v^T A v, and sigma by step parity
    __shared__ unsigned long long err_s;
    __shared__ int fail_s;

    // ---- 0: L to global scratch (R1 is reused for the eigenvectors) ----
    for (size_t e = tid; e < rsize; e += nthr) gscr[e] = R1[e];
    if (tid == 0) fail_s = 0;

    // Gram of the columns of a column-major matrix M (stride ldm, nc columns of nr rows) into R2 (row-major, lda)
    auto gram_to_R2 = [&](const double* M, int ldm, bool batch) {
        for (int t0 = 0; t0 < ntiles; t0 += nwaves) {
            if (t0 + wave >= ntiles) continue;    // `wave` is a scalar: a uniform branch; a repeated tile would queue on the same matrix pipe
            const int tile = t0 + wave;
            const int ti = tile / T16, tj = tile - ti * T16;
            const int ci = 16 * ti + (lane & 15), cj = 16 * tj + (lane & 15), kq = lane >> 4;
            const double4_t acc = tile_mma(n, ci, cj, kq, [&](int i, int k) { return M[(size_t)i * ldm + k]; },
                                           [&](int k, int c) { return M[(size_t)c * ldm + k]; }, batch);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * ti + 4 * v + kq;
                if (i < n && cj < n) R2[(size_t)i * lda + cj] = acc[v];
            }
        }
    };

    // ---- 1: A = L^T L ----
    gram_to_R2(R1, ld, false);                    // the factor's column stride suits the sweeps, not these reads: no batching
    __syncthreads();
    // ---- 2: tridiagonalisation (lower), row r on lanes q = 0..7, columns q, q+8, ... in registers.
    //         Step j, two barriers: every live wave forms the reflector's scalars and its own pieces of v from
    //         column j (xx) | p_r = A[r][:] v and the wave's share of v^T A v || rank-2 update, then column j+1
    //         with its squared norm for the next step.  xx and pp are kept zero up to row j (and from n up), so
    //         dead rows and columns update by exactly zero without any test; waves whose rows are all dead only
    //         keep the barriers. ----
    {
        const int r = tid >> 3, q = tid & 7;
        const bool row_ok = r < n;
        const int nw_rows = (n + 7) >> 3;         // waves that hold rows
        double areg[NR];
#pragma unroll
        for (int e = 0; e < NR; ++e) {
            const int c = q + 8 * e;
            areg[e] = (row_ok && c < n) ? R2[(size_t)r * lda + c] : 0.0;
        }
        for (int c = tid; c < n16; c += nthr) { pp[c] = 0.0; xx[c] = 0.0; }
        __syncthreads();
        {
            if (row_ok && q == 0 && r >= 1) xx[r] = areg[0];
            const double y = (row_ok && r >= 2 && q == 0) ? areg[0] * areg[0] : 0.0;
            const double t = wave_sum_of_groups8(group8_sum(y));
            if (lane == 0 && wave < 16) { part_s[0][wave] = t; part_s[1][wave] = 0.0; part_k[wave] = 0.0; }
        }
        auto step = [&](int j, auto ES) {
            constexpr int es = decltype(ES)::value;            // (j + 1) / 8: the register block of column j + 1
            __syncthreads();                      // column j (xx) and the partial sums of its sigma are complete
            const bool live = wave < nw_rows && 8 * wave + 7 > j;       // some row of this wave is below row j
            double vreg[NR], vr = 0.0, tau = 0.0;
            if (live || wave == 0) {
                // every live wave works out the reflector's scalars for itself: cheaper than a third barrier
                const double sg = group_sum<16>((lane & 15) < nw_rows ? part_s[j & 1][lane & 15] : 0.0);
                const double alpha = xx[j + 1];
                double scale = 0.0, beta = alpha;
                if (sg > 0.0) {
                    const double h = alpha * alpha + sg;
                    double ri = __builtin_amdgcn_rsq(h);          // 1/sqrt(h), two Newton steps
                    ri = ri * (1.5 - 0.5 * h * ri * ri);
                    ri = ri * (1.5 - 0.5 * h * ri * ri);
                    const double nr = h * ri;
                    beta = alpha >= 0.0 ? -nr : nr;
                    tau = (beta - alpha) * (alpha >= 0.0 ? -ri : ri);
                    scale = rcp_nr2(alpha - beta);
                }
                if (tid == 0) { pp[j] = 0.0; ee[j] = beta; tauv[j] = tau; scl[j] = scale; }
                // v_c = x_c * scale below row j+1 (xx is zero up to row j), 1 at row j+1
                const int qj = (j + 1) & 7;
#pragma unroll
                for (int e = 0; e < NR; ++e) vreg[e] = xx[q + 8 * e] * scale;
                if (q == qj) vreg[es] = 1.0;
                vr = r == j + 1 ? 1.0 : xx[r] * scale;
            }
            if (live) {                           // p_r = sum_c A[r][c] v_c
                double p0 = 0.0, p1 = 0.0;
#pragma unroll
                for (int e = 0; e < NR; e += 2) {
                    p0 += areg[e] * vreg[e];
                    if (e + 1 < NR) p1 += areg[e + 1] * vreg[e + 1];
                }
                const double p = group8_sum(p0 + p1);
                const double t = wave_sum_of_groups8(p * vr);
                if (q == 0 && r > j && row_ok) pp[r] = p;
                if (lane == 0) part_k[wave] = t;
            } else if (lane == 0 && wave < nw_rows) {
                part_k[wave] = 0.0;
                part_s[(j + 1) & 1][wave] = 0.0;
            }
            __syncthreads();
            if (tid == 0) xx[j + 1] = 0.0;        // the column's head is spent: rows up to j+1 read as zero from now on
            if (live) {
                const double ks = group_sum<16>((lane & 15) < nw_rows ? part_k[lane & 15] : 0.0);
                const double K = 0.5 * tau * tau * ks;
                const double wr = tau * pp[r] - K * vr;
#pragma unroll
                for (int e = 0; e < NR; ++e) {
                    const double wc = tau * pp[q + 8 * e] - K * vreg[e];
                    areg[e] -= vr * wc + wr * vreg[e];
                }
                // column j+1 below its diagonal for the next step, and the partial sums of its sigma
                const double xn = areg[es];
                const bool own = q == ((j + 1) & 7);
                if (own && r >= j + 2 && row_ok) xx[r] = xn;
                const double y = (own && r >= j + 3 && row_ok) ? xn * xn : 0.0;
                const double t = wave_sum_of_groups8(group8_sum(y));
                if (lane == 0) part_s[(j + 1) & 1][wave] = t;
            }
        };
        for_each_block<NR>([&](auto ES) {
            constexpr int es = decltype(ES)::value;
            const int jlo = es == 0 ? 0 : 8 * es - 1, jhi = min(8 * es + 6, n - 3);
            for (int j = jlo; j <= jhi; ++j) step(j, ES);
        });
        __syncthreads();
        // the reflectors, normalised, stay in the strict lower triangle: v^(j)_i = R2[i][j] for every i (zeros down
        // to the diagonal, 1 below it); the diagonal and the subdiagonal move to dd, ee first
#pragma unroll
        for (int e = 0; e < NR; ++e) {
            const int c = q + 8 * e;
            if (row_ok && c < n) {
                if (c == r) dd[r] = areg[e];
                if (c == r - 1 && r == n - 1) ee[n - 2] = areg[e];
                double v = 0.0;
                if (c + 2 < n) v = r == c + 1 ? 1.0 : (r > c + 1 ? areg[e] * scl[c] : 0.0);
                R2[(size_t)r * lda + c] = v;
            }
        }
        if (tid == 0) { tauv[n - 2] = 0.0; tauv[n - 1] = 0.0; ee[n - 1] = 0.0; }
        __syncthreads();
    }
    // ---- 3: eigenvalues of T.  Scale T by a power of two so that |d| + 2|e| <= 1, then multisection ----
    {
        if (wave == 0) {
            double g = 0.0;
            for (int i = lane; i < n; i += 64)
                g = fmax(g, fabs(dd[i]) + fabs(ee[i]) + (i ? fabs(ee[i - 1]) : 0.0));
            g = wave_max(g);
            const double s = g > 0.0 ? ldexp(1.0, -ilogb(g) - 1) : 1.0;
            for (int i = lane; i < n8; i += 64) {
                const double d = i < n ? dd[i] * s : 4.0, e = i < n ? ee[i] * s : 0.0;
                if (i < n) { dd[i] = d; ee[i] = e; }
                de[i] = d;
                if (i + 1 < n8) de[n8 + i + 1] = e * e;
                if (i == 0) de[n8] = 0.0;
            }
        }
        __syncthreads();
        const int i = tid >> 3, q = tid & 7;
        if (i < n) {
            double lo = -1.0 - 1e-9, hi = 1.0 + 1e-9;       // Gershgorin after scaling
            for (int round = 0; round < PRE_MAX_ROUNDS; ++round) {
                // enough once the interval is below 1e-11 of the spectrum's scale and 1e-6 of the eigenvalue itself
                // (small eigenvalues of a graded matrix keep going); the lanes of a wave leave together
                const bool done = round >= PRE_ROUNDS && (hi - lo) <= 1e-6 * fmax(fabs(lo), fabs(hi));
                if (__ballot(!done) == 0ull) break;
                const double w = (hi - lo) * (1.0 / 9.0);
                const double mu = lo + w * (double)(q + 1);
                // Sturm count: sign changes in the sequence of leading principal minors of T - mu,
                // p_k = (d_k - mu) p_{k-1} - e_{k-1}^2 p_{k-2}; the pair is renormalised every 8 steps
                double p2 = 0.0, p1 = 1.0;
                int cnt = 0, hprev = 0;
                for (int k0 = 0; k0 < n8; k0 += 8) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const double p = (de[k0 + u] - mu) * p1 - de[n8 + k0 + u] * p2;
                        const int h = __double2hiint(p);
                        cnt += (unsigned)(h ^ hprev) >> 31;
                        hprev = h;
                        p2 = p1; p1 = p;
                    }
                    const int ex = max((__double2hiint(p1) >> 20) & 0x7ff, (__double2hiint(p2) >> 20) & 0x7ff);
                    p1 = ldexp(p1, 1023 - ex);
                    p2 = ldexp(p2, 1023 - ex);
                }
                // probes at or below lambda_i have cnt <= i; they form a prefix of the group's 8 lanes
                const unsigned long long b = __ballot(cnt <= i);
                const int k0 = __popc((unsigned)((b >> (lane & 56)) & 0xFFull));
                const double nlo = k0 > 0 ? lo + w * (double)k0 : lo;
                const double nhi = k0 < 8 ? lo + w * (double)(k0 + 1) : hi;
                lo = nlo; hi = nhi;
            }
            if (q == 0) lamv[i] = 0.5 * (lo + hi);
        }
        __syncthreads();
        // eigenvalues closer than the accuracy of the vectors that follow (repeated eigenvalues, rank deficiency):
        // those vectors would not come out orthogonal, so the remaining phases are skipped
        if (tid + 1 < n) {
            const double a = lamv[tid], b = lamv[tid + 1], m = fmax(fabs(a), fabs(b));
            if (b - a < 1e-9 * m || m < 1e-14) atomicOr(&fail_s, 1);    // relative: a graded spectrum is fine
        }
        __syncthreads();
    }
    // ---- 4: eigenvectors of T by twisted factorisation, thread i -> column i of Z (R1, column-major, lda) ----
    const bool early_fail = fail_s != 0;          // uniform: read after a barrier
    if (tid < n && !early_fail) {
        double* z = R1 + (size_t)tid * lda;
        const double lam = lamv[tid], pm = 1e-100;
        auto e2_ = [&](int k) { return de[n8 + k + 1]; };    // e_k^2, k = 0 .. n-2
        auto piv = [&](double D) { return fabs(D) < pm ? -pm : D; };
        // forward pivots D+ into z
        double D = dd[0] - lam;
        z[0] = D;
        for (int k = 1; k < n; ++k) {
            D = (dd[k] - lam) - e2_(k - 1) * rcp_nr2(piv(D));
            z[k] = D;
        }
        // backward pivots D- over z, remembering where |gamma_k| = |D+_k + D-_k - (d_k - lam)| is smallest
        double Dm = dd[n - 1] - lam;
        double best = fabs(z[n - 1]);                        // gamma_{n-1} = D+_{n-1}
        int rr = n - 1;
        z[n - 1] = Dm;
        for (int k = n - 2; k >= 0; --k) {
            const double a = dd[k] - lam;
            Dm = a - e2_(k) * rcp_nr2(piv(Dm));
            const double gam = fabs(z[k] + Dm - a);
            if (gam < best) { best = gam; rr = k; }
            z[k] = Dm;
        }
        // forward pivots again for the rows above the twist
        D = dd[0] - lam;
        if (rr > 0) z[0] = D;
        for (int k = 1; k < rr; ++k) {
            D = (dd[k] - lam) - e2_(k - 1) * rcp_nr2(piv(D));
            z[k] = D;
        }
        // z_rr = 1; upwards z_k = -e_k z_{k+1} / D+_k; downwards z_{k+1} = -e_k z_k / D-_{k+1}
        double zz = 1.0, nrm2 = 1.0;
        for (int k = rr - 1; k >= 0; --k) {
            zz = -ee[k] * zz * rcp_nr2(piv(z[k]));
            z[k] = zz;
            nrm2 += zz * zz;
        }
        zz = 1.0;
        for (int k = rr; k + 1 < n; ++k) {
            zz = -ee[k] * zz * rcp_nr2(piv(z[k + 1]));
            z[k + 1] = zz;
            nrm2 += zz * zz;
        }
        z[rr] = 1.0;
        if (!(nrm2 < 1e300)) atomicOr(&fail_s, 1);
        const double rn = rsqrt_nr(nrm2);
        for (int k = 0; k < n; ++k) z[k] *= rn;
    }
    __syncthreads();
    // ---- 5: P = H_0 H_1 ... H_{n-3} Z, column c on lanes q = 0..7.  Reflector j is zero in rows 0 .. j, so the
    //         register blocks e < (j+1)/8 are skipped (one instantiation of the inner loop per first block) ----
    {
        const int c = tid >> 3, q = tid & 7;
        if (c < n && !early_fail) {
            double* z = R1 + (size_t)c * lda;
            double zr[NR];
#pragma unroll
            for (int e = 0; e < NR; ++e) zr[e] = (q + 8 * e < n) ? z[q + 8 * e] : 0.0;
            back_blocks<NR, NR - 1>(zr, R2, lda, n, q, tauv);
#pragma unroll
            for (int e = 0; e < NR; ++e)
                if (q + 8 * e < n) z[q + 8 * e] = zr[e];
        }
    }
    __syncthreads();
    // ---- 6: orthogonality check and Newton-Schulz polish ----
    bool ok = fail_s == 0;
    for (int it = 0; it < 4 && ok; ++it) {
        if (tid == 0) err_s = 0ull;
        gram_to_R2(R1, lda, true);                // E + I = P^T P
        __syncthreads();
        double m = 0.0;
        for (int e = tid; e < n * n; e += nthr) {
            const int i = e / n, j = e - i * n;
            m = fmax(m, fabs(R2[(size_t)i * lda + j] - (i == j ? 1.0 : 0.0)));
        }
        m = wave_max(m);
        if (lane == 0) atomicMax(&err_s, (unsigned long long)__double_as_longlong(m));
        __syncthreads();
        const double err = __longlong_as_double((long long)err_s);
        __syncthreads();
        if (!(err < 0.03)) { ok = false; break; }
        if (err < 1e-10) break;
        if (it == 3) { ok = false; break; }
        const bool last = err < 1e-4;             // one step squares the error (to < 1e-8): no need to look again
        // P <- P - P E / 2: every wave first forms its output tiles, then all store
        double4_t acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int tile = wave + t * nwaves;
            if (tile >= ntiles) continue;
            const int ti = tile / T16, tj = tile - ti * T16;
            const int ia = 16 * ti + (lane & 15), jb = 16 * tj + (lane & 15), kq = lane >> 4;
            acc[t] = tile_mma(n, ia, jb, kq, [&](int i, int k) { return R1[(size_t)k * lda + i]; },
                              [&](int k, int c) { return R2[(size_t)k * lda + c] - (k == c ? 1.0 : 0.0); });
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int tile = wave + t * nwaves;
            if (tile < ntiles) {
                const int ti = tile / T16, tj = tile - ti * T16;
                const int jb = 16 * tj + (lane & 15), kq = lane >> 4;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = 16 * ti + 4 * v + kq;
                    if (i < n && jb < n) R1[(size_t)jb * lda + i] -= 0.5 * acc[t][v];
                }
            }
        }
        __syncthreads();
        if (last) break;
    }
    // ---- 7: W0 = L P into R2 (or L itself when the preconditioner was dropped) ----
    __syncthreads();
    for (size_t e = tid; e < rsize; e += nthr) R2[e] = ok ? 0.0 : gscr[e];
    __syncthreads();
    if (ok) {
        for (int t0 = 0; t0 < ntiles; t0 += nwaves) {
            if (t0 + wave >= ntiles) continue;
            const int tile = t0 + wave;
            const int ti = tile / T16, tj = tile - ti * T16;
            const int ia = 16 * ti + (lane & 15), jb = 16 * tj + (lane & 15), kq = lane >> 4;
            const double4_t a4 = tile_mma(n, ia, jb, kq, [&](int i, int k) { return gscr[(size_t)k * ld + i]; },   // L[i][k]
                                          [&](int k, int c) { return R1[(size_t)c * lda + k]; });       // P[k][c]
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * ti + 4 * v + kq;
                if (i < n && jb < n) R2[(size_t)jb * ld + i] = a4[v];
            }
        }
    }
    __syncthreads();
}

// One-sided Jacobi on the Cholesky factor of G.  JGL lanes share a pair of columns, NE = ceil(n / JGL)
// elements of each column per lane; the two columns of a group live in registers for a whole sweep.
//
// Ordering: odd-even transposition.  The active columns sit in slots 0 .. m-1; on even steps group g
// rotates slots (2g, 2g+1), on odd steps slots (2g+1, 2g+2), and after every rotation the two
// columns trade slots, so in m steps every pair of columns meets exactly once.  Between steps a
// group keeps one column and passes the other to a neighbour through an LDS mailbox (one column
// written and one read per group and step, one barrier per step).
//
// Deflation: a column that met every partner of a sweep without rotating is orthogonal (to tol)
// to all the others, and rotations among the others keep it so; it leaves the tournament, and
// the later sweeps run over the columns that still move.
template <int NE, int JGL>
__global__ void __launch_bounds__(1024)
k_jacobi_eig(const JacobiBatch batch, int n, int kk, int use_pre) {
    extern __shared__ double sm[];
    const JacobiProblem& prob = batch.p[blockIdx.x];
    const double* __restrict__ G = prob.G;
    double* __restrict__ lam = prob.lam;
    double* __restrict__ vec = prob.vec;
    double* __restrict__ tmat = prob.tmat;
    float* __restrict__ sval = prob.sval;
    double* __restrict__ gscr = use_pre ? prob.gscr : nullptr;
    const int ne = n + (n & 1);             // even number of columns (a zero column pads odd n)
    // Column stride = 8 (mod 16) doubles spreads the columns that one LDS instruction touches over the banks.
    const int ld = jacobi_ld(n, JGL);
    const size_t rsize = (size_t)(ne + 1) * ld;
    // gscr != nullptr: the eigenvector preconditioner runs and needs a second matrix-sized region
    double* W = sm;                              // column-major: W[p*ld + i] = element i of column p; column ne is a spare zero column
    double* mailn = sm + (gscr ? 2 : 1) * rsize; // [ne/2] squared norm of the column in transit to even slot 2j
    double* nrm = mailn + ne / 2;                // [ne + 1]
    int* order = (int*)(nrm + ne + 1);           // [ne]
    int* colmap = order + ne;                    // [ne + 1] slot -> column of the columns still rotating
    int* rotf = colmap + ne + 1;                 // [ne + 1] column took part in a rotation this sweep
    // [10 n + 40] the preconditioner's vectors, past the int arrays, on an even double index (16-byte loads)
    double* pre_sa = sm + (((gscr ? 2 : 1) * rsize + ne / 2 + ne + 1 + (3 * ne + 4) / 2 + 2) & ~(size_t)1);
    __shared__ int nact_sh, wcnt[2];
    __shared__ double amax_sh;
    const int tid = threadIdx.x, nthr = blockDim.x, grp = tid / JGL, gl = tid % JGL;

    for (int e = tid; e < (ne + 1) * ld; e += nthr) {
        int p = e / ld, i = e - p * ld;
        W[e] = (p < n && i < n) ? G[(size_t)i * n + p] : 0.0;
    }
    if (tid <= ne) { colmap[tid] = tid; rotf[tid] = 0; nrm[tid] = 0.0; }
    if (tid == 0) { nact_sh = ne; wcnt[0] = 0; wcnt[1] = 0; }
    __syncthreads();
    // Precondition: replace G by its Cholesky factor L (G = L L^T, column j of L in column j of W).
    // The columns of L are far closer to orthogonal than those of G (one Cholesky-LR step), the
    // rotations then converge in about half the sweeps, and column j ends as sigma_j u_j with
    // sigma_j^2 = lambda_j, u_j the eigenvector of G.  A pivot at rounding level (semi-definite G)
    // zeroes its column.
    {
        __shared__ double piv_floor;
        __shared__ double rinv_sh[SM_MAX_N];
        if (tid == 0) {
            double m = 0.0;
            for (int j = 0; j < n; ++j) m = fmax(m, W[(size_t)j * ld + j]);
            piv_floor = m * 1e-30;
        }
        __syncthreads();
        chol_blocked<true>(W, ld, n, rinv_sh, piv_floor, nullptr);
        // the rotations work on whole columns: clear the part above the diagonal
        for (int e = tid; e < n * n; e += nthr) {
            const int c = e / n, i = e - c * n;
            if (i < c) W[(size_t)c * ld + i] = 0.0;
        }
        __syncthreads();
    }
    if (gscr) {
        eig_precondition<NE>(sm, sm + rsize, ld, n, ne, gscr, pre_sa);
        W = sm + rsize;
    }

    // Rotate while gamma^2 > tol^2 alpha beta + (c eps)^2 amax (alpha + beta), tol = 1e-7: the
    // eigenvectors are then accurate to ~1e-7 / (relative gap), far inside the 1e-2 rad the split needs.  The second term is
    // the rounding floor of a dot product of two columns that each carry an absolute error of
    // ~eps * lambda_max (the columns are lambda_j v_j, formed from O(lambda_max) entries): below it
    // a rotation only reshuffles noise and the sweeps would never end.
    const double tol2 = 1e-14, floor2 = 1e-28;
    double amax = 0.0;
    double X[NE], Y[NE];
    double nX = 0.0, nY = 0.0;

    // rows n .. JGL*NE-1 of every column are zero padding: no bounds checks
    auto load_col = [&](double* dst, const double* src) {
#pragma unroll
        for (int e = 0; e < NE; ++e) dst[e] = src[gl + JGL * e];
    };
    auto store_col = [&](double* dst, const double* src) {
#pragma unroll
        for (int e = 0; e < NE; ++e) dst[gl + JGL * e] = src[e];
    };
    // orthogonalise the pair in registers: X <- c X - s Y, Y <- s X + c Y.  The squared norms travel with
    // their columns; a set sign bit marks a column that has rotated in this sweep.
    auto rotate = [&]() {
        double g0 = 0.0, g1 = 0.0;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if (e & 1) g1 += X[e] * Y[e]; else g0 += X[e] * Y[e];
        }
        const double gamma = group_sum<JGL>(g0 + g1);
        const double a = fabs(nX), b = fabs(nY);
        // (a zero column gives gamma = 0 and never passes the test)
        if (gamma * gamma > tol2 * a * b + floor2 * amax * (a + b)) {
            // With tau = beta - alpha and hyp = sqrt(tau^2 + 4 gamma^2) the rotation that zeroes the pair
            // (angle at most 45 degrees) has c^2 = (1 + |tau| / hyp) / 2 and s c = sign(tau) gamma / hyp.
            // The hardware reciprocal square roots are good to ~1e-7, which only steers the angle; the
            // pair (c, s) is then rescaled to unit length to second order (error ~1e-21).
            const double tau = b - a;
            const double hh = tau * tau + 4.0 * gamma * gamma;
            const double rh = __builtin_amdgcn_rsq(hh);
            const double c2 = 0.5 + 0.5 * fabs(tau) * rh;
            const double rc = __builtin_amdgcn_rsq(c2);
            double c = c2 * rc;
            double s = (tau < 0.0 ? -gamma : gamma) * rh * rc;
            const double d = c * c + (s * s - 1.0);
            const double f = 1.0 + d * (0.375 * d - 0.5);
            c *= f;
            s *= f;
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const double x = X[e], y = Y[e];
                X[e] = c * x - s * y;
                Y[e] = s * x + c * y;
            }
            // squared norms after the rotation (their sum is preserved), flagged as rotated
            const double na = fabs(a + (s * s) * tau - 2.0 * (c * s) * gamma);
            nX = -na;
            nY = -fabs((a + b) - na);
        }
    };

    for (int sweep = 0; sweep < 40; ++sweep) {
        const int m = nact_sh, gs = m / 2;           // even number of slots, groups this sweep
        const bool act = grp < gs, inner = grp < gs - 1;
        int idX = ne, idY = ne;
        if (act) {
            idX = colmap[2 * grp];
            idY = colmap[2 * grp + 1];
            load_col(X, W + (size_t)idX * ld);
            load_col(Y, W + (size_t)idY * ld);
            double sx = 0.0, sy = 0.0;
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                sx += X[e] * X[e];
                sy += Y[e] * Y[e];
            }
            nX = group_sum<JGL>(sx);              // exact squared norms at the start of every sweep
            nY = group_sum<JGL>(sy);
        }
        double* const mail_lo = W + (size_t)idX * ld;                                  // mailbox of slot 2g
        double* const mail_hi = W + (size_t)(inner ? colmap[2 * grp + 2] : ne) * ld;   // mailbox of slot 2g + 2
        // a full sweep reverses the slot order: the columns this group ends up with
        const int endX = act ? colmap[m - 1 - 2 * grp] : ne, endY = act ? colmap[m - 2 - 2 * grp] : ne;
        __syncthreads();                          // every column is in registers before the first mailbox write
        if (sweep == 0) {
            if (act && gl == 0) { nrm[idX] = nX; nrm[idY] = nY; }
            __syncthreads();
            if (tid == 0) {
                double mx = 0.0;
                for (int j = 0; j < ne; ++j) mx = fmax(mx, nrm[j]);
                amax_sh = mx;
            }
            __syncthreads();
            amax = amax_sh;
        }
        for (int s2 = 0; s2 < gs; ++s2) {
            // even step: slots (2g, 2g+1) are (X, Y); afterwards Y moves down to group g-1
            if (act) {
                rotate();
                store_col(mail_lo, Y);
                mailn[grp] = nY;                  // all lanes of the group write the same value
            }
            __syncthreads();
            if (inner) {
                load_col(Y, mail_hi);
                nY = mailn[grp + 1];
            }
            // odd step: slots (2g+1, 2g+2) are (X, Y); afterwards X moves up to group g+1.  The last
            // group holds the unpaired top slot and only renames it.
            if (inner) {
                rotate();
                store_col(mail_hi, X);
                mailn[grp + 1] = nX;
            } else if (act) {
#pragma unroll
                for (int e = 0; e < NE; ++e) Y[e] = X[e];
                nY = nX;
            }
            __syncthreads();
            if (act) {
                load_col(X, mail_lo);
                nX = mailn[grp];
            }
        }
        __syncthreads();                          // the last mailbox reads are done
        if (act) {
            store_col(W + (size_t)endX * ld, X);
            store_col(W + (size_t)endY * ld, Y);
            if (gl == 0) {
                if (__double2hiint(nX) < 0) rotf[endX] = 1;
                if (__double2hiint(nY) < 0) rotf[endY] = 1;
            }
        }
        // keep the columns that rotated, in slot order
        int myc = -1, f = 0;
        __syncthreads();
        if (tid < m) { myc = colmap[tid]; f = rotf[myc]; }
        const unsigned long long bal = __ballot(f);
        const int wv = tid >> 6, ln = tid & 63;
        if (ln == 0 && wv < 2) wcnt[wv] = __popcll(bal);
        __syncthreads();
        const int total = wcnt[0] + wcnt[1];
        if (f) {
            colmap[__popcll(bal & ((1ull << ln) - 1ull)) + (wv == 1 ? wcnt[0] : 0)] = myc;
            rotf[myc] = 0;
        }
        if (tid == 0) {
            if (total & 1) colmap[total] = ne;
            nact_sh = total + (total & 1);
        }
        __syncthreads();
        if (total == 0) break;
    }
    // column norms = singular values of L = square roots of the eigenvalues
    for (int pp = grp; pp < ne; pp += nthr / JGL) {
        double s = 0.0;
        for (int i = gl; i < n; i += JGL) s += W[(size_t)pp * ld + i] * W[(size_t)pp * ld + i];
        s = group_sum<JGL>(s);
        if (gl == 0) nrm[pp] = (pp < n) ? sqrt(s) : -1.0;
    }
    __syncthreads();
    if (tid < ne) {                          // rank by counting: descending, ties by index
        double me = nrm[tid];
        int r = 0;
        for (int j = 0; j < ne; ++j) r += (nrm[j] > me) || (nrm[j] == me && j < tid);
        order[r] = tid;
    }
    __syncthreads();
    for (int e = tid; e < n * n; e += nthr) {
        int i = e / n, j = e - i * n;
        int pp = order[j];
        double l = nrm[pp];
        double v = l > 0.0 ? W[(size_t)pp * ld + i] / l : (i == j ? 1.0 : 0.0);
        if (vec) vec[e] = v;
        if (tmat && j < kk) tmat[(size_t)i * kk + j] = l > 0.0 ? v / l : 0.0;
    }
    if (tid < n) {
        double l = nrm[order[tid]];              // sigma_j = sqrt(lambda_j)
        lam[tid] = l * l;
        if (sval && tid < kk) sval[tid] = (float)l;
    }
}

int launch_chol_inv_batch(hipStream_t s, const CholProblem* probs, int count, int n) {
    if (n < 1 || n > SM_MAX_CHOL || count < 0) return METIS_UNSUPPORTED;
    size_t lds = 2 * (size_t)n * (n + 1) * sizeof(double);
    static LdsLimitCache lds_set;
    if (!ensure_dyn_lds((const void*)k_chol_inv, lds, lds_set)) return METIS_HIP_ERROR;
    for (int b0 = 0; b0 < count; b0 += SM_MAX_BATCH) {
        const int nb = count - b0 < SM_MAX_BATCH ? count - b0 : SM_MAX_BATCH;
        CholBatch batch;
        for (int i = 0; i < SM_MAX_BATCH; ++i) batch.p[i] = probs[b0 + (i < nb ? i : 0)];
        hipLaunchKernelGGL(k_chol_inv, dim3(nb), dim3(1024), lds, s, batch, n);
        METIS_LAUNCH_CHECK();
    }
    return METIS_OK;
}

int launch_jacobi_eig_batch(hipStream_t s, const JacobiProblem* probs, int count, int n, int kk) {
    if (n < 1 || n > 128 || count < 0) return METIS_UNSUPPORTED;
    const int jgl = jacobi_lanes(n);
    const int ne = n + (n & 1), ld = jacobi_ld(n, jgl);
    const size_t rsize = (size_t)(ne + 1) * ld;
    const size_t small = ((size_t)ne / 2 + ne + 1) * sizeof(double) + (size_t)(3 * ne + 4) * sizeof(int) + 16;
    // the preconditioner needs two matrix-sized regions and 10 n + 40 doubles; it pays from n ~ 72 on (about 250 us
    // against 7 of 9 sweeps of 46 us at n = 80; at n = 64 the plain sweeps win), and its second region fits in
    // the 160 KB of LDS up to n = 88.  It runs when every problem of the batch brings scratch.
    size_t lds = rsize * sizeof(double) + small;
    const size_t lds_pre = 2 * rsize * sizeof(double) + small + (10 * (size_t)n + 44) * sizeof(double);
    bool all_scratch = count > 0;
    for (int i = 0; i < count; ++i) all_scratch = all_scratch && probs[i].gscr != nullptr;
    const int use_pre = all_scratch && n >= 72 && lds_pre <= 160 * 1024;
    if (use_pre) lds = lds_pre;
    // one group of jgl lanes per column pair, in whole waves and at least 512 threads (the Cholesky pre-pass, the
    // bookkeeping and the preconditioner's 8 lanes per row use them); no idle waves beyond that: every wave of
    // the workgroup takes part in every barrier
    const int need = (ne / 2 * jgl + 63) / 64 * 64;
    const int threads = need > 512 ? need : 512;
    if (ne / 2 * jgl > threads) return METIS_UNSUPPORTED;
    for (int b0 = 0; b0 < count; b0 += SM_MAX_BATCH) {
        const int nb = count - b0 < SM_MAX_BATCH ? count - b0 : SM_MAX_BATCH;
        JacobiBatch batch;
        for (int i = 0; i < SM_MAX_BATCH; ++i) batch.p[i] = probs[b0 + (i < nb ? i : 0)];
#define JACOBI_CASE(NE, JGL)                                                                                  \
    {                                                                                                         \
        static LdsLimitCache lds_set;                                                                         \
        if (!ensure_dyn_lds((const void*)k_jacobi_eig<NE, JGL>, lds, lds_set)) return METIS_HIP_ERROR;        \
        hipLaunchKernelGGL((k_jacobi_eig<NE, JGL>), dim3(nb), dim3(threads), lds, s, batch, n, kk, use_pre);  \
    }
        switch ((n + 15) / 16) {
            case 1: JACOBI_CASE(1, 16) break;
            case 2: JACOBI_CASE(2, 16) break;
            case 3: JACOBI_CASE(3, 16) break;
            case 4: JACOBI_CASE(4, 16) break;
            case 5: JACOBI_CASE(5, 16) break;
            case 6: JACOBI_CASE(6, 16) break;
            case 7: JACOBI_CASE(7, 16) break;
            default: JACOBI_CASE(8, 16) break;
        }
#undef JACOBI_CASE
        METIS_LAUNCH_CHECK();
    }
    return METIS_OK;
}

size_t jacobi_scratch_doubles(int n) {
    const int ne = n + (n & 1);
    return (size_t)(ne + 1) * jacobi_ld(n, jacobi_lanes(n));
}
