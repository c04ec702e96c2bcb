// One-workgroup fp64 factorizations of the small (k+p)x(k+p) matrices of the decomposition
// (Sec. 3.1): Cholesky + triangular inverse for CholeskyQR2 (thin QR Z = H R), and a
// one-sided Jacobi eigensolver for the Gram matrices of the reduced problem.
#include "smallmat.h"
#include <cstdlib>

// ---------------------------------------------------------------------------------------
// Blocked Cholesky in LDS, shared by both kernels below.  On entry W holds the lower triangle of a
// symmetric matrix column-major (element (i, c), i >= c, at W[c*ld + i]); on exit the same places
// hold L, and rinv[c] = 1 / L[c][c].  Blocks of 4 columns, two workgroup barriers per block:
//   1  one thread per row at or below the block reads the 4x4 diagonal block (LDS broadcast), factors
//      it on its own (every thread repeats the same ~30 operations: cheaper than a barrier and a round
//      trip through LDS) and solves its row's four entries against it,
//   2  the trailing matrix takes the rank-4 update on the fp64 matrix cores: one
//      v_mfma_f64_16x16x4_f64 per 16x16 tile, the block width being exactly the instruction's depth.
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

template <bool BAD_PIVOT_ZEROES>
__device__ void chol_blocked(double* __restrict__ W, int ld, int n, double* __restrict__ rinv, double floor_,
                             int32_t* __restrict__ info) {
    const int tid = threadIdx.x, nthr = blockDim.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthr >> 6;
#ifdef JAC_PROF
    long long ca = 0, cc = 0, c0 = clock64();
#define CH_MARK(acc) { long long c1 = clock64(); acc += c1 - c0; c0 = c1; }
#else
#define CH_MARK(acc)
#endif
    for (int k0 = 0; k0 < n; k0 += 4) {
        // ---- 1: diagonal block (entries past n act as an identity block) and the rows below ----
        double d[4][4];                                  // lower triangle of the diagonal block
        double r[4];
        if (tid < n - k0) {
            const int i = k0 + tid;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int c = 0; c <= q; ++c)
                    d[q][c] = (k0 + q < n) ? W[(size_t)(k0 + c) * ld + k0 + q] : (q == c ? 1.0 : 0.0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
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
                for (int q = c + 1; q < 4; ++q) {
                    double v = d[q][c];
#pragma unroll
                    for (int t = 0; t < c; ++t) v -= d[q][t] * d[c][t];
                    d[q][c] = v * r[c];
                }
            }
            if (tid >= 4) {
                double x[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    double v = W[(size_t)(k0 + c) * ld + i];
#pragma unroll
                    for (int t = 0; t < c; ++t) v -= x[t] * d[c][t];
                    x[c] = v * r[c];
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) W[(size_t)(k0 + c) * ld + i] = x[c];
            }
        }
        __syncthreads();
        // the block's own rows are written once every thread has read the unfactored block; nothing
        // reads them again before the next barrier
        if (tid < 4 && tid < n - k0) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (tid == q) {
                    rinv[k0 + q] = r[q];
#pragma unroll
                    for (int c = 0; c <= q; ++c) W[(size_t)(k0 + c) * ld + k0 + q] = d[q][c];
                }
        }
        CH_MARK(ca)
        if (n - k0 <= 4) break;
        // ---- 2: trailing update A22 -= L21 L21^T over the 16-aligned lower tiles that reach past k0 + 4 ----
        const int t0 = (k0 + 4) & ~15;
        const int T = (n - t0 + 15) / 16, ntiles = T * (T + 1) / 2;
        for (int tile = wave; tile < ntiles; tile += nwaves) {
            int ti = 0, rem = tile;
            while (rem > ti) { rem -= ti + 1; ++ti; }       // tile -> (ti, tc), tc <= ti
            const int i0 = t0 + 16 * ti, c0 = t0 + 16 * rem;
            const int ia = i0 + (lane & 15), cb = c0 + (lane & 15);
            const size_t col = (size_t)(k0 + (lane >> 4)) * ld;
            const double av = (ia < n && ia >= k0 + 4) ? W[col + ia] : 0.0;
            const double bv = (cb < n && cb >= k0 + 4) ? W[col + cb] : 0.0;
            double4_t acc = {0.0, 0.0, 0.0, 0.0};
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
            // D: lane l, element v -> (row 4 v + l / 16, column l % 16) of the tile
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + 4 * v + (lane >> 4), c = cb;
                if (i < n && c < n && c >= k0 + 4 && i >= c) W[(size_t)c * ld + i] -= acc[v];
            }
        }
        __syncthreads();
        CH_MARK(cc)
    }
    __syncthreads();                                     // the last block's rows are visible to the caller
#ifdef JAC_PROF
    if (tid == 0) printf("chol n=%d: phase1 %lld trailing %lld\n", n, ca, cc);
#endif
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
k_chol_inv(const double* __restrict__ G, int n, double* __restrict__ Linv, int32_t* __restrict__ info,
           int32_t* __restrict__ wellcond_out, const int32_t* __restrict__ skip_in) {
    extern __shared__ double sm[];
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
    // forward substitution: column c of L^-1 by a group of 8 lanes (same wave, so the group's own
    // LDS writes are visible to it without a workgroup barrier); X[t][c] keeps groups conflict-free
    {
        const int c = tid >> 3, gl = tid & 7;
        if (c < n) {
            for (int i = c; i < n; ++i) {
                double s = 0.0;
                for (int t = c + gl; t < i; t += 8) s -= L[t * ld + i] * X[t * ld + c];
                s = chol_group8_sum(s);
                if (gl == 0) X[i * ld + c] = ((i == c ? 1.0 : 0.0) + s) * dinv[i];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
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
k_jacobi_eig(const double* __restrict__ G, int n, int kk, double* __restrict__ lam, double* __restrict__ vec,
             double* __restrict__ tmat, float* __restrict__ sval) {
    extern __shared__ double sm[];
    const int ne = n + (n & 1);             // even number of columns (a zero column pads odd n)
    // Column stride = 8 (mod 16) doubles spreads the columns that one LDS instruction touches over the banks.
    const int ld = jacobi_ld(n, JGL);
    double* W = sm;                              // column-major: W[p*ld + i] = element i of column p; column ne is a spare zero column
    double* mailn = W + (size_t)(ne + 1) * ld;   // [ne/2] squared norm of the column in transit to even slot 2j
    double* nrm = mailn + ne / 2;                // [ne + 1]
    int* order = (int*)(nrm + ne + 1);           // [ne]
    int* colmap = order + ne;                    // [ne + 1] slot -> column of the columns still rotating
    int* rotf = colmap + ne + 1;                 // [ne + 1] column took part in a rotation this sweep
    __shared__ int nact_sh, wcnt[2];
    __shared__ double amax_sh;
    const int tid = threadIdx.x, nthr = blockDim.x, grp = tid / JGL, gl = tid % JGL;

#ifdef JAC_PROF
    const long long pt0 = clock64();
#endif
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
#ifdef JAC_PROF
        const long long pt1 = clock64();
#endif
        chol_blocked<true>(W, ld, n, rinv_sh, piv_floor, nullptr);
#ifdef JAC_PROF
        if (tid == 0) printf("jacobi n=%d: load %lld chol %lld\n", n, pt1 - pt0, (long long)(clock64() - pt1));
#endif
        // the rotations work on whole columns: clear the part above the diagonal
        for (int e = tid; e < n * n; e += nthr) {
            const int c = e / n, i = e - c * n;
            if (i < c) W[(size_t)c * ld + i] = 0.0;
        }
        __syncthreads();
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

int launch_chol_inv(hipStream_t s, const double* G, int n, double* Linv, int32_t* info, int32_t* wellcond_out,
                    const int32_t* skip_in) {
    size_t lds = 2 * (size_t)n * (n + 1) * sizeof(double);
    if (hipFuncSetAttribute((const void*)k_chol_inv, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return METIS_HIP_ERROR;
    hipLaunchKernelGGL(k_chol_inv, dim3(1), dim3(1024), lds, s, G, n, Linv, info, wellcond_out, skip_in);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

int launch_jacobi_eig(hipStream_t s, const double* G, int n, int kk, double* lam, double* vec, double* tmat,
                      float* sval) {
    if (n < 1 || n > 128) return METIS_UNSUPPORTED;
    int jgl = jacobi_lanes(n);
    if (const char* e = getenv("METIS_JACOBI_LANES")) jgl = atoi(e);
    const int ne = n + (n & 1), ld = jacobi_ld(n, jgl);
    const size_t lds = ((size_t)(ne + 1) * ld + ne / 2 + ne + 1) * sizeof(double) +
                       (size_t)(3 * ne + 2 + ne / 2) * sizeof(int);
    // one group of jgl lanes per column pair; the Cholesky pre-pass and the bookkeeping use all 512 threads
    const int threads = ne / 2 * jgl > 512 ? 1024 : 512;
    if (ne / 2 * jgl > threads) return METIS_UNSUPPORTED;
#define JACOBI_CASE(NE, JGL)                                                                                  \
    {                                                                                                         \
        if (hipFuncSetAttribute((const void*)k_jacobi_eig<NE, JGL>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                (int)lds) != hipSuccess)                                                      \
            return METIS_HIP_ERROR;                                                                           \
        hipLaunchKernelGGL((k_jacobi_eig<NE, JGL>), dim3(1), dim3(threads), lds, s, G, n, kk, lam, vec, tmat, sval); \
    }
    if (jgl == 4) {
        switch ((n + 15) / 16) {
            case 1: JACOBI_CASE(4, 4) break;
            case 2: JACOBI_CASE(8, 4) break;
            case 3: JACOBI_CASE(12, 4) break;
            case 4: JACOBI_CASE(16, 4) break;
            case 5: JACOBI_CASE(20, 4) break;
            case 6: JACOBI_CASE(24, 4) break;
            case 7: JACOBI_CASE(28, 4) break;
            default: JACOBI_CASE(32, 4) break;
        }
    } else if (jgl == 8) {
        switch ((n + 15) / 16) {
            case 1: JACOBI_CASE(2, 8) break;
            case 2: JACOBI_CASE(4, 8) break;
            case 3: JACOBI_CASE(6, 8) break;
            case 4: JACOBI_CASE(8, 8) break;
            case 5: JACOBI_CASE(10, 8) break;
            case 6: JACOBI_CASE(12, 8) break;
            case 7: JACOBI_CASE(14, 8) break;
            default: JACOBI_CASE(16, 8) break;
        }
    } else if (jgl == 16) {
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
    } else {
        return METIS_UNSUPPORTED;
    }
#undef JACOBI_CASE
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
