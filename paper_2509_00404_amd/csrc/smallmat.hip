// One-workgroup fp64 factorizations of the small (k+p)x(k+p) matrices of the decomposition
// (Sec. 3.1): Cholesky + triangular inverse for CholeskyQR2 (thin QR Z = H R), and a
// one-sided Jacobi eigensolver for the Gram matrices of the reduced problem.
#include "smallmat.h"
#include <cstdlib>

// ---------------------------------------------------------------------------------------
// Cholesky G = L L^T and Linv = L^-1 (lower triangular), n <= SM_MAX_N.
// LDS: L [n][n+1] doubles, X [n][n+1] doubles.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double chol_rsqrt(double x) {
    double y = __builtin_amdgcn_rsq(x);
    y = y * (1.5 - 0.5 * x * y * y);
    y = y * (1.5 - 0.5 * x * y * y);
    return y;
}

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
k_chol_inv(const double* __restrict__ G, int n, double* __restrict__ Linv, int32_t* __restrict__ info) {
    extern __shared__ double sm[];
    const int ld = n + 1;
    double* L = sm;
    double* X = sm + (size_t)n * ld;
    __shared__ double dinv[SM_MAX_CHOL];
    const int tid = threadIdx.x;
    for (int e = tid; e < n * n; e += 1024) {
        int i = e / n, j = e - i * n;
        L[i * ld + j] = G[e];
        X[i * ld + j] = 0.0;
    }
    __syncthreads();
    // right-looking Cholesky, one barrier per column: the trailing update uses the unscaled
    // column and 1/pivot; the columns are scaled by 1/sqrt(pivot) in one pass at the end
    const int ti = tid >> 5, tc = tid & 31;
    for (int j = 0; j < n; ++j) {
        double d = L[j * ld + j];
        if (!(d > 0.0)) {                   // rank-deficient sketch: flag it, keep going finitely
            if (tid == 0 && info) *info = j + 1;
            d = 1e-300;
        }
        const double r = chol_rsqrt(d);
        if (tid == 0) dinv[j] = r;
        const double r2 = r * r;
        for (int i = j + 1 + ti; i < n; i += 32) {
            double lij = L[i * ld + j] * r2;
            for (int c = j + 1 + tc; c <= i; c += 32) L[i * ld + c] -= lij * L[c * ld + j];
        }
        __syncthreads();
    }
    for (int e = tid; e < n * n; e += 1024) {
        int i = e / n, j = e - i * n;
        if (j <= i) {
            double v = L[i * ld + j];
            if (i == j && !(v > 0.0)) v = 1e-300;
            L[i * ld + j] = v * dinv[j];
        }
    }
    __syncthreads();
    // forward substitution: column c of L^-1 by a group of 8 lanes (same wave, so the group's own
    // LDS writes are visible to it without a workgroup barrier); X[t][c] keeps groups conflict-free
    {
        const int c = tid >> 3, gl = tid & 7;
        if (c < n) {
            for (int i = c; i < n; ++i) {
                double s = 0.0;
                for (int t = c + gl; t < i; t += 8) s -= L[i * ld + t] * X[t * ld + c];
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
    int* mailid = rotf + ne + 1;                 // [ne/2] column index of the column in transit
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
        if (tid == 0) {
            double m = 0.0;
            for (int j = 0; j < n; ++j) m = fmax(m, W[(size_t)j * ld + j]);
            piv_floor = m * 1e-30;
        }
        __syncthreads();
        for (int j = 0; j < n; ++j) {
            const double d = W[(size_t)j * ld + j];
            const bool ok = d > piv_floor;
            const double r = ok ? rsqrt_nr(d) : 0.0, r2 = r * r;
            // trailing update with the unscaled column j: L[i][c] -= L[i][j] L[c][j] / d   (i >= c > j);
            // 16 threads walk down each column
            for (int c = j + 1 + (tid >> 4); c < n; c += nthr >> 4) {
                const double f = W[(size_t)j * ld + c] * r2;
                for (int i = c + (tid & 15); i < n; i += 16) W[(size_t)c * ld + i] -= W[(size_t)j * ld + i] * f;
            }
            __syncthreads();
            // scale column j, clear the part above the diagonal (row index < column index)
            for (int i = tid; i < n; i += nthr) {
                double v = i >= j ? W[(size_t)j * ld + i] * r : 0.0;
                W[(size_t)j * ld + i] = v;
            }
            // (column j is not read again by later steps, no barrier needed before the next pivot read:
            //  the next pivot W[j+1][j+1] was finalised by the update above)
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
    int idX = ne, idY = ne;

    // rows n .. JGL*NE-1 of every column are zero padding: no bounds checks
    auto load_col = [&](double* dst, const double* src) {
#pragma unroll
        for (int e = 0; e < NE; ++e) dst[e] = src[gl + JGL * e];
    };
    auto store_col = [&](double* dst, const double* src) {
#pragma unroll
        for (int e = 0; e < NE; ++e) dst[gl + JGL * e] = src[e];
    };
    // orthogonalise the pair in registers: X <- c X - s Y, Y <- s X + c Y
    auto rotate = [&]() {
        double g0 = 0.0, g1 = 0.0;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if (e & 1) g1 += X[e] * Y[e]; else g0 += X[e] * Y[e];
        }
        const double gamma = group_sum<JGL>(g0 + g1);
        if (gamma * gamma > tol2 * nX * nY + floor2 * amax * (nX + nY) && nX > 0.0 && nY > 0.0) {
            // With tau = beta - alpha and hyp = sqrt(tau^2 + 4 gamma^2) the rotation that zeroes the pair
            // (angle at most 45 degrees) has c^2 = (1 + |tau| / hyp) / 2 and s c = sign(tau) gamma / hyp.
            // The hardware reciprocal square roots are good to ~1e-7, which only steers the angle; the
            // pair (c, s) is then rescaled to unit length to second order (error ~1e-21).
            const double tau = nY - nX;
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
            // squared norms after the rotation; their sum is preserved
            const double na = c * c * nX - 2.0 * c * s * gamma + s * s * nY;
            nY = (nX + nY) - na;
            nX = na;
            if (gl == 0) {
                rotf[idX] = 1;
                rotf[idY] = 1;
            }
        }
    };

    for (int sweep = 0; sweep < 40; ++sweep) {
        const int m = nact_sh, gs = m / 2;           // even number of slots, groups this sweep
        const bool act = grp < gs, inner = grp < gs - 1;
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
                if (gl == 0) { mailn[grp] = nY; mailid[grp] = idY; }
            }
            __syncthreads();
            if (inner) {
                load_col(Y, mail_hi);
                nY = mailn[grp + 1];
                idY = mailid[grp + 1];
            }
            // odd step: slots (2g+1, 2g+2) are (X, Y); afterwards X moves up to group g+1.  The last
            // group holds the unpaired top slot and only renames it.
            if (inner) {
                rotate();
                store_col(mail_hi, X);
                if (gl == 0) { mailn[grp + 1] = nX; mailid[grp + 1] = idX; }
            } else if (act) {
#pragma unroll
                for (int e = 0; e < NE; ++e) Y[e] = X[e];
                nY = nX;
                idY = idX;
            }
            __syncthreads();
            if (act) {
                load_col(X, mail_lo);
                nX = mailn[grp];
                idX = mailid[grp];
            }
        }
        __syncthreads();                          // the last mailbox reads are done
        if (act) {
            store_col(W + (size_t)idX * ld, X);
            store_col(W + (size_t)idY * ld, Y);
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

int launch_chol_inv(hipStream_t s, const double* G, int n, double* Linv, int32_t* info) {
    size_t lds = 2 * (size_t)n * (n + 1) * sizeof(double);
    if (hipFuncSetAttribute((const void*)k_chol_inv, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return METIS_HIP_ERROR;
    hipLaunchKernelGGL(k_chol_inv, dim3(1), dim3(1024), lds, s, G, n, Linv, info);
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
