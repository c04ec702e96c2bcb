// One-workgroup fp64 factorizations of the small (k+p)x(k+p) matrices of the decomposition
// (Sec. 3.1): Cholesky + triangular inverse for CholeskyQR2 (thin QR Z = H R), and a
// one-sided Jacobi eigensolver for the Gram matrices of the reduced problem.
#include "smallmat.h"

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
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xF, 0xF, false);
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

#define JG 8      // lanes per column pair

__host__ __device__ static inline int jacobi_ld(int n) { return ((n + 7) / 16) * 16 + 8; }

// NE = ceil(n / 8): elements of one column held by each of the 8 lanes of a group.
// blockDim = 64 * ceil(ceil(n/2) / 8): one group of 8 lanes per column pair.
template <int NE>
__global__ void __launch_bounds__(512)
k_jacobi_eig(const double* __restrict__ G, int n, int kk, double* __restrict__ lam, double* __restrict__ vec,
             double* __restrict__ tmat, float* __restrict__ sval) {
    extern __shared__ double sm[];
    const int ne = n + (n & 1);             // even number of columns (a zero column pads odd n)
    // Column stride = 8 (mod 16) doubles: the 8 groups of a wave touch 8 consecutive columns in
    // one LDS instruction, and this stride spreads them evenly over the banks.
    const int ld = jacobi_ld(n);
    double* W = sm;                         // column-major: W[p*ld + i] = element i of column p
    double* nrm = sm + (size_t)ne * ld;     // [ne] squared column norms during the sweeps
    int* order = (int*)(nrm + ne);          // [ne]
    __shared__ int rotated;
    __shared__ double amax_sh;
    const int tid = threadIdx.x, nthr = blockDim.x, grp = tid / JG, gl = tid % JG;

    for (int e = tid; e < ne * ld; e += nthr) {
        int p = e / ld, i = e - p * ld;
        W[e] = (p < n && i < n) ? G[(size_t)i * n + p] : 0.0;
    }
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
            // trailing update with the unscaled column j: L[i][c] -= L[i][j] L[c][j] / d   (i >= c > j)
            for (int e = tid; e < (n - j - 1) * (n - j - 1); e += nthr) {
                int c = j + 1 + e / (n - j - 1), i = j + 1 + e % (n - j - 1);
                if (i >= c) W[(size_t)c * ld + i] -= W[(size_t)j * ld + i] * W[(size_t)j * ld + c] * r2;
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

    const int npairs = ne / 2, nm1 = ne - 1;
    const bool active = grp < npairs;

    // Rotate while gamma^2 > tol^2 alpha beta + (c eps)^2 amax (alpha + beta), tol = 1e-7: the
    // eigenvectors are then accurate to ~1e-7 / (relative gap), far inside the 1e-2 rad the split needs.  The second term is
    // the rounding floor of a dot product of two columns that each carry an absolute error of
    // ~eps * lambda_max (the columns are lambda_j v_j, formed from O(lambda_max) entries): below it
    // a rotation only reshuffles noise and the sweeps would never end.
    const double tol2 = 1e-14, floor2 = 1e-28;
    for (int sweep = 0; sweep < 40; ++sweep) {
        // exact squared norms at the start of every sweep (the in-sweep updates only track them)
        if (active) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                int p = 2 * grp + h;
                double s = 0.0;
#pragma unroll
                for (int e = 0; e < NE; ++e) {
                    int i = gl + JG * e;
                    double x = i < n ? W[(size_t)p * ld + i] : 0.0;
                    s += x * x;
                }
                s = group8_sum(s);
                if (gl == 0) nrm[p] = s;
            }
        }
        if (tid == 0) rotated = 0;
        __syncthreads();
        if (tid == 0) {
            double m = 0.0;
            for (int j = 0; j < ne; ++j) m = fmax(m, nrm[j]);
            amax_sh = m;
        }
        __syncthreads();
        const double amax = amax_sh;
        // round-robin pairing: column nm1 stays, the others rotate through the slots
        int p = grp == 0 ? nm1 : grp % nm1;
        int q = grp == 0 ? 0 : (nm1 - grp % nm1) % nm1;
        for (int step = 0; step < nm1; ++step) {
            if (active) {
                double* wp = W + (size_t)p * ld;
                double* wq = W + (size_t)q * ld;
                double a[NE], b[NE];
                double g0 = 0.0, g1 = 0.0;
#pragma unroll
                for (int e = 0; e < NE; ++e) {
                    int i = gl + JG * e;
                    a[e] = i < n ? wp[i] : 0.0;
                    b[e] = i < n ? wq[i] : 0.0;
                    if (e & 1) g1 += a[e] * b[e]; else g0 += a[e] * b[e];
                }
                const double alpha = nrm[p], beta = nrm[q];
                const double gamma = group8_sum(g0 + g1);
                if (gamma * gamma > tol2 * alpha * beta + floor2 * amax * (alpha + beta) && alpha > 0.0 && beta > 0.0) {
                    // t = tan(theta) of the rotation that orthogonalises the pair (smaller root)
                    const double tau = beta - alpha;
                    const double hh = tau * tau + 4.0 * gamma * gamma;
                    const double hyp = hh * rsqrt_nr(hh);
                    const double t = (tau < 0.0 ? -2.0 : 2.0) * gamma * rcp_nr(fabs(tau) + hyp);
                    const double c = rsqrt_nr(1.0 + t * t), s = c * t;
#pragma unroll
                    for (int e = 0; e < NE; ++e) {
                        int i = gl + JG * e;
                        if (i < n) {
                            wp[i] = c * a[e] - s * b[e];
                            wq[i] = s * a[e] + c * b[e];
                        }
                    }
                    if (gl == 0) {
                        nrm[p] = alpha - t * gamma;
                        nrm[q] = beta + t * gamma;
                        rotated = 1;
                    }
                }
                if (grp == 0) {
                    q = q + 1;
                } else {
                    p = p + 1 == nm1 ? 0 : p + 1;
                    q = q + 1 == nm1 ? 0 : q + 1;
                }
            }
            __syncthreads();
        }
        int any = rotated;
        __syncthreads();
        if (!any) break;
    }
    // column norms = eigenvalues
    if (active) {
        for (int h = 0; h < 2; ++h) {
            int pp = 2 * grp + h;
            double s = 0.0;
            for (int i = gl; i < n; i += JG) s += W[(size_t)pp * ld + i] * W[(size_t)pp * ld + i];
            s = group8_sum(s);
            if (gl == 0) nrm[pp] = (pp < n) ? sqrt(s) : -1.0;
        }
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
    int ne = n + (n & 1);
    size_t lds = ((size_t)ne * jacobi_ld(n) + ne) * sizeof(double) + (size_t)ne * sizeof(int);
const int npairs = ne / 2;
    const int threads = 64 * ((npairs + 7) / 8);          // one 8-lane group per column pair
    if (threads > 512 || ne > threads) return METIS_UNSUPPORTED;
#define JACOBI_CASE(NE)                                                                                       \
    {                                                                                                         \
        if (hipFuncSetAttribute((const void*)k_jacobi_eig<NE>, hipFuncAttributeMaxDynamicSharedMemorySize,    \
                                (int)lds) != hipSuccess)                                                      \
            return METIS_HIP_ERROR;                                                                           \
        hipLaunchKernelGGL(k_jacobi_eig<NE>, dim3(1), dim3(threads), lds, s, G, n, kk, lam, vec, tmat, sval); \
    }
    const int need = (n + 7) / 8;
    if (need <= 1) JACOBI_CASE(1)
    else if (need <= 2) JACOBI_CASE(2)
    else if (need <= 4) JACOBI_CASE(4)
    else if (need <= 8) JACOBI_CASE(8)
    else if (need <= 10) JACOBI_CASE(10)
    else if (need <= 12) JACOBI_CASE(12)
    else if (need <= 16) JACOBI_CASE(16)
    else return METIS_UNSUPPORTED;
#undef JACOBI_CASE
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
