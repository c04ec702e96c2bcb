// One-workgroup fp64 factorizations of the small (k+p)x(k+p) matrices of the decomposition
// (Sec. 3.1): Cholesky + triangular inverse for CholeskyQR2 (thin QR Z = H R), and a
// one-sided Jacobi eigensolver for the Gram matrices of the reduced problem.
#include "smallmat.h"

// ---------------------------------------------------------------------------------------
// Cholesky G = L L^T and Linv = L^-1 (lower triangular), n <= SM_MAX_N.
// LDS: L [n][n+1] doubles, X [n][n+1] doubles.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_chol_inv(const double* __restrict__ G, int n, double* __restrict__ Linv, int32_t* __restrict__ info) {
    extern __shared__ double sm[];
    const int ld = n + 1;
    double* L = sm;
    double* X = sm + (size_t)n * ld;
    const int tid = threadIdx.x;
    for (int e = tid; e < n * n; e += 256) {
        int i = e / n, j = e - i * n;
        L[i * ld + j] = G[e];
        X[i * ld + j] = 0.0;
    }
    __syncthreads();
    for (int j = 0; j < n; ++j) {
        if (tid == 0) {
            double d = L[j * ld + j];
            if (!(d > 0.0)) {               // rank-deficient sketch: flag it, keep going finitely
                if (info) *info = j + 1;
                d = 1e-300;
            }
            L[j * ld + j] = sqrt(d);
        }
        __syncthreads();
        double djj = L[j * ld + j];
        for (int i = j + 1 + tid; i < n; i += 256) L[i * ld + j] /= djj;
        __syncthreads();
        const int ti = tid >> 4, tc = tid & 15;
        for (int i = j + 1 + ti; i < n; i += 16) {
            double lij = L[i * ld + j];
            for (int c = j + 1 + tc; c <= i; c += 16) L[i * ld + c] -= lij * L[c * ld + j];
        }
        __syncthreads();
    }
    // forward substitution, one column of L^-1 per thread; X[t][c] keeps lanes conflict-free
    if (tid < n) {
        const int c = tid;
        for (int i = 0; i < n; ++i) {
            double s = (i == c) ? 1.0 : 0.0;
            for (int t = 0; t < i; ++t) s -= L[i * ld + t] * X[t * ld + c];
            X[i * ld + c] = (i < c) ? 0.0 : s / L[i * ld + i];
        }
    }
    __syncthreads();
    for (int e = tid; e < n * n; e += 256) {
        int i = e / n, j = e - i * n;
        Linv[e] = X[i * ld + j];
    }
}

// ---------------------------------------------------------------------------------------
// One-sided Jacobi on a symmetric positive semi-definite G (n <= SM_MAX_N):
// rotate the columns of W = G until they are mutually orthogonal; then column j is
// lambda_j v_j.  1024 threads = 64 groups of 16 lanes, one column pair per group and
// step, round-robin ordering; dot products by 16-lane shuffles.
// Outputs (eigenvalues descending):
//   lam  [n]            eigenvalues
//   vec  [n][n]         vec[i*n + j] = component i of eigenvector j          (optional)
//   tmat [n][kk]        tmat[i*kk + c] = vec[i][c] / sqrt(lam_c), c < kk     (optional)
//   sval [kk]           (float) sqrt(lam_c)                                  (optional)
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double group16_sum(double x) {
    x += __shfl_xor(x, 8, 16);
    x += __shfl_xor(x, 4, 16);
    x += __shfl_xor(x, 2, 16);
    x += __shfl_xor(x, 1, 16);
    return x;
}

__global__ void __launch_bounds__(1024)
k_jacobi_eig(const double* __restrict__ G, int n, int kk, double* __restrict__ lam, double* __restrict__ vec,
             double* __restrict__ tmat, float* __restrict__ sval) {
    extern __shared__ double sm[];
    const int ne = n + (n & 1);             // even number of columns (a zero column pads odd n)
    const int ld = n + 1;
    double* W = sm;                         // column-major: W[p*ld + i] = element i of column p
    double* nrm = sm + (size_t)ne * ld;     // [ne]
    int* order = (int*)(nrm + ne);          // [ne]
    __shared__ int rotated;
    const int tid = threadIdx.x, grp = tid >> 4, gl = tid & 15;

    for (int e = tid; e < ne * ld; e += 1024) {
        int p = e / ld, i = e - p * ld;
        W[e] = (p < n && i < n) ? G[(size_t)i * n + p] : 0.0;
    }
    __syncthreads();

    const int npairs = ne / 2, nm1 = ne - 1;
    const double tol = 1e-15;
    for (int sweep = 0; sweep < 40; ++sweep) {
        if (tid == 0) rotated = 0;
        __syncthreads();
        for (int step = 0; step < nm1; ++step) {
            if (grp < npairs) {
                int p, q;
                if (grp == 0) { p = nm1; q = step; }
                else { p = (step + grp) % nm1; q = (step - grp + nm1) % nm1; }
                double* wp = W + (size_t)p * ld;
                double* wq = W + (size_t)q * ld;
                double a[SM_MAX_N / 16], b[SM_MAX_N / 16];
                double alpha = 0.0, beta = 0.0, gamma = 0.0;
#pragma unroll
                for (int e = 0; e < SM_MAX_N / 16; ++e) {
                    int i = gl + 16 * e;
                    a[e] = i < n ? wp[i] : 0.0;
                    b[e] = i < n ? wq[i] : 0.0;
                    alpha += a[e] * a[e];
                    beta += b[e] * b[e];
                    gamma += a[e] * b[e];
                }
                alpha = group16_sum(alpha);
                beta = group16_sum(beta);
                gamma = group16_sum(gamma);
                if (fabs(gamma) > tol * sqrt(alpha * beta) && alpha > 0.0 && beta > 0.0) {
                    double zeta = (beta - alpha) / (2.0 * gamma);
                    double t = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
#pragma unroll
                    for (int e = 0; e < SM_MAX_N / 16; ++e) {
                        int i = gl + 16 * e;
                        if (i < n) {
                            wp[i] = c * a[e] - s * b[e];
                            wq[i] = s * a[e] + c * b[e];
                        }
                    }
                    if (gl == 0) rotated = 1;
                }
            }
            __syncthreads();
        }
        int any = rotated;
        __syncthreads();
        if (!any) break;
    }
    // column norms = eigenvalues
    if (grp < npairs) {
        for (int h = 0; h < 2; ++h) {
            int p = 2 * grp + h;
            double s = 0.0;
            for (int i = gl; i < n; i += 16) s += W[(size_t)p * ld + i] * W[(size_t)p * ld + i];
            s = group16_sum(s);
            if (gl == 0) nrm[p] = (p < n) ? sqrt(s) : -1.0;
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
    for (int e = tid; e < n * n; e += 1024) {
        int i = e / n, j = e - i * n;
        int p = order[j];
        double l = nrm[p];
        double v = l > 0.0 ? W[(size_t)p * ld + i] / l : (i == j ? 1.0 : 0.0);
        if (vec) vec[e] = v;
        if (tmat && j < kk) tmat[(size_t)i * kk + j] = l > 0.0 ? v / sqrt(l) : 0.0;
    }
    if (tid < n) {
        double l = nrm[order[tid]];
        lam[tid] = l;
        if (sval && tid < kk) sval[tid] = (float)sqrt(l);
    }
}

int launch_chol_inv(hipStream_t s, const double* G, int n, double* Linv, int32_t* info) {
    size_t lds = 2 * (size_t)n * (n + 1) * sizeof(double);
    if (hipFuncSetAttribute((const void*)k_chol_inv, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return METIS_HIP_ERROR;
    hipLaunchKernelGGL(k_chol_inv, dim3(1), dim3(256), lds, s, G, n, Linv, info);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

int launch_jacobi_eig(hipStream_t s, const double* G, int n, int kk, double* lam, double* vec, double* tmat,
                      float* sval) {
    int ne = n + (n & 1);
    size_t lds = ((size_t)ne * (n + 1) + ne) * sizeof(double) + (size_t)ne * sizeof(int);
    if (hipFuncSetAttribute((const void*)k_jacobi_eig, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return METIS_HIP_ERROR;
    hipLaunchKernelGGL(k_jacobi_eig, dim3(1), dim3(1024), lds, s, G, n, kk, lam, vec, tmat, sval);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
