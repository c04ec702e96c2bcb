// One-workgroup fp64 factorizations (see smallmat.hip).
#pragma once
#include "common.h"
#define SM_MAX_N 128          // Jacobi: largest matrix order
#define SM_MAX_CHOL 96        // Cholesky + inverse: two n x (n+1) fp64 arrays must fit in 160 KB of LDS
// wellcond_out (optional): set to 1 when the factor's diagonal spans less than 1e3 (the QR pass that used it is
// then orthonormal to ~1e-10); skip_in (optional): nonzero -> Linv = identity without factoring
int launch_chol_inv(hipStream_t s, const double* G, int n, double* Linv, int32_t* info, int32_t* wellcond_out = nullptr,
                    const int32_t* skip_in = nullptr);
// gscr (optional): jacobi_scratch_doubles(n) doubles of device scratch; when given (and the order allows it) the
// sweeps start from columns preconditioned with approximate eigenvectors
int launch_jacobi_eig(hipStream_t s, const double* G, int n, int kk, double* lam, double* vec, double* tmat,
                      float* sval, double* gscr = nullptr);
size_t jacobi_scratch_doubles(int n);
