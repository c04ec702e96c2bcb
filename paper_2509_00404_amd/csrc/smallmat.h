// One-workgroup fp64 factorizations (see smallmat.hip).  Every launch takes a batch: one workgroup per problem,
// all problems of a launch of the same order, their pointers travelling by value in the kernel arguments.
#pragma once
#include "common.h"
#define SM_MAX_N 128          // Jacobi: largest matrix order
#define SM_MAX_CHOL 96        // Cholesky + inverse: two n x (n+1) fp64 arrays must fit in 160 KB of LDS
#define SM_MAX_BATCH 32       // problems per launch (longer batches are cut into several launches)

struct CholProblem {
    const double* G;          // n x n Gram matrix
    double* Linv;             // n x n inverse of its Cholesky factor
    int32_t* info;            // optional: index + 1 of a pivot that was not positive
    int32_t* wellcond_out;    // optional: set to 1 when the factor's diagonal spans less than 1e3 (the QR pass that
                              // used it is then orthonormal to ~1e-10)
    const int32_t* skip_in;   // optional: nonzero -> Linv = identity without factoring
};
struct CholBatch { CholProblem p[SM_MAX_BATCH]; };

struct JacobiProblem {
    const double* G;          // n x n symmetric positive semi-definite
    double* lam;              // n eigenvalues, descending
    double* vec;              // optional n x kk eigenvectors
    double* tmat;             // optional n x kk eigenvectors scaled by 1 / sqrt(lambda)
    float* sval;              // optional kk square roots of the eigenvalues
    double* gscr;             // optional jacobi_scratch_doubles(n) doubles of device scratch; when given (and the order
                              // allows it) the sweeps start from columns preconditioned with approximate eigenvectors
};
struct JacobiBatch { JacobiProblem p[SM_MAX_BATCH]; };

int launch_chol_inv_batch(hipStream_t s, const CholProblem* probs, int count, int n);
int launch_jacobi_eig_batch(hipStream_t s, const JacobiProblem* probs, int count, int n, int kk);
size_t jacobi_scratch_doubles(int n);

static inline int launch_chol_inv(hipStream_t s, const double* G, int n, double* Linv, int32_t* info,
                                  int32_t* wellcond_out = nullptr, const int32_t* skip_in = nullptr) {
    const CholProblem p = {G, Linv, info, wellcond_out, skip_in};
    return launch_chol_inv_batch(s, &p, 1, n);
}
static inline int launch_jacobi_eig(hipStream_t s, const double* G, int n, int kk, double* lam, double* vec, double* tmat,
                                    float* sval, double* gscr = nullptr) {
    const JacobiProblem p = {G, lam, vec, tmat, sval, gscr};
    return launch_jacobi_eig_batch(s, &p, 1, n, kk);
}
