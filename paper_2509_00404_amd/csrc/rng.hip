// Random draws of the scalable decomposition (Sec. 3.1): stratified row sample and the
// Gaussian test matrix, both from Philox4x32-10.
#include "common.h"
#include "rng_dev.h"

__global__ void k_sample_rows(uint64_t seed, int64_t M, int64_t Ms, int64_t group, uint32_t* __restrict__ idx) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= Ms) return;
    idx[j] = sample_row_grouped(seed, M, Ms, group, j);
}

// One thread per pair of entries (one Philox block = 4 words = 2 entries).
__global__ void k_gaussian_omega(uint64_t seed, int64_t count, bf16_t* __restrict__ omega) {
    gaussian_pair(seed, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, count, omega);
}

extern "C" int64_t metis_sample_count(int64_t M, int k, int p, double rho) {
    if (M < 1 || k < 0 || p < 0 || !(rho > 0.0) || rho > 1.0) return 0;
    double want = rho * (double)M - 1e-12;
    int64_t c = (int64_t)want;
    if ((double)c < want) ++c;
    int64_t r = (int64_t)k + p;
    if (c < r) c = r;
    if (c > M) c = M;
    return c;
}

extern "C" int64_t metis_sample_count_sequences(int64_t M, int k, int p, double rho, int64_t group) {
    if (group <= 1) return metis_sample_count(M, k, p, rho);
    if (M < 1 || k < 0 || p < 0 || !(rho > 0.0) || rho > 1.0 || M % group) return 0;
    const int64_t G = M / group;
    double want = rho * (double)G - 1e-12;
    int64_t c = (int64_t)want;
    if ((double)c < want) ++c;
    const int64_t need = ((int64_t)k + p + group - 1) / group;
    if (c < need) c = need;
    if (c > G) c = G;
    return c * group;
}

extern "C" int metis_sample_sequences(void* stream, uint64_t seed, int64_t M, int64_t Ms, int64_t group, uint32_t* idx) {
    if (!idx || M < 1 || Ms < 1 || group < 1) return METIS_INVALID_ARG;
    if (Ms > M || M >= ((int64_t)1 << 32) || M % group || Ms % group) return METIS_BAD_SHAPE;
    int blocks = (int)ceil_div64(Ms, 256);
    hipLaunchKernelGGL(k_sample_rows, dim3(blocks), dim3(256), 0, (hipStream_t)stream, seed, M, Ms, group, idx);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

extern "C" int metis_sample_rows(void* stream, uint64_t seed, int64_t M, int64_t Ms, uint32_t* idx) {
    return metis_sample_sequences(stream, seed, M, Ms, 1, idx);
}

extern "C" int metis_gaussian_omega(void* stream, uint64_t seed, int64_t N, int r, uint16_t* omega) {
    if (!omega || N < 1 || r < 1) return METIS_INVALID_ARG;
    int64_t count = N * (int64_t)r;
    int blocks = (int)ceil_div64(ceil_div64(count, 2), 256);
    hipLaunchKernelGGL(k_gaussian_omega, dim3(blocks), dim3(256), 0, (hipStream_t)stream, seed, count, omega);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
