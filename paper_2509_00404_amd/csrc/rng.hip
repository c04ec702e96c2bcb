// Random draws of the scalable decomposition (Sec. 3.1): stratified row sample and the
// Gaussian test matrix, both from Philox4x32-10.
#include "common.h"

__global__ void k_sample_rows(uint64_t seed, int64_t M, int64_t Ms, uint32_t* __restrict__ idx) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= Ms) return;
    u32x4 b = philox_block(seed, 1u, (uint64_t)j >> 2);
    uint32_t u = (j & 3) == 0 ? b.x : (j & 3) == 1 ? b.y : (j & 3) == 2 ? b.z : b.w;
    // 128-bit-safe floor(j*M/Ms): j, M < 2^32 in every supported shape
    uint64_t lo = ((uint64_t)j * (uint64_t)M) / (uint64_t)Ms;
    uint64_t hi = ((uint64_t)(j + 1) * (uint64_t)M) / (uint64_t)Ms;
    idx[j] = (uint32_t)(lo + u % (uint32_t)(hi - lo));
}

// One thread per pair of entries (one Philox block = 4 words = 2 entries).
__global__ void k_gaussian_omega(uint64_t seed, int64_t count, bf16_t* __restrict__ omega) {
    int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t e0 = b * 2;
    if (e0 >= count) return;
    u32x4 w = philox_block(seed, 2u, (uint64_t)b);
    const float two_pi = 6.283185307179586f;
    {
        float u1 = ((float)(w.x >> 9) + 0.5f) * 1.1920928955078125e-07f;   // 2^-23
        float u2 = (float)(w.y >> 8) * 5.9604644775390625e-08f;            // 2^-24
        float z = sqrtf(-2.0f * logf(u1)) * cosf(two_pi * u2);
        omega[e0] = f32_to_bf16_rne(z);
    }
    if (e0 + 1 < count) {
        float u1 = ((float)(w.z >> 9) + 0.5f) * 1.1920928955078125e-07f;
        float u2 = (float)(w.w >> 8) * 5.9604644775390625e-08f;
        float z = sqrtf(-2.0f * logf(u1)) * cosf(two_pi * u2);
        omega[e0 + 1] = f32_to_bf16_rne(z);
    }
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

extern "C" int metis_sample_rows(void* stream, uint64_t seed, int64_t M, int64_t Ms, uint32_t* idx) {
    if (!idx || M < 1 || Ms < 1) return METIS_INVALID_ARG;
    if (Ms > M || M >= ((int64_t)1 << 32)) return METIS_BAD_SHAPE;
    int blocks = (int)ceil_div64(Ms, 256);
    hipLaunchKernelGGL(k_sample_rows, dim3(blocks), dim3(256), 0, (hipStream_t)stream, seed, M, Ms, idx);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

extern "C" int metis_gaussian_omega(void* stream, uint64_t seed, int64_t N, int r, uint16_t* omega) {
    if (!omega || N < 1 || r < 1) return METIS_INVALID_ARG;
    int64_t count = N * (int64_t)r;
    int blocks = (int)ceil_div64(ceil_div64(count, 2), 256);
    hipLaunchKernelGGL(k_gaussian_omega, dim3(blocks), dim3(256), 0, (hipStream_t)stream, seed, count, omega);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
