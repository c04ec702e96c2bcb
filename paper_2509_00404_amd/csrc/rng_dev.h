// Draws of the decomposition (Sec. 3.1), one element per call, shared by the stand-alone kernels and the
// decomposition's set-up kernel.
#pragma once
#include "common.h"

// Row j of the sample: uniform in stratum [floor(j M / Ms), floor((j+1) M / Ms)), offset = word j of stream 1.
__device__ __forceinline__ uint32_t sample_row(uint64_t seed, int64_t M, int64_t Ms, int64_t j) {
    u32x4 b = philox_block(seed, 1u, (uint64_t)j >> 2);
    uint32_t u = (j & 3) == 0 ? b.x : (j & 3) == 1 ? b.y : (j & 3) == 2 ? b.z : b.w;
    // 128-bit-safe floor(j*M/Ms): j, M < 2^32 in every supported shape
    uint64_t lo = ((uint64_t)j * (uint64_t)M) / (uint64_t)Ms;
    uint64_t hi = ((uint64_t)(j + 1) * (uint64_t)M) / (uint64_t)Ms;
    return (uint32_t)(lo + u % (uint32_t)(hi - lo));
}

// Row j of a sample of whole sequences of `group` consecutive rows: sequence j / group of the sample is drawn like
// a row above among the M / group sequences, and contributes its rows in order.  group = 1 is sample_row.
__device__ __forceinline__ uint32_t sample_row_grouped(uint64_t seed, int64_t M, int64_t Ms, int64_t group, int64_t j) {
    if (group <= 1) return sample_row(seed, M, Ms, j);
    const int64_t jg = j / group;
    return sample_row(seed, M / group, Ms / group, jg) * (uint32_t)group + (uint32_t)(j - jg * group);
}

// Entries 2 b and 2 b + 1 of Omega (one Philox block of stream 2 = 4 words = 2 Box-Muller entries).
__device__ __forceinline__ void gaussian_pair(uint64_t seed, int64_t b, int64_t count, bf16_t* __restrict__ omega) {
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
