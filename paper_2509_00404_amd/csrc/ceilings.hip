// Measurement aids: what this GPU sustains for a plain streaming read, a plain copy, and a register-resident
// fp16 matrix-instruction loop, so that roofline fractions can be quoted against measured ceilings as well
// as against the datasheet peaks.  Not part of the hot path.
#include "common.h"

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// grid-stride copy in 16-byte pieces, four in flight per lane
__global__ void __launch_bounds__(256) k_ceiling_copy(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4_t a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

// grid-stride read; the xor of everything read goes to one word per workgroup so the loads cannot be dropped
__global__ void __launch_bounds__(256) k_ceiling_read(const u32x4_t* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4_t a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride) acc ^= src[i];
    const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9E3779B9u) sink[blockIdx.x] = x;            // practically never taken; keeps the loads alive
}

// every wave issues `iters` rounds of eight independent 32x32x16 fp16 matrix instructions on registers
__global__ void __launch_bounds__(256) k_ceiling_mfma(int iters, float* __restrict__ sink) {
    half8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(0.001f * (float)(threadIdx.x & 7) + (float)i); b[i] = (_Float16)(0.5f * (float)i); }
    float16_t c[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) c[t][i] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) c[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c[t], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += c[t][i];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// The FP4 GEMM's instruction mix without its memory system: every wave issues `iters` rounds of four independent
// 32x32x16 fp16 matrix instructions (accumulators in the accumulation registers), each followed by NV independent
// packed fp16 multiplies on registers -- the expansion work of the GEMM is NV ~ 4.5 per matrix instruction.
template <int NV>
__global__ void __launch_bounds__(256) k_ceiling_mfma_mix(int iters, float* __restrict__ sink) {
    half8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(0.001f * (float)(threadIdx.x & 7) + (float)i); b[i] = (_Float16)(0.5f * (float)i); }
    float16_t c0, c1, c2, c3;
#pragma unroll
    for (int i = 0; i < 16; ++i) { c0[i] = 0.0f; c1[i] = 1.0f; c2[i] = 2.0f; c3[i] = 3.0f; }
    uint32_t r0 = threadIdx.x, r1 = r0 * 3u, r2 = r0 * 5u, r3 = r0 * 7u, r4 = r0 * 11u, r5 = r0 * 13u, r6 = r0 * 17u, r7 = r0 * 19u;
    uint32_t d0 = 0, d1 = 0, d2 = 0, d3 = 0, d4 = 0, d5 = 0, d6 = 0, d7 = 0;
#define MIX_MFMA(C) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(C) : "v"(a), "v"(b));
#define MIX_MUL(D, S) asm volatile("v_pk_mul_f16 %0, %1, %1" : "=v"(D) : "v"(S));
    for (int it = 0; it < iters; ++it) {
        MIX_MFMA(c0)
        if (NV >= 1) MIX_MUL(d0, r0)
        if (NV >= 2) MIX_MUL(d1, r1)
        if (NV >= 3) MIX_MUL(d2, r2)
        if (NV >= 4) MIX_MUL(d3, r3)
        if (NV >= 5) MIX_MUL(d4, r4)
        if (NV >= 6) MIX_MUL(d5, r5)
        if (NV >= 7) MIX_MUL(d6, r6)
        if (NV >= 8) MIX_MUL(d7, r7)
        MIX_MFMA(c1)
        if (NV >= 1) MIX_MUL(d0, r1)
        if (NV >= 2) MIX_MUL(d1, r2)
        if (NV >= 3) MIX_MUL(d2, r3)
        if (NV >= 4) MIX_MUL(d3, r4)
        if (NV >= 5) MIX_MUL(d4, r5)
        if (NV >= 6) MIX_MUL(d5, r6)
        if (NV >= 7) MIX_MUL(d6, r7)
        if (NV >= 8) MIX_MUL(d7, r0)
        MIX_MFMA(c2)
        if (NV >= 1) MIX_MUL(d0, r2)
        if (NV >= 2) MIX_MUL(d1, r3)
        if (NV >= 3) MIX_MUL(d2, r4)
        if (NV >= 4) MIX_MUL(d3, r5)
        if (NV >= 5) MIX_MUL(d4, r6)
        if (NV >= 6) MIX_MUL(d5, r7)
        if (NV >= 7) MIX_MUL(d6, r0)
        if (NV >= 8) MIX_MUL(d7, r1)
        MIX_MFMA(c3)
        if (NV >= 1) MIX_MUL(d0, r3)
        if (NV >= 2) MIX_MUL(d1, r4)
        if (NV >= 3) MIX_MUL(d2, r5)
        if (NV >= 4) MIX_MUL(d3, r6)
        if (NV >= 5) MIX_MUL(d4, r7)
        if (NV >= 6) MIX_MUL(d5, r0)
        if (NV >= 7) MIX_MUL(d6, r1)
        if (NV >= 8) MIX_MUL(d7, r2)
    }
#undef MIX_MFMA
#undef MIX_MUL
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == 12345.678f || (d0 ^ d1 ^ d2 ^ d3 ^ d4 ^ d5 ^ d6 ^ d7) == 0x9E3779B9u) sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// The FP4 GEMM's stage loop with its memory system taken away: per step a wave expands eight fragments from raw
// words that sit in registers (four FP4 -> fp16 conversions and four packed multiplies by the block scale each, the
// GEMM's own expansion) and issues the 16 matrix instructions of a 128 x 128 wave tile on them; the compiler orders
// the step.  What is missing against the GEMM: LDS reads and writes, global loads, waits and the barrier.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ half8_t expand8(uint32_t cw, uint32_t spair, bool hi) {
    const half2_t sp = __builtin_bit_cast(half2_t, spair);
    const half2_t s2 = hi ? (half2_t){sp[1], sp[1]} : (half2_t){sp[0], sp[0]};
    const half2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 0) * s2;
    const half2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 1) * s2;
    const half2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 2) * s2;
    const half2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 3) * s2;
    return (half8_t){p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}
// FP6 = the same step with the codes held in 6-bit containers and expanded by the 32-wide converter
// (v_cvt_scalef32_pk32_f16_fp6: one instruction for the four fragments of an operand) instead of 32 two-wide FP4
// conversions; the packed multiplies by the block scales stay.
typedef _Float16 half32_t __attribute__((ext_vector_type(32)));
typedef uint32_t u32x6_t __attribute__((ext_vector_type(6)));
template <bool FP6>
__global__ void __launch_bounds__(256) k_ceiling_mfma_expand(int iters, float* __restrict__ sink) {
    float16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    uint32_t raw[8], sc[8];
    u32x6_t r6[2];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        raw[t] = 0x9E3779B9u * (threadIdx.x + 1u) * (uint32_t)(t + 3);
        sc[t] = 0x3C003800u;                                  // fp16 scales 0.5 and 1.0
    }
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int e = 0; e < 6; ++e) r6[g][e] = (0x9E3779B9u * (threadIdx.x + 7u) * (uint32_t)(e + 6 * g + 1)) & 0x3CF3CF3Cu;   // E2M1 values in E2M3 fields
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {                          // the two blocks of a scale pair
            half8_t f[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) asm volatile("" : "+v"(raw[t]), "+v"(sc[t]));  // new raw words every step, as if read from LDS
            if (FP6) {
                asm volatile("" : "+v"(r6[0]), "+v"(r6[1]));
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const half32_t c = __builtin_amdgcn_cvt_scalef32_pk32_f16_fp6(r6[g], 1.0f);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const half2_t sp = __builtin_bit_cast(half2_t, sc[4 * g + t]);
                        const half2_t s2 = h ? (half2_t){sp[1], sp[1]} : (half2_t){sp[0], sp[0]};
                        const half2_t p0 = (half2_t){c[8 * t], c[8 * t + 1]} * s2, p1 = (half2_t){c[8 * t + 2], c[8 * t + 3]} * s2;
                        const half2_t p2 = (half2_t){c[8 * t + 4], c[8 * t + 5]} * s2, p3 = (half2_t){c[8 * t + 6], c[8 * t + 7]} * s2;
                        f[4 * g + t] = (half8_t){p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
                    }
                }
            } else {
#pragma unroll
                for (int t = 0; t < 8; ++t) f[t] = expand8(raw[t], sc[t], h);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[i], f[4 + j], acc[i][j], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" int metis_ceiling_mfma_mix(void* stream, int iters, int valu_per_mfma, int waves_per_simd, float* sink,
                                      double* flops_out) {
    if (iters < 1 || !sink || waves_per_simd < 1 || waves_per_simd > 2) return METIS_INVALID_ARG;
    const int cus = device_cu_count();
    if (cus < 1) return METIS_HIP_ERROR;
    if (cus * waves_per_simd > 512) return METIS_UNSUPPORTED;          // the sink holds 512 workgroups
    const dim3 grid((unsigned)(cus * waves_per_simd));                 // workgroups of four waves, one wave per SIMD each
    hipStream_t s = (hipStream_t)stream;
    if (valu_per_mfma == METIS_MIX_GEMM_EXPANSION || valu_per_mfma == METIS_MIX_GEMM_EXPANSION_FP6) {
        if (waves_per_simd != 1) return METIS_INVALID_ARG;            // 16 accumulator tiles: one wave per SIMD
        const int steps = (iters + 1) / 2 * 2;
        if (valu_per_mfma == METIS_MIX_GEMM_EXPANSION)
            hipLaunchKernelGGL(k_ceiling_mfma_expand<false>, grid, dim3(256), 0, s, steps, sink);
        else
            hipLaunchKernelGGL(k_ceiling_mfma_expand<true>, grid, dim3(256), 0, s, steps, sink);
        METIS_LAUNCH_CHECK();
        if (flops_out) *flops_out = (double)grid.x * 4.0 * (double)steps * 16.0 * 2.0 * 32.0 * 32.0 * 16.0;
        return METIS_OK;
    }
    switch (valu_per_mfma) {
        case 0: hipLaunchKernelGGL(k_ceiling_mfma_mix<0>, grid, dim3(256), 0, s, iters, sink); break;
        case 2: hipLaunchKernelGGL(k_ceiling_mfma_mix<2>, grid, dim3(256), 0, s, iters, sink); break;
        case 4: hipLaunchKernelGGL(k_ceiling_mfma_mix<4>, grid, dim3(256), 0, s, iters, sink); break;
        case 5: hipLaunchKernelGGL(k_ceiling_mfma_mix<5>, grid, dim3(256), 0, s, iters, sink); break;
        case 6: hipLaunchKernelGGL(k_ceiling_mfma_mix<6>, grid, dim3(256), 0, s, iters, sink); break;
        case 8: hipLaunchKernelGGL(k_ceiling_mfma_mix<8>, grid, dim3(256), 0, s, iters, sink); break;
        default: return METIS_INVALID_ARG;
    }
    METIS_LAUNCH_CHECK();
    if (flops_out) *flops_out = (double)grid.x * 4.0 * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return METIS_OK;
}

extern "C" int metis_ceiling_copy(void* stream, const void* src, void* dst, size_t bytes) {
    if (!src || !dst || bytes < 16 || bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16 ||
        reinterpret_cast<uintptr_t>(dst) % 16)
        return METIS_INVALID_ARG;
    hipLaunchKernelGGL(k_ceiling_copy, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream, (const u32x4_t*)src,
                       (u32x4_t*)dst, bytes / 16);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

extern "C" int metis_ceiling_read(void* stream, const void* src, size_t bytes, uint32_t* sink) {
    if (!src || !sink || bytes < 16 || bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16) return METIS_INVALID_ARG;
    hipLaunchKernelGGL(k_ceiling_read, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream, (const u32x4_t*)src, bytes / 16,
                       sink);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

extern "C" int metis_ceiling_mfma(void* stream, int iters, float* sink, double* flops_out) {
    if (iters < 1 || !sink) return METIS_INVALID_ARG;
    const int blocks = 256 * 2;                           // two workgroups of four waves per CU: two waves per SIMD
    hipLaunchKernelGGL(k_ceiling_mfma, dim3(blocks), dim3(256), 0, (hipStream_t)stream, iters, sink);
    METIS_LAUNCH_CHECK();
    if (flops_out) *flops_out = (double)blocks * 4.0 * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return METIS_OK;
}
