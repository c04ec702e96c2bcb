// Plain NVFP4 quantization of a dense matrix (Sec. 2.3), row orientation and/or transposed.
#include "quant_dev.h"
#include "splitq.h"

// ---- row orientation, bf16 input: one lane per block of 16, 32 contiguous bytes per lane ----
#define SR_STREAM 3u          // Philox stream of the stochastic-rounding draws, row orientation
#define SR_STREAM_T 4u        // ... of the transposed copy

// RHT: the block is first rotated, z = (x * d) H_16 / 4 (16-point Sylvester Hadamard matrix, random signs d: bit i of
// `signs` set = d_i = -1), by the radix-2 butterfly in natural order in fp32 -- the comparison recipe of Sec. 4.3
// (random Hadamard transform + stochastic rounding).
template <bool SR, bool RHT>
__global__ void __launch_bounds__(256)
k_quantize_rows_bf16(const bf16_t* __restrict__ A, int64_t ld, int64_t M, int64_t nblk /* N/16 */,
                     QuantParams qp, uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, uint64_t seed,
                     uint32_t signs) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= M * nblk) return;
    int64_t row = t / nblk, bc = t - row * nblk;
    const uint4* src = reinterpret_cast<const uint4*>(A + row * ld + bc * 16);
    uint4 a = src[0], b = src[1];
    uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    float v[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[2 * i] = bf16lo_to_f32(w[i]);
        v[2 * i + 1] = bf16hi_to_f32(w[i]);
    }
    if (RHT) {
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = (signs >> i) & 1u ? -v[i] : v[i];
#pragma unroll
        for (int h = 1; h < 16; h <<= 1)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (!(i & h)) {
                    const float a = v[i], b = v[i + h];
                    v[i] = a + b;
                    v[i + h] = a - b;
                }
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] *= 0.25f;
    }
    uint2 c;
    // block t covers the elements 16 t .. 16 t + 15 of the row-major matrix: their draws are those words
    uint32_t sc = SR ? quantize_block16_sr(v, qp, c, seed, SR_STREAM, (uint64_t)t * 16) : quantize_block16(v, qp, c);
    *reinterpret_cast<uint2*>(codes + t * 8) = c;     // codes are [M, N/2] contiguous: block t at byte 8t
    scales[t] = (uint8_t)sc;
}

// ---- generic tile kernel: 64x64 tile through LDS, either orientation, bf16 or fp32 ----
template <typename T> __device__ __forceinline__ float load_as_f32(const T* p);
template <> __device__ __forceinline__ float load_as_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <> __device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }

template <typename T, bool SR>
__device__ __forceinline__ void
quantize_tile_body(const T* __restrict__ A, int64_t ld, int64_t M, int64_t N, QuantParams qp, QuantParams qpt,
                   uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                   uint8_t* __restrict__ codes_t, uint8_t* __restrict__ scales_t, uint64_t seed, int64_t bx, int64_t by) {
    __shared__ float tile[64][65];
    const int64_t m0 = by * 64, n0 = bx * 64;
    const int tid = threadIdx.x;
    for (int i = tid; i < 64 * 64; i += 256) {
        int r = i >> 6, c = i & 63;
        float v = 0.0f;
        if (m0 + r < M && n0 + c < N) v = load_as_f32<T>(A + (m0 + r) * ld + n0 + c);
        tile[r][c] = v;
    }
    __syncthreads();
    const int line = tid >> 2, blk = tid & 3;      // 64 lines x 4 blocks of 16
    if (codes) {
        int64_t m = m0 + line, n = n0 + blk * 16;
        if (m < M && n < N) {
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = tile[line][blk * 16 + i];
            uint2 c;
            uint32_t sc = SR ? quantize_block16_sr(v, qp, c, seed, SR_STREAM, (uint64_t)(m * N + n))
                             : quantize_block16(v, qp, c);
            *reinterpret_cast<uint2*>(codes + m * (N / 2) + n / 2) = c;
            scales[m * (N / 16) + n / 16] = (uint8_t)sc;
        }
    }
    if (codes_t) {
        int64_t n = n0 + line, m = m0 + blk * 16;
        if (n < N && m < M) {
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = tile[blk * 16 + i][line];
            uint2 c;
            // the transposed copy draws from its own stream, indexed by its own row-major positions
            uint32_t sc = SR ? quantize_block16_sr(v, qpt, c, seed, SR_STREAM_T, (uint64_t)(n * M + m))
                             : quantize_block16(v, qpt, c);
            *reinterpret_cast<uint2*>(codes_t + n * (M / 2) + m / 2) = c;
            scales_t[n * (M / 16) + m / 16] = (uint8_t)sc;
        }
    }
}

template <typename T, bool SR>
__global__ void __launch_bounds__(256)
k_quantize_tile(const T* __restrict__ A, int64_t ld, int64_t M, int64_t N, QuantParams qp, QuantParams qpt,
                uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                uint8_t* __restrict__ codes_t, uint8_t* __restrict__ scales_t, uint64_t seed) {
    quantize_tile_body<T, SR>(A, ld, M, N, qp, qpt, codes, scales, codes_t, scales_t, seed, blockIdx.x, blockIdx.y);
}

// The transposed quantization of the two fp32 factors of a split, U [M, k] -> Q(U^T) [k, M] and V [N, k] -> Q(V^T)
// [k, N], and the copy of S, in one launch (three tiny launches otherwise): blocks [0, tiles of U) take U, the rest V.
template <bool SR>
__global__ void __launch_bounds__(256)
k_quantize_factors_t(const float* __restrict__ U, int64_t M, const float* __restrict__ V, int64_t N, int k, QuantParams qu,
                     QuantParams qv, uint8_t* __restrict__ ut_codes, uint8_t* __restrict__ ut_scales,
                     uint8_t* __restrict__ vt_codes, uint8_t* __restrict__ vt_scales, uint64_t seed_u, uint64_t seed_v,
                     const float* __restrict__ S_src, float* __restrict__ S_dst) {
    const int64_t gx = (k + 63) / 64, tiles_u = gx * ((M + 63) / 64);
    const int64_t b = blockIdx.x;
    if (b == 0 && S_src && (int)threadIdx.x < k) S_dst[threadIdx.x] = S_src[threadIdx.x];
    const bool u = b < tiles_u;
    const int64_t t = u ? b : b - tiles_u;
    quantize_tile_body<float, SR>(u ? U : V, k, u ? M : N, k, u ? qu : qv, u ? qu : qv, nullptr, nullptr, u ? ut_codes : vt_codes,
                                  u ? ut_scales : vt_scales, u ? seed_u : seed_v, t % gx, t / gx);
}

static bool pow2(float g) {
    if (!(g > 0.0f)) return false;
    uint32_t u;
    __builtin_memcpy(&u, &g, 4);
    return (u & 0x7FFFFFu) == 0 && (u >> 23) != 0 && (u >> 23) != 255;
}

template <bool SR>
static int quantize_impl(void* stream, const metis_mat* A, metis_fp4* out, metis_fp4* out_t, uint64_t seed) {
    if (!A || !A->ptr || (!out && !out_t)) return METIS_INVALID_ARG;
    if (A->dtype != METIS_BF16 && A->dtype != METIS_F32) return METIS_INVALID_ARG;
    const int64_t M = A->rows, N = A->cols;
    if (M < 1 || N < 1 || A->ld < N) return METIS_BAD_SHAPE;
    if (out) {
        if (!out->codes || !out->scales || !pow2(out->tscale)) return METIS_INVALID_ARG;
        if (out->rows != M || out->cols != N || N % 16) return METIS_BAD_SHAPE;
    }
    if (out_t) {
        if (!out_t->codes || !out_t->scales || !pow2(out_t->tscale)) return METIS_INVALID_ARG;
        if (out_t->rows != N || out_t->cols != M || M % 16) return METIS_BAD_SHAPE;
    }
    hipStream_t s = (hipStream_t)stream;
    const bool vec_ok = A->dtype == METIS_BF16 && !out_t && (A->ld % 8 == 0) &&
                        (reinterpret_cast<uintptr_t>(A->ptr) % 16 == 0);
    if (vec_ok) {
        int64_t nb = M * (N / 16);
        const int pi = metis_prof_begin(METIS_PROF_QUANTIZE, s);
        hipLaunchKernelGGL((k_quantize_rows_bf16<SR, false>), dim3((unsigned)ceil_div64(nb, 256)), dim3(256), 0, s,
                           (const bf16_t*)A->ptr, A->ld, M, N / 16, make_quant_params(out->tscale),
                           out->codes, out->scales, seed, 0u);
        metis_prof_end(METIS_PROF_QUANTIZE, pi, s);
        METIS_LAUNCH_CHECK();
        return METIS_OK;
    }
    dim3 grid((unsigned)ceil_div64(N, 64), (unsigned)ceil_div64(M, 64));
    QuantParams qp = make_quant_params(out ? out->tscale : 1.0f);
    QuantParams qpt = make_quant_params(out_t ? out_t->tscale : 1.0f);
    uint8_t* c = out ? out->codes : nullptr;
    uint8_t* sc = out ? out->scales : nullptr;
    uint8_t* ct = out_t ? out_t->codes : nullptr;
    uint8_t* sct = out_t ? out_t->scales : nullptr;
    if (A->dtype == METIS_BF16)
        hipLaunchKernelGGL((k_quantize_tile<bf16_t, SR>), grid, dim3(256), 0, s, (const bf16_t*)A->ptr, A->ld, M, N,
                           qp, qpt, c, sc, ct, sct, seed);
    else
        hipLaunchKernelGGL((k_quantize_tile<float, SR>), grid, dim3(256), 0, s, (const float*)A->ptr, A->ld, M, N,
                           qp, qpt, c, sc, ct, sct, seed);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

extern "C" int metis_quantize(void* stream, const metis_mat* A, metis_fp4* out, metis_fp4* out_t) {
    return quantize_impl<false>(stream, A, out, out_t, 0);
}

extern "C" int metis_quantize_sr(void* stream, const metis_mat* A, uint64_t seed, metis_fp4* out, metis_fp4* out_t) {
    return quantize_impl<true>(stream, A, out, out_t, seed);
}

// Random Hadamard rotation + stochastic rounding (the recipe Sec. 4.3 compares with).
extern "C" int metis_quantize_rht_sr(void* stream, const metis_mat* A, uint64_t seed, metis_fp4* out) {
    if (!A || !A->ptr || !out || !out->codes || !out->scales || !pow2(out->tscale)) return METIS_INVALID_ARG;
    if (A->dtype != METIS_BF16) return METIS_UNSUPPORTED;
    const int64_t M = A->rows, N = A->cols;
    if (M < 1 || N < 1 || A->ld < N || N % 16 || out->rows != M || out->cols != N) return METIS_BAD_SHAPE;
    if (A->ld % 8 || reinterpret_cast<uintptr_t>(A->ptr) % 16) return METIS_BAD_SHAPE;      // 16-byte loads
    // the 16 signs: top bits of words 0..15 of Philox stream 5 (host side of the same generator)
    uint32_t signs = 0;
    for (int b = 0; b < 4; ++b) {
        const u32x4 w = philox_block(seed, 5u, (uint64_t)b);
        signs |= (w.x >> 31) << (4 * b) | (w.y >> 31) << (4 * b + 1) | (w.z >> 31) << (4 * b + 2) | (w.w >> 31) << (4 * b + 3);
    }
    hipStream_t s = (hipStream_t)stream;
    const int64_t nb = M * (N / 16);
    const int pi = metis_prof_begin(METIS_PROF_QUANTIZE, s);
    hipLaunchKernelGGL((k_quantize_rows_bf16<true, true>), dim3((unsigned)ceil_div64(nb, 256)), dim3(256), 0, s,
                       (const bf16_t*)A->ptr, A->ld, M, N / 16, make_quant_params(out->tscale), out->codes, out->scales,
                       seed, signs);
    metis_prof_end(METIS_PROF_QUANTIZE, pi, s);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

// Q(U^T), Q(V^T) and S of a split in one launch (see k_quantize_factors_t); M % 16 == 0, N % 16 == 0, S_src null for no copy
int launch_quantize_factors_t(hipStream_t s, const float* U, int64_t M, const float* V, int64_t N, int k, const metis_fp4& Ut,
                              const metis_fp4& Vt, bool sr, uint64_t seed_u, uint64_t seed_v, const float* S_src, float* S_dst) {
    if (!pow2(Ut.tscale) || !pow2(Vt.tscale) || k < 1 || k > 256) return METIS_INVALID_ARG;
    const int64_t gx = (k + 63) / 64, blocks = gx * (ceil_div64(M, 64) + ceil_div64(N, 64));
    if (blocks > 0x7FFFFFFF) return METIS_UNSUPPORTED;
    const QuantParams qu = make_quant_params(Ut.tscale), qv = make_quant_params(Vt.tscale);
    if (sr)
        hipLaunchKernelGGL(k_quantize_factors_t<true>, dim3((unsigned)blocks), dim3(256), 0, s, U, M, V, N, k, qu, qv, Ut.codes,
                           Ut.scales, Vt.codes, Vt.scales, seed_u, seed_v, S_src, S_dst);
    else
        hipLaunchKernelGGL(k_quantize_factors_t<false>, dim3((unsigned)blocks), dim3(256), 0, s, U, M, V, N, k, qu, qv, Ut.codes,
                           Ut.scales, Vt.codes, Vt.scales, seed_u, seed_v, S_src, S_dst);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
