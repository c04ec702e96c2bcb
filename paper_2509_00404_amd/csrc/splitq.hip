// metis_split_quantize: R = A - U diag(S) V^T fused with the NVFP4 quantizer (Sec. 3.2:
// the split; Q_b applied to U, V and R separately; Sec. 2.3: the quantizer).
//
// The low-rank product runs on the bf16 matrix cores with both factors split in two bf16
// parts (hi*hi + hi*lo + lo*hi, ~2^-16 relative), fp32 accumulation; A is streamed once and
// the fp32 residual tile is quantized along both axes before it leaves the workgroup.
#include "quant_dev.h"

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

namespace {

union Frag {
    uint4 u;
    bf16x8_t v;
};

// (U diag(S)) and V as bf16 hi/lo, row-major with the rank padded to a multiple of 16
__global__ void k_split_factors(const float* __restrict__ U, const float* __restrict__ S, const float* __restrict__ V,
                                int64_t M, int64_t N, int k, int kp, bf16_t* __restrict__ us_hi,
                                bf16_t* __restrict__ us_lo, bf16_t* __restrict__ v_hi, bf16_t* __restrict__ v_lo,
                                float* __restrict__ S_out) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < k && S_out) S_out[t] = S[t];
    if (t >= (M + N) * kp) return;
    int64_t row = t / kp;
    int c = (int)(t - row * kp);
    float x = 0.0f;
    bf16_t *hi, *lo;
    if (row < M) {
        if (c < k) x = U[row * k + c] * S[c];
        hi = us_hi + row * kp + c;
        lo = us_lo + row * kp + c;
    } else {
        row -= M;
        if (c < k) x = V[row * k + c];
        hi = v_hi + row * kp + c;
        lo = v_lo + row * kp + c;
    }
    bf16_t h = f32_to_bf16_rne(x);
    *hi = h;
    *lo = f32_to_bf16_rne(x - bf16_to_f32(h));
}

#define RQ_T 64

// grid (ceil(N/64), ceil(M/64)); block 256: 4 waves, each one 32x32 MFMA tile of the residual
__global__ void __launch_bounds__(256)
k_residual_quant(const bf16_t* __restrict__ A, int64_t lda, int64_t M, int64_t N, int kp,
                 const bf16_t* __restrict__ us_hi, const bf16_t* __restrict__ us_lo,
                 const bf16_t* __restrict__ v_hi, const bf16_t* __restrict__ v_lo, QuantParams qp,
                 uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, uint8_t* __restrict__ codes_t,
                 uint8_t* __restrict__ scales_t, float* __restrict__ R_debug) {
    __shared__ float tile[RQ_T][RQ_T + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t m0 = (int64_t)blockIdx.y * RQ_T, n0 = (int64_t)blockIdx.x * RQ_T;
    const int rt = (wave >> 1) * 32, ct = (wave & 1) * 32;
    const int half = lane >> 5;
    int64_t arow = m0 + rt + (lane & 31), bcol = n0 + ct + (lane & 31);
    if (arow >= M) arow = M - 1;            // in-bounds loads; the products are discarded below
    if (bcol >= N) bcol = N - 1;
    float16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    for (int ks = 0; ks < kp; ks += 16) {
        Frag ah, al, bh, bl;
        ah.u = *reinterpret_cast<const uint4*>(us_hi + arow * kp + ks + 8 * half);
        al.u = *reinterpret_cast<const uint4*>(us_lo + arow * kp + ks + 8 * half);
        bh.u = *reinterpret_cast<const uint4*>(v_hi + bcol * kp + ks + 8 * half);
        bl.u = *reinterpret_cast<const uint4*>(v_lo + bcol * kp + ks + 8 * half);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah.v, bh.v, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah.v, bl.v, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al.v, bh.v, acc, 0, 0, 0);
    }
    // residual: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the wave tile
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        int rl = rt + 8 * (v >> 2) + 4 * half + (v & 3), cl = ct + (lane & 31);
        int64_t m = m0 + rl, n = n0 + cl;
        float r = 0.0f;
        if (m < M && n < N) {
            r = bf16_to_f32(A[m * lda + n]) - acc[v];
            if (R_debug) R_debug[m * N + n] = r;
        }
        tile[rl][cl] = r;
    }
    __syncthreads();
    const int line = tid >> 2, blk = tid & 3;
    if (codes) {
        int64_t m = m0 + line, n = n0 + blk * 16;
        if (m < M && n < N) {
            float x[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = tile[line][blk * 16 + i];
            uint2 c;
            uint32_t sc = quantize_block16(x, qp, c);
            *reinterpret_cast<uint2*>(codes + m * (N / 2) + n / 2) = c;
            scales[m * (N / 16) + n / 16] = (uint8_t)sc;
        }
    }
    if (codes_t) {
        int64_t n = n0 + line, m = m0 + blk * 16;
        if (n < N && m < M) {
            float x[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = tile[blk * 16 + i][line];
            uint2 c;
            uint32_t sc = quantize_block16(x, qp, c);
            *reinterpret_cast<uint2*>(codes_t + n * (M / 2) + m / 2) = c;
            scales_t[n * (M / 16) + m / 16] = (uint8_t)sc;
        }
    }
}

bool pow2f(float g) {
    uint32_t u;
    __builtin_memcpy(&u, &g, 4);
    return g > 0.0f && (u & 0x7FFFFFu) == 0 && (u >> 23) != 0 && (u >> 23) != 255;
}

bool fp4_ok(const metis_fp4& f, int64_t rows, int64_t cols) {
    return f.codes && f.scales && pow2f(f.tscale) && f.rows == rows && f.cols == cols && cols % 16 == 0;
}

}  // namespace

extern "C" size_t metis_split_workspace_bytes(int64_t M, int64_t N, int k) {
    if (M < 1 || N < 1 || k < 1) return 0;
    int64_t kp = (k + 15) / 16 * 16;
    return align_up((size_t)M * kp * 2, 256) * 2 + align_up((size_t)N * kp * 2, 256) * 2;
}

extern "C" int metis_split_quantize(void* stream, const metis_mat* A, const float* U, const float* S, const float* V,
                                    int k, metis_split* out, float* R_debug, void* workspace,
                                    size_t workspace_bytes) {
    if (!A || !A->ptr || !U || !S || !V || !out || !workspace) return METIS_INVALID_ARG;
    if (k < 1 || out->k != k || !out->S) return METIS_INVALID_ARG;
    if (A->dtype != METIS_BF16 || k > 128) return METIS_UNSUPPORTED;
    const int64_t M = A->rows, N = A->cols;
    if (M < 1 || N < 1 || A->ld < N) return METIS_BAD_SHAPE;
    const bool want_t = out->Rt.codes != nullptr;
    if (!fp4_ok(out->R, M, N)) return METIS_BAD_SHAPE;
    if (want_t && (!fp4_ok(out->Rt, N, M) || out->Rt.tscale != out->R.tscale)) return METIS_BAD_SHAPE;
    if (!fp4_ok(out->Ut, k, M) || !fp4_ok(out->Vt, k, N)) return METIS_BAD_SHAPE;
    if (workspace_bytes < metis_split_workspace_bytes(M, N, k)) return METIS_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16) return METIS_INVALID_ARG;

    hipStream_t s = (hipStream_t)stream;
    const int kp = (k + 15) / 16 * 16;
    char* ws = (char*)workspace;
    const size_t ub = align_up((size_t)M * kp * 2, 256), vb = align_up((size_t)N * kp * 2, 256);
    bf16_t* us_hi = (bf16_t*)ws;
    bf16_t* us_lo = (bf16_t*)(ws + ub);
    bf16_t* v_hi = (bf16_t*)(ws + 2 * ub);
    bf16_t* v_lo = (bf16_t*)(ws + 2 * ub + vb);
    int64_t tot = (M + N) * kp;
    hipLaunchKernelGGL(k_split_factors, dim3((unsigned)ceil_div64(tot, 256)), dim3(256), 0, s, U, S, V, M, N, k, kp,
                       us_hi, us_lo, v_hi, v_lo, out->S);
    dim3 grid((unsigned)ceil_div64(N, RQ_T), (unsigned)ceil_div64(M, RQ_T));
    const int pi = metis_prof_begin(METIS_PROF_RESIDUAL_QUANT, s);
    hipLaunchKernelGGL(k_residual_quant, grid, dim3(256), 0, s, (const bf16_t*)A->ptr, A->ld, M, N, kp, us_hi, us_lo,
                       v_hi, v_lo, make_quant_params(out->R.tscale), out->R.codes, out->R.scales,
                       want_t ? out->Rt.codes : nullptr, want_t ? out->Rt.scales : nullptr, R_debug);
    metis_prof_end(METIS_PROF_RESIDUAL_QUANT, pi, s);
    METIS_LAUNCH_CHECK();
    // factors: Q(U^T) [k,M], Q(V^T) [k,N], blocks along the long axis
    metis_mat um = {(void*)U, M, k, k, METIS_F32}, vm = {(void*)V, N, k, k, METIS_F32};
    int st = metis_quantize(stream, &um, nullptr, &out->Ut);
    if (st != METIS_OK) return st;
    return metis_quantize(stream, &vm, nullptr, &out->Vt);
}
