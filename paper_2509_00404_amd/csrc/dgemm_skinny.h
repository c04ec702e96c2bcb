// The two contractions of the sample stage that read every sampled row of the bf16 input
// (Sec. 3.1): the sketch Z = A_s Omega and the projection B = H^T A_s.  One side of each
// product is skinny (r = k + p <= 128 columns), so a workgroup owns a full-width strip of the
// output, the bf16 input travels HBM -> registers -> LDS in 16-byte row pieces, and the fp64
// matrix cores (v_mfma_f64_16x16x4_f64) do the arithmetic: bf16 values are exact in fp64 and the
// accumulation is fp64 throughout.  The contraction is split over blockIdx.z; chunk z stores its partial
// strip at part z of the output (parts Ms r resp. r N elements apart), and k_sum_parts_batch adds the parts in
// a fixed order afterwards: no atomics, so the result does not depend on the order workgroups finish in.
#pragma once
#include "dgemm.h"

__device__ __forceinline__ double bf16_bits_to_f64(uint16_t h) {
    return (double)__uint_as_float(((uint32_t)h) << 16);
}

// ---------------------------------------------------------------------------------------
// Sketch: Z[m][j] += sum_k A[rowmap[m]][k] * Om[k][j],  m < Ms, j < r, k in the split's chunk.
//   A   bf16, row stride lda (multiple of 8, base 16-byte aligned), K % 8 == 0
//   Om  bf16 [K][r] row-major, r % 8 == 0, base 16-byte aligned
//   Z   fp64 [ksplit][Ms][r] partial products
// grid (1, ceil(Ms/64), ksplit), block 256: wave w owns rows 16w..16w+15 and all NT column tiles.
// ---------------------------------------------------------------------------------------
#define SK_ROWS 64
#define SK_KS 64
#define SK_LDA 72                     // bf16 per LDS row of the A stage (144 B: 16-byte aligned, bank-spread)
template <int NT>
struct SketchCfg {
    // LDS row length of the Omega stage, = 16 (mod 32) so that the four k-rows a B fragment
    // touches fall into disjoint bank ranges
    static constexpr int LDO = NT * 16 + ((NT * 16) % 32 == 16 ? 0 : 16);
    static constexpr int OM_LOADS = (SK_KS * NT * 2 + 255) / 256;    // 16-byte pieces per thread and stage
};

template <int NT>
__global__ void __launch_bounds__(256)
k_sketch(const bf16_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ rowmap, int64_t Ms, int64_t K,
         const bf16_t* __restrict__ Om, int r, int64_t kchunk, double* __restrict__ Z) {
    constexpr int LDO = SketchCfg<NT>::LDO;
    constexpr int OML = SketchCfg<NT>::OM_LOADS;
    __shared__ __align__(16) uint16_t As[2][SK_ROWS * SK_LDA];
    __shared__ __align__(16) uint16_t Os[2][SK_KS * LDO];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t m0 = (int64_t)blockIdx.y * SK_ROWS;
    const int64_t kbeg = (int64_t)blockIdx.z * kchunk;
    const int64_t kend = kbeg + kchunk < K ? kbeg + kchunk : K;
    if (kbeg >= kend) return;

    // the pad columns r .. 16 NT of the Omega stage stay zero
    for (int e = tid; e < 2 * SK_KS * LDO; e += 256) (&Os[0][0])[e] = 0;
    __syncthreads();

    // A pieces: 64 rows x 8 pieces of 8 bf16, two per thread
    const bf16_t* arow[2];
    bool aok[2];
    int a_lds[2], a_k[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        const int64_t m = m0 + row;
        aok[i] = m < Ms;
        const int64_t src = aok[i] ? (rowmap ? (int64_t)rowmap[m] : m) : 0;
        arow[i] = A + src * lda;
        a_lds[i] = row * SK_LDA + 8 * kc;
        a_k[i] = 8 * kc;
    }
    // Omega pieces: 64 k-rows x r/8 pieces
    const int rc = r >> 3;
    int o_k[OML], o_j[OML];
    bool ook[OML];
#pragma unroll
    for (int i = 0; i < OML; ++i) {
        const int c = tid + 256 * i;
        o_k[i] = c / rc;
        o_j[i] = 8 * (c - o_k[i] * rc);
        ook[i] = o_k[i] < SK_KS;
    }

    uint4 ra[2], ro[OML];
    auto fetch = [&](int64_t kt) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t k = kt + a_k[i];
            ra[i] = (aok[i] && k < kend) ? *reinterpret_cast<const uint4*>(arow[i] + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < OML; ++i) {
            const int64_t k = kt + o_k[i];
            ro[i] = (ook[i] && k < kend) ? *reinterpret_cast<const uint4*>(Om + k * r + o_j[i]) : make_uint4(0, 0, 0, 0);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4*>(&As[buf][a_lds[i]]) = ra[i];
#pragma unroll
        for (int i = 0; i < OML; ++i)
            if (ook[i]) *reinterpret_cast<uint4*>(&Os[buf][o_k[i] * LDO + o_j[i]]) = ro[i];
    };

    double4_t acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[j] = (double4_t){0.0, 0.0, 0.0, 0.0};

    fetch(kbeg);
    stash(0);
    __syncthreads();
    int buf = 0;
    const int arow_l = (wave * 16 + (lane & 15)) * SK_LDA;
    for (int64_t kt = kbeg; kt < kend; kt += SK_KS) {
        const bool more = kt + SK_KS < kend;
        if (more) fetch(kt + SK_KS);
#pragma unroll 4
        for (int s = 0; s < SK_KS / 4; ++s) {
            const int kr = 4 * s + (lane >> 4);
            const double a = bf16_bits_to_f64(As[buf][arow_l + kr]);
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const double b = bf16_bits_to_f64(Os[buf][kr * LDO + 16 * j + (lane & 15)]);
                acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[j], 0, 0, 0);
            }
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    // D layout: lane l, element v -> row 4 v + l / 16, column l % 16
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t m = m0 + wave * 16 + 4 * v + (lane >> 4);
            const int col = 16 * j + (lane & 15);
            if (m < Ms && col < r) Z[(int64_t)blockIdx.z * Ms * r + m * r + col] = acc[j][v];
        }
}

// ---------------------------------------------------------------------------------------
// Projection: B[j][n] += sum_k H[k][j] * A[rowmap[k]][n],  j < r, n < N, k < Ms in the split's chunk.
//   H   fp64 [Ms][r] row-major, r even
//   A   bf16 as above, N % 8 == 0
//   B   fp64 [ksplit][r][N] partial products
// grid (ceil(N/64), 1, ksplit), block 256: wave w owns columns 16w..16w+15 and all NT row tiles.
// Dynamic LDS: 2 H stages (fp64) + 2 A stages (bf16).
// ---------------------------------------------------------------------------------------
#define PJ_COLS 64
#define PJ_KS 32
#define PJ_LDA 80                     // bf16 per LDS row of the A stage: = 16 (mod 32)
template <int NT>
struct ProjectCfg {
    static constexpr int LDH = NT * 16 + ((NT * 16) % 32 == 16 ? 0 : 16);    // doubles, = 16 (mod 32)
    static constexpr int H_LOADS = (PJ_KS * NT * 8 + 255) / 256;              // double2 pieces per thread and stage
    static constexpr size_t LDS = 2 * (size_t)PJ_KS * LDH * sizeof(double) + 2 * (size_t)PJ_KS * PJ_LDA * sizeof(uint16_t);
};

template <int NT>
__global__ void __launch_bounds__(256)
k_project(const double* __restrict__ H_main, const double* __restrict__ H_alt, const int32_t* __restrict__ use_alt, int r,
          const bf16_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ rowmap, int64_t Ms, int64_t N,
          int64_t kchunk, double* __restrict__ B) {
    // the orthonormal basis: the second CholeskyQR pass's output, or the first pass's when that was enough
    const double* __restrict__ H = (use_alt && *use_alt) ? H_alt : H_main;
    constexpr int LDH = ProjectCfg<NT>::LDH;
    constexpr int HL = ProjectCfg<NT>::H_LOADS;
    extern __shared__ __align__(16) unsigned char pj_smem[];
    double* Hs = reinterpret_cast<double*>(pj_smem);                                   // [2][PJ_KS * LDH]
    uint16_t* As = reinterpret_cast<uint16_t*>(pj_smem + 2 * (size_t)PJ_KS * LDH * sizeof(double));   // [2][PJ_KS * PJ_LDA]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * PJ_COLS;
    const int64_t kbeg = (int64_t)blockIdx.z * kchunk;
    const int64_t kend = kbeg + kchunk < Ms ? kbeg + kchunk : Ms;
    if (kbeg >= kend) return;

    for (int e = tid; e < 2 * PJ_KS * LDH; e += 256) Hs[e] = 0.0;      // pad columns r .. 16 NT stay zero
    __syncthreads();

    // H pieces: 32 k-rows x r/2 pairs of doubles
    const int rc = r >> 1;
    int h_k[HL], h_j[HL];
    bool hok[HL];
#pragma unroll
    for (int i = 0; i < HL; ++i) {
        const int c = tid + 256 * i;
        h_k[i] = c / rc;
        h_j[i] = 2 * (c - h_k[i] * rc);
        hok[i] = h_k[i] < PJ_KS;
    }
    // A pieces: 32 k-rows x 8 pieces of 8 bf16, one per thread
    const int a_kr = tid >> 3, a_n = 8 * (tid & 7);
    const bool a_nok = n0 + a_n < N;

    double2 rh[HL];
    uint4 ra;
    auto fetch = [&](int64_t kt) {
#pragma unroll
        for (int i = 0; i < HL; ++i) {
            const int64_t k = kt + h_k[i];
            rh[i] = (hok[i] && k < kend) ? *reinterpret_cast<const double2*>(H + k * r + h_j[i]) : make_double2(0.0, 0.0);
        }
        const int64_t k = kt + a_kr;
        if (a_nok && k < kend) {
            const int64_t src = rowmap ? (int64_t)rowmap[k] : k;
            ra = *reinterpret_cast<const uint4*>(A + src * lda + n0 + a_n);
        } else {
            ra = make_uint4(0, 0, 0, 0);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < HL; ++i)
            if (hok[i]) *reinterpret_cast<double2*>(&Hs[(size_t)buf * PJ_KS * LDH + h_k[i] * LDH + h_j[i]]) = rh[i];
        *reinterpret_cast<uint4*>(&As[buf * PJ_KS * PJ_LDA + a_kr * PJ_LDA + a_n]) = ra;
    };

    double4_t acc[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[i] = (double4_t){0.0, 0.0, 0.0, 0.0};

    fetch(kbeg);
    stash(0);
    __syncthreads();
    int buf = 0;
    for (int64_t kt = kbeg; kt < kend; kt += PJ_KS) {
        const bool more = kt + PJ_KS < kend;
        if (more) fetch(kt + PJ_KS);
        const double* hs = Hs + (size_t)buf * PJ_KS * LDH;
        const uint16_t* as = As + buf * PJ_KS * PJ_LDA;
#pragma unroll 4
        for (int s = 0; s < PJ_KS / 4; ++s) {
            const int kr = 4 * s + (lane >> 4);
            const double b = bf16_bits_to_f64(as[kr * PJ_LDA + wave * 16 + (lane & 15)]);
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const double a = hs[kr * LDH + 16 * i + (lane & 15)];
                acc[i] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[i], 0, 0, 0);
            }
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int j = 16 * i + 4 * v + (lane >> 4);
            const int64_t n = n0 + wave * 16 + (lane & 15);
            if (j < r && n < N) B[((int64_t)blockIdx.z * r + j) * N + n] = acc[i][v];
        }
}

// contraction split for ~768 workgroups, every split at least one stage deep
static inline int64_t skinny_kchunk(int64_t K, int64_t tiles, int stage) {
    int64_t want = ceil_div64(768, tiles), maxs = ceil_div64(K, stage);
    int64_t ks = want < maxs ? want : maxs;
    if (ks < 1) ks = 1;
    return ceil_div64(ceil_div64(K, ks), stage) * stage;
}

// true when the fast kernels' layout preconditions hold
static inline bool skinny_ok(const bf16_t* A, int64_t lda, int64_t N, int r) {
    return r % 8 == 0 && r >= 8 && r <= 128 && N % 8 == 0 && lda % 8 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0;
}

// number of partial products the two kernels write
static inline int sketch_parts(int64_t Ms, int64_t K) {
    return (int)ceil_div64(K, skinny_kchunk(K, ceil_div64(Ms, SK_ROWS), SK_KS));
}
static inline int project_parts(int64_t Ms, int64_t N) {
    return (int)ceil_div64(Ms, skinny_kchunk(Ms, ceil_div64(N, PJ_COLS), PJ_KS));
}

// Z = sketch_parts(Ms, K) partial products [Ms][r]
static inline int launch_sketch(hipStream_t s, const bf16_t* A, int64_t lda, const uint32_t* rowmap, int64_t Ms, int64_t K,
                                const bf16_t* Om, int r, double* Z) {
    const int64_t kchunk = skinny_kchunk(K, ceil_div64(Ms, SK_ROWS), SK_KS);
    dim3 grid(1, (unsigned)ceil_div64(Ms, SK_ROWS), (unsigned)ceil_div64(K, kchunk));
#define SKETCH_CASE(NT)                                                                                          \
    hipLaunchKernelGGL(k_sketch<NT>, grid, dim3(256), 0, s, A, lda, rowmap, Ms, K, Om, r, kchunk, Z);
    switch ((r + 15) / 16) {
        case 1: SKETCH_CASE(1) break;
        case 2: SKETCH_CASE(2) break;
        case 3: SKETCH_CASE(3) break;
        case 4: SKETCH_CASE(4) break;
        case 5: SKETCH_CASE(5) break;
        case 6: SKETCH_CASE(6) break;
        case 7: SKETCH_CASE(7) break;
        case 8: SKETCH_CASE(8) break;
        default: return METIS_UNSUPPORTED;
    }
#undef SKETCH_CASE
    return METIS_OK;
}

// B = project_parts(Ms, N) partial products [r][N]
static inline int launch_project(hipStream_t s, const double* H, const double* H_alt, const int32_t* use_alt, int r,
                                 const bf16_t* A, int64_t lda, const uint32_t* rowmap, int64_t Ms, int64_t N, double* B) {
    const int64_t kchunk = skinny_kchunk(Ms, ceil_div64(N, PJ_COLS), PJ_KS);
    dim3 grid((unsigned)ceil_div64(N, PJ_COLS), 1, (unsigned)ceil_div64(Ms, kchunk));
#define PROJECT_CASE(NT)                                                                                         \
    {                                                                                                            \
        const size_t lds = ProjectCfg<NT>::LDS;                                                                  \
        static LdsLimitCache lds_set;                                                                            \
        if (!ensure_dyn_lds((const void*)k_project<NT>, lds, lds_set)) return METIS_HIP_ERROR;                   \
        hipLaunchKernelGGL(k_project<NT>, grid, dim3(256), lds, s, H, H_alt, use_alt, r, A, lda, rowmap, Ms, N, kchunk, B);      \
    }
    switch ((r + 15) / 16) {
        case 1: PROJECT_CASE(1) break;
        case 2: PROJECT_CASE(2) break;
        case 3: PROJECT_CASE(3) break;
        case 4: PROJECT_CASE(4) break;
        case 5: PROJECT_CASE(5) break;
        case 6: PROJECT_CASE(6) break;
        case 7: PROJECT_CASE(7) break;
        case 8: PROJECT_CASE(8) break;
        default: return METIS_UNSUPPORTED;
    }
#undef PROJECT_CASE
    return METIS_OK;
}

// ---------------------------------------------------------------------------------------
// Gram matrix of a tall skinny matrix given as a sum of partial arrays (the broadcast's per-split
// partial products):  S = sum_p C_p  (M x r, fp32),  G_b = S_b^T S_b  (r x r, fp64) for the rows S_b of workgroup b:
// G holds ceil(M / GR_ROWS) partial Gram matrices, added in a fixed order afterwards (k_sum_parts_batch).
// The summed matrix is written back as fp32 (sum_out, may alias part 0) for the later U = S T.
//   r % 4 == 0, C 16-byte aligned.
// grid (ceil(M / GR_ROWS)), block 256; wave w owns row tiles w, w+4 of G and all NT column tiles.
// ---------------------------------------------------------------------------------------
#define GR_ROWS 64                    // rows of C per workgroup
#define GR_KS 32                      // rows per stage
template <int NT>
__global__ void __launch_bounds__(256)
k_gram_parts(const float* C, int r, int64_t M, int nparts, int64_t part_stride, float* sum_out,
             double* __restrict__ G) {
    constexpr int LDC = NT * 16 + ((NT * 16) % 32 == 16 ? 0 : 16);      // doubles, = 16 (mod 32)
    constexpr int PIECES = (GR_KS * NT * 4 + 255) / 256;                // float4 pieces per thread and stage
    constexpr int RT = (NT + 3) / 4;                                     // row tiles per wave
    __shared__ double Cs[GR_KS * LDC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t m0 = (int64_t)blockIdx.x * GR_ROWS;
    const int rc = r >> 2;
    for (int e = tid; e < GR_KS * LDC; e += 256) Cs[e] = 0.0;           // pad columns r .. 16 NT stay zero
    double4_t acc[RT][NT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = (double4_t){0.0, 0.0, 0.0, 0.0};
    __syncthreads();
    for (int64_t mt = m0; mt < m0 + GR_ROWS && mt < M; mt += GR_KS) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int c = tid + 256 * i, row = c / rc, col = 4 * (c - row * rc);
            if (row < GR_KS) {
                const int64_t m = mt + row;
                double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
                if (m < M) {
                    const float* src = C + m * r + col;
                    int p = 0;
                    for (; p + 4 <= nparts; p += 4) {          // four loads in flight
                        float4 v[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(src + (p + u) * part_stride);
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            s0 += (double)v[u].x;
                            s1 += (double)v[u].y;
                            s2 += (double)v[u].z;
                            s3 += (double)v[u].w;
                        }
                    }
                    for (; p < nparts; ++p) {
                        const float4 v = *reinterpret_cast<const float4*>(src + p * part_stride);
                        s0 += (double)v.x;
                        s1 += (double)v.y;
                        s2 += (double)v.z;
                        s3 += (double)v.w;
                    }
                    if (sum_out) {
                        // the Gram matrix is taken of the rounded sums, the same matrix the caller multiplies later
                        const float4 o = make_float4((float)s0, (float)s1, (float)s2, (float)s3);
                        *reinterpret_cast<float4*>(sum_out + m * r + col) = o;
                        s0 = o.x; s1 = o.y; s2 = o.z; s3 = o.w;
                    }
                }
                double* d = &Cs[row * LDC + col];
                d[0] = s0; d[1] = s1; d[2] = s2; d[3] = s3;
            }
        }
        __syncthreads();
#pragma unroll 2
        for (int s = 0; s < GR_KS / 4; ++s) {
            const int kr = 4 * s + (lane >> 4);
            double b[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) b[j] = Cs[kr * LDC + 16 * j + (lane & 15)];
            // no branch around the matrix instructions: a wave whose row tile does not exist recomputes
            // tile 0 and drops the result in the epilogue
#pragma unroll
            for (int i = 0; i < RT; ++i) {
                const int it = wave + 4 * i < NT ? wave + 4 * i : 0;
                const double a = Cs[kr * LDC + 16 * it + (lane & 15)];
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b[j], acc[i][j], 0, 0, 0);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        const int it = wave + 4 * i;
        if (it >= NT) continue;
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int a = 16 * it + 4 * v + (lane >> 4), b = 16 * j + (lane & 15);
                if (a < r && b < r) G[((int64_t)blockIdx.x * r + a) * r + b] = acc[i][j][v];
            }
    }
}

static inline int launch_gram_parts(hipStream_t s, const float* C, int r, int64_t M, int nparts, int64_t part_stride,
                                    float* sum_out, double* G) {
    dim3 grid((unsigned)ceil_div64(M, GR_ROWS));
#define GRAM_CASE(NT) hipLaunchKernelGGL(k_gram_parts<NT>, grid, dim3(256), 0, s, C, r, M, nparts, part_stride, sum_out, G);
    switch ((r + 15) / 16) {
        case 1: GRAM_CASE(1) break;
        case 2: GRAM_CASE(2) break;
        case 3: GRAM_CASE(3) break;
        case 4: GRAM_CASE(4) break;
        case 5: GRAM_CASE(5) break;
        case 6: GRAM_CASE(6) break;
        case 7: GRAM_CASE(7) break;
        case 8: GRAM_CASE(8) break;
        default: return METIS_UNSUPPORTED;
    }
#undef GRAM_CASE
    return METIS_OK;
}
