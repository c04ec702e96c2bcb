// MXFP4 variant of the block-FP4 GEMM: the microscaling format that Sec. 2.3 names next to NVFP4
// (OCP MX v1.0: blocks of 32, one power-of-two E8M0 scale per block, E2M1 elements).  Its scales are
// exactly what gfx950's block-scaled matrix instruction applies in hardware, so the codes go from
// LDS straight into v_mfma_scale_f32_32x32x64_f8f6f4 with no expansion in the vector ALUs: this is
// the chip's FP4 rate, against which the NVFP4 path (E4M3 scales per 16, expanded to fp16) can be read.
#include <type_traits>
#include "common.h"
#include "gemm_tile.h"
#include "../../include/metis.h"

typedef int int8v_t __attribute__((ext_vector_type(8)));
typedef uint32_t uvec4_t __attribute__((ext_vector_type(4)));   // a native vector: copies stay in registers
typedef uint32_t uvec2_t __attribute__((ext_vector_type(2)));

namespace {

// ---- quantizer: one lane per block of 32 consecutive elements of a row ----
// X = 2^(floor(log2 amax) - 2); elements round to the nearest E2M1 value of e / X, ties to the even code,
// magnitudes above 6 saturate (the packed converter does the rounding, saturation and nibble packing).
template <typename T>
__global__ void __launch_bounds__(256)
k_quantize_mx(const T* __restrict__ A, int64_t ld, int64_t M, int64_t nblk /* cols / 32 */, uint8_t* __restrict__ codes,
              uint8_t* __restrict__ scales) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= M * nblk) return;
    const int64_t row = t / nblk, bc = t - row * nblk;
    float v[32];
    if constexpr (sizeof(T) == 2) {
        const uint4* src = reinterpret_cast<const uint4*>(A + row * ld + bc * 32);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 a = src[i];
            const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[8 * i + 2 * j] = bf16lo_to_f32(w[j]);
                v[8 * i + 2 * j + 1] = bf16hi_to_f32(w[j]);
            }
        }
    } else {
        const float4* src = reinterpret_cast<const float4*>(A + row * ld + bc * 32);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float4 a = src[i];
            v[4 * i] = a.x; v[4 * i + 1] = a.y; v[4 * i + 2] = a.z; v[4 * i + 3] = a.w;
        }
    }
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(v[i]));
    int sh = -127;
    if (amax > 0.0f) {
        sh = ilogbf(amax) - 2;
        sh = sh < -127 ? -127 : (sh > 127 ? 127 : sh);
    }
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float y0 = ldexpf(v[8 * i + 2 * j], -sh), y1 = ldexpf(v[8 * i + 2 * j + 1], -sh);   // exact
            switch (j) {
                case 0: w[i] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w[i], y0, y1, 1.0f, 0); break;
                case 1: w[i] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w[i], y0, y1, 1.0f, 1); break;
                case 2: w[i] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w[i], y0, y1, 1.0f, 2); break;
                default: w[i] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w[i], y0, y1, 1.0f, 3); break;
            }
        }
    }
    *reinterpret_cast<uint4*>(codes + t * 16) = make_uint4(w[0], w[1], w[2], w[3]);     // [M, cols/2] contiguous
    scales[t] = (uint8_t)(sh + 127);
}

// ---- GEMM C[M,N] = A[M,K] B[N,K]^T ----
// 256 x 256 tile, 8 waves of 128 x 64 (4 x 2 accumulator tiles of 32 x 32, two waves per SIMD).  A lane's operand of
// one matrix instruction is the 32 codes (16 bytes) of row lane % 32, contraction half lane / 32, and the E8M0 byte
// of exactly that block of 32.  With no expansion work the kernel lives on operand delivery:
//  * a stage is 256 contraction elements = 128 bytes of every row = whole cache lines (with 64-byte stages every
//    line crossed L2 -> L1 twice, which was the limit), four matrix instructions deep;
//  * the next stage's global data sits in registers for one stage before it is written to the other LDS buffer;
//  * fragments are double-buffered in registers: step s+1 is read from LDS while step s multiplies;
//  * a wave issues in order and a matrix instruction holds its pipe for 32 cycles, so memory instructions of one
//    wave leave the pipe idle while they issue: the second wave on the SIMD fills those gaps (four waves of
//    128 x 128 need fewer LDS bytes per flop but reach 10 % less).
// The stage body is branch-free (stage indices are clamped; the last stage loads and stores data nobody uses).
#define MX_KI 256
#define MX_CROW (MX_KI / 2 + 16)      // padded code row in LDS: 144 bytes, 16-byte reads of 8 consecutive rows hit 8 bank groups
#define MX_SROW 8                     // the row's eight scale bytes of a stage

struct MxOperand {
    const uint8_t* codes;             // [rows, K/2]
    const uint8_t* scales;            // [rows, K/32]
    int64_t rows;
};

// TAIL: K is not a multiple of the 256-deep stage.  The last stage then exists only in part: its missing blocks of 32
// enter as zero codes under a unit scale, and because scale rows are no longer 8-byte aligned every stage's scale
// bytes are fetched one by one.
template <typename OUT, bool TAIL>
__global__ void __launch_bounds__(512)
k_mxfp4_gemm_nt(MxOperand A, MxOperand B, int64_t K, OUT* __restrict__ C, int64_t ldc, TileMap tmap) {
    constexpr int TM = 4, TN = 2, BM = 256, BN = 256, KS = MX_KI / 64, NV = 4;   // NV: 16-byte code vectors per thread, operand and stage
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int OFF_CB = BM * MX_CROW, OFF_SA = (BM + BN) * MX_CROW, OFF_SB = OFF_SA + BM * MX_SROW,
                  BUF = OFF_SB + BN * MX_SROW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int tile_m, tile_n;
    tile_coords(tmap, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int wm = (wave >> 2) * 128, wn = (wave & 3) * 64;
    const int li = lane & 31, half = lane >> 5;

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int niter = (int)((K + MX_KI - 1) / MX_KI);
    // this thread's share of a stage: code vectors v = 0..3 of each operand (row tid/8 + 64 v, 16-byte segment
    // tid % 8: a row's 128 bytes are read by 8 consecutive lanes) and the 8 scale bytes of rows tid (A) and tid (B);
    // rows past the operand's end re-read its last row.  Byte offsets fit 32 bits (checked by the host).
    uint32_t oa[NV], ob[NV], osga, osgb;
    const uint32_t cstride = (uint32_t)(K / 2), sstride = (uint32_t)(K / 32);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        int64_t ga = m0 + (tid >> 3) + 64 * v, gb = n0 + (tid >> 3) + 64 * v;
        if (ga >= A.rows) ga = A.rows - 1;
        if (gb >= B.rows) gb = B.rows - 1;
        oa[v] = (uint32_t)ga * cstride + 16u * (tid & 7);
        ob[v] = (uint32_t)gb * cstride + 16u * (tid & 7);
    }
    {
        // threads 0..255 carry A's scale rows, threads 256..511 B's
        int64_t ga = m0 + (tid & 255), gb = n0 + (tid & 255);
        if (ga >= A.rows) ga = A.rows - 1;
        if (gb >= B.rows) gb = B.rows - 1;
        osga = (uint32_t)ga * sstride;
        osgb = (uint32_t)gb * sstride;
    }
    uvec4_t ra[NV], rb[NV];
    uvec2_t rs;
    auto clampst = [&](int st) { return st < niter ? st : niter - 1; };
    auto load_stage = [&](int st) __attribute__((always_inline)) {
        const uint8_t* ca = A.codes + (size_t)st * (MX_KI / 2);
        const uint8_t* cb = B.codes + (size_t)st * (MX_KI / 2);
        if (!TAIL) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                ra[v] = *reinterpret_cast<const uvec4_t*>(ca + oa[v]);
                rb[v] = *reinterpret_cast<const uvec4_t*>(cb + ob[v]);
            }
            rs = *reinterpret_cast<const uvec2_t*>((tid < 256 ? A.scales + osga : B.scales + osgb) + (size_t)st * (MX_KI / 32));
        } else {
            // this lane's 16-byte segment is one block of 32 contraction elements: it exists or it does not
            const bool seg_ok = (int64_t)st * MX_KI + 32 * (tid & 7) < K;
            const uvec4_t zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const uvec4_t xa = *reinterpret_cast<const uvec4_t*>(seg_ok ? ca + oa[v] : A.codes);
                const uvec4_t xb = *reinterpret_cast<const uvec4_t*>(seg_ok ? cb + ob[v] : B.codes);
                ra[v] = seg_ok ? xa : zero4;
                rb[v] = seg_ok ? xb : zero4;
            }
            const uint8_t* sp = tid < 256 ? A.scales + osga : B.scales + osgb;
            const int64_t b0 = (int64_t)st * (MX_KI / 32), nb = K / 32;
            uint32_t w[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t byte = b0 + i < nb ? (uint32_t)sp[b0 + i] : 127u;          // 127 = scale 1 for an absent block
                w[i >> 2] |= byte << (8 * (i & 3));
            }
            rs.x = w[0];
            rs.y = w[1];
        }
    };
    auto store_stage = [&](uint8_t* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int row = (tid >> 3) + 64 * v, seg = tid & 7;
            *reinterpret_cast<uvec4_t*>(buf + row * MX_CROW + 16 * seg) = ra[v];
            *reinterpret_cast<uvec4_t*>(buf + OFF_CB + row * MX_CROW + 16 * seg) = rb[v];
        }
        *reinterpret_cast<uvec2_t*>(buf + OFF_SA + tid * MX_SROW) = rs;          // B's scale rows follow A's
    };

    // per-lane byte offsets of this wave's fragment rows inside a buffer
    const int oca = (wm + li) * MX_CROW + 16 * half, ocb = OFF_CB + (wn + li) * MX_CROW + 16 * half;
    const int osa = OFF_SA + (wm + li) * MX_SROW, osb = OFF_SB + (wn + li) * MX_SROW;
    uvec4_t fa[2][TM], fb[2][TN];     // code fragments, two slots
    uint32_t sa[2][TM], sb[2][TN];    // the rows' two scale words of the stage, shifted so that byte 0 / byte 2 are this lane's blocks
    auto read_codes = [&](const uint8_t* buf, int ks, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[slot][i] = *reinterpret_cast<const uvec4_t*>(buf + oca + 32 * i * MX_CROW + 32 * ks);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[slot][j] = *reinterpret_cast<const uvec4_t*>(buf + ocb + 32 * j * MX_CROW + 32 * ks);
    };
    auto read_scales = [&](const uint8_t* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const uvec2_t w = *reinterpret_cast<const uvec2_t*>(buf + osa + 32 * i * MX_SROW);
            sa[0][i] = w.x >> (8 * half);
            sa[1][i] = w.y >> (8 * half);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const uvec2_t w = *reinterpret_cast<const uvec2_t*>(buf + osb + 32 * j * MX_SROW);
            sb[0][j] = w.x >> (8 * half);
            sb[1][j] = w.y >> (8 * half);
        }
    };
    auto mma = [&](auto KSC) __attribute__((always_inline)) {
        constexpr int ks = decltype(KSC)::value, slot = ks & 1, word = ks >> 1, sel = 2 * (ks & 1);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int8v_t a = {(int)fa[slot][i].x, (int)fa[slot][i].y, (int)fa[slot][i].z, (int)fa[slot][i].w, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int8v_t b = {(int)fb[slot][j].x, (int)fb[slot][j].y, (int)fb[slot][j].z, (int)fb[slot][j].w, 0, 0, 0, 0};
                // formats 4 = FP4 (E2M1) for both operands; the scale byte is byte `sel` of the shifted word
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i][j], 4, 4, sel, (int)sa[word][i],
                                                                             sel, (int)sb[word][j]);
            }
        }
    };

    load_stage(0);
    store_stage(lds);
    __syncthreads();
    load_stage(clampst(1));
    read_codes(lds, 0, 0);
    read_scales(lds);

#pragma unroll 1
    for (int it = 0; it < niter; ++it) {
        const uint8_t* bufc = lds + (it & 1) * BUF;
        uint8_t* bufn = lds + ((it & 1) ^ 1) * BUF;
        read_codes(bufc, 1, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(std::integral_constant<int, 0>{});
        store_stage(bufn);                        // stage it + 1 (loaded one stage ago) to the other buffer ...
        load_stage(clampst(it + 2));              // ... and its registers take stage it + 2
        __builtin_amdgcn_sched_barrier(0);
        read_codes(bufc, 2, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(std::integral_constant<int, 1>{});
        __builtin_amdgcn_sched_barrier(0);
        read_codes(bufc, 3, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(std::integral_constant<int, 2>{});
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();                          // next stage is in LDS; this stage's codes are all in registers
        read_codes(bufn, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(std::integral_constant<int, 3>{});
        __builtin_amdgcn_sched_barrier(0);
        read_scales(bufn);
    }

    const bool interior = m0 + BM <= A.rows && n0 + BN <= B.rows;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t c = n0 + wn + 32 * j + li;
            const int64_t rbase = m0 + wm + 32 * i + 4 * half;
            if (interior) {
                store_tile16<OUT>(C + rbase * ldc + c, ldc, acc[i][j], 1.0f);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t r = rbase + 8 * (v >> 2) + (v & 3);
                    if (r < A.rows && c < B.rows) store_out<OUT>(C + r * ldc + c, acc[i][j][v]);
                }
            }
        }
}

constexpr size_t MX_LDS = 2 * (size_t)(256 + 256) * (MX_CROW + MX_SROW);

template <typename OUT>
int launch_mx_gemm(hipStream_t s, const MxOperand& a, const MxOperand& b, int64_t K, OUT* C, int64_t ldc) {
    const int64_t tm = ceil_div64(a.rows, 256), tn = ceil_div64(b.rows, 256);
    if (tm * tn > 0x7FFFFFFF) return METIS_UNSUPPORTED;
    if (K % MX_KI == 0) {
        auto kern = k_mxfp4_gemm_nt<OUT, false>;
        static LdsLimitCache lds_set;
        if (!ensure_dyn_lds((const void*)kern, MX_LDS, lds_set)) return METIS_HIP_ERROR;
        hipLaunchKernelGGL(kern, dim3((unsigned)(tm * tn)), dim3(512), MX_LDS, s, a, b, K, C, ldc, make_tile_map(tm, tn));
    } else {
        auto kern = k_mxfp4_gemm_nt<OUT, true>;
        static LdsLimitCache lds_set;
        if (!ensure_dyn_lds((const void*)kern, MX_LDS, lds_set)) return METIS_HIP_ERROR;
        hipLaunchKernelGGL(kern, dim3((unsigned)(tm * tn)), dim3(512), MX_LDS, s, a, b, K, C, ldc, make_tile_map(tm, tn));
    }
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

bool mx_ok(const metis_mxfp4* t) { return t && t->codes && t->scales && t->rows >= 1 && t->cols >= 32 && t->cols % 32 == 0; }

}  // namespace

extern "C" int metis_quantize_mx(void* stream, const metis_mat* A, metis_mxfp4* out) {
    if (!A || !A->ptr || !mx_ok(out)) return METIS_INVALID_ARG;
    if (A->dtype != METIS_BF16 && A->dtype != METIS_F32) return METIS_INVALID_ARG;
    if (A->rows != out->rows || A->cols != out->cols || A->ld < A->cols) return METIS_BAD_SHAPE;
    const int64_t esz = A->dtype == METIS_BF16 ? 2 : 4;
    if ((A->ld * esz) % 16 || reinterpret_cast<uintptr_t>(A->ptr) % 16 || reinterpret_cast<uintptr_t>(out->codes) % 16)
        return METIS_BAD_SHAPE;                                       // 16-byte row loads and code stores
    const int64_t nblk = A->cols / 32, total = A->rows * nblk;
    hipStream_t s = (hipStream_t)stream;
    if (A->dtype == METIS_BF16)
        hipLaunchKernelGGL(k_quantize_mx<bf16_t>, dim3((unsigned)ceil_div64(total, 256)), dim3(256), 0, s,
                           (const bf16_t*)A->ptr, A->ld, A->rows, nblk, out->codes, out->scales);
    else
        hipLaunchKernelGGL(k_quantize_mx<float>, dim3((unsigned)ceil_div64(total, 256)), dim3(256), 0, s,
                           (const float*)A->ptr, A->ld, A->rows, nblk, out->codes, out->scales);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

extern "C" int metis_mxfp4_gemm_nt(void* stream, const metis_mxfp4* A, const metis_mxfp4* B, metis_mat* C) {
    if (!mx_ok(A) || !mx_ok(B) || !C || !C->ptr) return METIS_INVALID_ARG;
    if (C->dtype != METIS_BF16 && C->dtype != METIS_F32) return METIS_INVALID_ARG;
    if (A->cols != B->cols || C->rows != A->rows || C->cols != B->rows || C->ld < C->cols) return METIS_BAD_SHAPE;
    const int64_t K = A->cols;
    if (A->rows * (K / 2) > 0xFFFFFFFFll || B->rows * (K / 2) > 0xFFFFFFFFll) return METIS_UNSUPPORTED;   // 32-bit byte offsets
    if (reinterpret_cast<uintptr_t>(A->codes) % 16 || reinterpret_cast<uintptr_t>(B->codes) % 16 ||
        (K % MX_KI == 0 && (reinterpret_cast<uintptr_t>(A->scales) % 8 || reinterpret_cast<uintptr_t>(B->scales) % 8)))
        return METIS_BAD_SHAPE;
    const MxOperand a = {A->codes, A->scales, A->rows}, b = {B->codes, B->scales, B->rows};
    hipStream_t s = (hipStream_t)stream;
    if (C->dtype == METIS_F32) return launch_mx_gemm<float>(s, a, b, K, (float*)C->ptr, C->ld);
    return launch_mx_gemm<bf16_t>(s, a, b, K, (bf16_t*)C->ptr, C->ld);
}
