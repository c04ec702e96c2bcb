// FP4 GEMMs on split operands (Sec. 3.2: Eq. 2 fprop, Eq. 3 dgrad, dL/dW_R wgrad).
//
// One NT kernel serves all three: C[M,N] = alpha * deq(A)[M,K] deq(B)[N,K]^T + Aext Bext^T.
// NVFP4 (block 16, E4M3 scale) is not an MX format, so the scaled-MFMA path cannot apply
// the block scales; codes are expanded in registers to fp16 (grid * e4m3 has at most 6
// significant bits: exact) and multiplied on the fp16 matrix cores with fp32 accumulation.
// The low-rank terms of the split enter as extra contraction columns (bf16, same
// accumulators):  Abar Bbar^T = Ra Rb^T + [(Ra Vb + Ua Sa Va^T Vb) Sb] Ub^T + (Ua Sa)(Rb Va)^T.
#include <stdlib.h>
#include "common.h"
#include "gemm_tile.h"

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

namespace {

#define G_KI 128                    // contraction elements per LDS stage
#define G_CROW (G_KI / 2 + 4)       // padded code row in LDS (bytes): dword stride 17, conflict-free
#define G_SROW 20                   // 8 block scales per row and stage as fp16, + pad (dword stride 5: conflict-free)

struct Fp4Operand {
    const uint8_t* codes;           // [rows, K/2]
    const uint8_t* scales;          // [rows, K/16]
    int64_t rows;
};

// One thread's share of a stage of ROWS rows x 64 B of codes: V = ROWS*4/NT 16-byte code vectors.
// NT = threads per workgroup.
template <int V>
struct StageRegs {
    uint4 c[V];
};

// The 8 scale bytes per row and stage of both operands, dealt over all threads of the workgroup:
// thread t takes rows t, t + NT, ... of the BM + BN staged rows (A's rows first).
template <int V>
struct ScaleRegs {
    uint2 s[V];
};

template <int BM, int BN, int NT, bool VEC>
__device__ __forceinline__ void scale_load(const Fp4Operand& A, const Fp4Operand& B, int64_t m0, int64_t n0, int64_t K,
                                           int64_t k0, ScaleRegs<(BM + BN + NT - 1) / NT>& rg, int tid) {
    constexpr int V = (BM + BN + NT - 1) / NT;
    const int64_t sstride = K / 16;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int e = tid + NT * v;
        if ((BM + BN) % NT == 0 || e < BM + BN) {
            const bool isa = e < BM;
            const Fp4Operand& op = isa ? A : B;
            int64_t gr = isa ? m0 + e : n0 + (e - BM);
            if (gr >= op.rows) gr = op.rows - 1;
            const uint8_t* src = op.scales + gr * sstride + k0 / 16;
            if (VEC) {
                rg.s[v] = *reinterpret_cast<const uint2*>(src);
            } else {
                uint32_t w[2] = {0, 0};
                for (int i = 0; i < 8; ++i)
                    if (k0 / 16 + i < sstride) w[i >> 2] |= (uint32_t)src[i] << (8 * (i & 3));
                rg.s[v] = make_uint2(w[0], w[1]);
            }
        }
    }
}

// E4M3 bytes -> fp16 with the hardware FP8 converter (exact; checked against the format's
// definition for all 256 bytes), 8 scales = 16 bytes per row
template <int BM, int BN, int NT>
__device__ __forceinline__ void scale_store(const ScaleRegs<(BM + BN + NT - 1) / NT>& rg, uint8_t* __restrict__ lsa,
                                            uint8_t* __restrict__ lsb, int tid) {
    constexpr int V = (BM + BN + NT - 1) / NT;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int e = tid + NT * v;
        if ((BM + BN) % NT == 0 || e < BM + BN) {
            uint32_t* dst = reinterpret_cast<uint32_t*>(e < BM ? lsa + e * G_SROW : lsb + (e - BM) * G_SROW);
            dst[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rg.s[v].x, 1.0f, false));
            dst[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rg.s[v].x, 1.0f, true));
            dst[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rg.s[v].y, 1.0f, false));
            dst[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rg.s[v].y, 1.0f, true));
        }
    }
}

template <int ROWS, int NT, bool VEC>
__device__ __forceinline__ void stage_load(const Fp4Operand& op, int64_t r0, int64_t K, int64_t k0,
                                           StageRegs<ROWS * 4 / NT>& rg, int tid) {
    constexpr int T = ROWS * 4 / NT;
    const int64_t cstride = K / 2, sstride = K / 16;
#pragma unroll
    for (int v = 0; v < T; ++v) {
        int e = tid + NT * v;
        int row = e >> 2, seg = e & 3;
        int64_t gr = r0 + row;
        if (gr >= op.rows) gr = op.rows - 1;
        const uint8_t* src = op.codes + gr * cstride + k0 / 2 + 16 * seg;
        if (VEC) {
            rg.c[v] = *reinterpret_cast<const uint4*>(src);
        } else {
            uint32_t w[4] = {0, 0, 0, 0};
            for (int b = 0; b < 16; ++b) {
                int64_t kb = k0 / 2 + 16 * seg + b;
                if (kb < cstride) w[b >> 2] |= (uint32_t)src[b] << (8 * (b & 3));
            }
            rg.c[v] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

template <int ROWS, int NT>
__device__ __forceinline__ void stage_store(const StageRegs<ROWS * 4 / NT>& rg, uint8_t* __restrict__ lc, int tid) {
    constexpr int T = ROWS * 4 / NT;
#pragma unroll
    for (int v = 0; v < T; ++v) {
        int e = tid + NT * v;
        int row = e >> 2, seg = e & 3;
        uint32_t* dst = reinterpret_cast<uint32_t*>(lc + row * G_CROW + 16 * seg);
        dst[0] = rg.c[v].x; dst[1] = rg.c[v].y; dst[2] = rg.c[v].z; dst[3] = rg.c[v].w;
    }
}

// 8 codes (one dword) times one block scale -> 8 fp16.  `spair` holds the fp16 scales of two
// consecutive blocks; `hi` picks the second (the splat folds into the packed multiply's operand select).
__device__ __forceinline__ half8_t dequant8(uint32_t cw, uint32_t spair, bool hi) {
    const half2_t sp = __builtin_bit_cast(half2_t, spair);
    const half2_t s2 = hi ? (half2_t){sp[1], sp[1]} : (half2_t){sp[0], sp[0]};
    const half2_t c0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 0);
    const half2_t c1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 1);
    const half2_t c2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 2);
    const half2_t c3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(cw, 1.0f, 3);
    half2_t p0 = c0 * s2, p1 = c1 * s2, p2 = c2 * s2, p3 = c3 * s2;
    half8_t r = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
    return r;
}

union BFrag {
    uint4 u;
    bf16x8_t v;
};

template <int BM, int BN>
constexpr size_t gemm_lds_bytes() {
    return 2 * ((size_t)BM * (G_CROW + G_SROW) + (size_t)BN * (G_CROW + G_SROW));
}

// 1-D grid of ceil(M / BM) * ceil(N / BN) workgroups of WMW x WNW waves, each wave TM x TN tiles of
// 32x32 (BM = 32 TM WMW, BN = 32 TN WNW); workgroup -> tile by TileMap.
template <int TM, int TN, int WMW, int WNW, bool VEC, typename OUT>
__global__ void __launch_bounds__(64 * WMW * WNW)
k_fp4_gemm_nt(Fp4Operand A, Fp4Operand B, int64_t K, const bf16_t* __restrict__ Aext,
              const bf16_t* __restrict__ Bext, int Ke, float alpha, OUT* __restrict__ C, int64_t ldc, TileMap tmap,
              int iters_per_split) {
    constexpr int BM = 32 * TM * WMW, BN = 32 * TN * WNW, NT = 64 * WMW * WNW;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // LDS: [buffer][codes A | codes B | scales A | scales B]
    constexpr int OFF_CB = BM * G_CROW, OFF_SA = (BM + BN) * G_CROW, OFF_SB = OFF_SA + BM * G_SROW,
                  BUF = OFF_SB + BN * G_SROW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int tile_m, tile_n;
    tile_coords(tmap, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int wm = (wave / WNW) * 32 * TM, wn = (wave % WNW) * 32 * TN;
    const int li = lane & 31, half = lane >> 5;

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // blockIdx.y = contraction split: stages [it0, it1); more than one split accumulates with fp32 atomics
    const int64_t niter_all = (K + G_KI - 1) / G_KI;
    const int64_t it0 = (int64_t)blockIdx.y * iters_per_split;
    const int64_t niter = it0 + iters_per_split < niter_all ? it0 + iters_per_split : niter_all;
    const bool split = gridDim.y > 1;
    StageRegs<BM * 4 / NT> ra;
    StageRegs<BN * 4 / NT> rb;
    ScaleRegs<(BM + BN + NT - 1) / NT> rs;
    stage_load<BM, NT, VEC>(A, m0, K, it0 * G_KI, ra, tid);
    stage_load<BN, NT, VEC>(B, n0, K, it0 * G_KI, rb, tid);
    scale_load<BM, BN, NT, VEC>(A, B, m0, n0, K, it0 * G_KI, rs, tid);
    stage_store<BM, NT>(ra, lds, tid);
    stage_store<BN, NT>(rb, lds + OFF_CB, tid);
    scale_store<BM, BN, NT>(rs, lds + OFF_SA, lds + OFF_SB, tid);
    __syncthreads();
    for (int64_t it = it0; it < niter; ++it) {
        const int cur = (int)((it - it0) & 1);
        const bool more = it + 1 < niter;
        if (more) {
            stage_load<BM, NT, VEC>(A, m0, K, (it + 1) * G_KI, ra, tid);
            stage_load<BN, NT, VEC>(B, n0, K, (it + 1) * G_KI, rb, tid);
            scale_load<BM, BN, NT, VEC>(A, B, m0, n0, K, (it + 1) * G_KI, rs, tid);
        }
        const uint8_t* bufc = lds + cur * BUF;
        uint8_t* bufn = lds + (cur ^ 1) * BUF;
        const uint8_t* ca = bufc + (wm + li) * G_CROW + 4 * half;
        const uint8_t* cb = bufc + OFF_CB + (wn + li) * G_CROW + 4 * half;
        const uint8_t* sa = bufc + OFF_SA + (wm + li) * G_SROW;
        const uint8_t* sb = bufc + OFF_SB + (wn + li) * G_SROW;
#pragma unroll
        for (int s = 0; s < G_KI / 16; ++s) {
            half8_t fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = dequant8(*reinterpret_cast<const uint32_t*>(ca + 32 * i * G_CROW + 8 * s),
                                 *reinterpret_cast<const uint32_t*>(sa + 32 * i * G_SROW + 4 * (s >> 1)), s & 1);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = dequant8(*reinterpret_cast<const uint32_t*>(cb + 32 * j * G_CROW + 8 * s),
                                 *reinterpret_cast<const uint32_t*>(sb + 32 * j * G_SROW + 4 * (s >> 1)), s & 1);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            stage_store<BM, NT>(ra, bufn, tid);
            stage_store<BN, NT>(rb, bufn + OFF_CB, tid);
            scale_store<BM, BN, NT>(rs, bufn + OFF_SA, bufn + OFF_SB, tid);
        }
        __syncthreads();
    }
    // low-rank terms: extra contraction columns in bf16, read straight from global memory
    if (Ke > 0 && blockIdx.y == 0) {
        for (int ks = 0; ks < Ke; ks += 16) {
            BFrag fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int64_t r = m0 + wm + 32 * i + li;
                if (r >= A.rows) r = A.rows - 1;
                fa[i].u = *reinterpret_cast<const uint4*>(Aext + r * Ke + ks + 8 * half);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int64_t r = n0 + wn + 32 * j + li;
                if (r >= B.rows) r = B.rows - 1;
                fb[j].u = *reinterpret_cast<const uint4*>(Bext + r * Ke + ks + 8 * half);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j], 0, 0, 0);
        }
    }
    // D layout 32x32: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int64_t c = n0 + wn + 32 * j + li;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int64_t r = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * half + (v & 3);
                if (r < A.rows && c < B.rows) {
                    if (split) atomic_out<OUT>(C + r * ldc + c, alpha * acc[i][j][v]);
                    else store_out<OUT>(C + r * ldc + c, alpha * acc[i][j][v]);
                }
            }
        }
}

// Software-pipelined variant: 256 x 256 tile, 4 waves of 128 x 128 (16 accumulator tiles per wave,
// one wave per SIMD).  Half as many code expansions per MFMA as the 8-wave kernel, so the matrix
// cores rather than the vector ALUs bound it -- provided the matrix pipe never drains:
//  * within a stage, the raw codes/scales of contraction step s+2 are read from LDS and step s+1
//    is expanded to fp16 between the 16 MFMAs of step s (register double-buffering, interleaving
//    pinned with sched_group_barrier);
//  * across stages, the next stage's global data is written to the other LDS buffer during steps
//    0-4 (each staging register is refilled with the stage after next right after its write), the
//    workgroup barrier sits at the start of step 6, and steps 6 and 7 already read and expand the
//    next stage's first two steps, so no MFMA waits for a barrier, an LDS round trip or a global load.
// The stage body is branch-free and the same for every stage (the last one stages and expands data
// that nobody uses), which keeps the whole loop one scheduling region.  Needs K % 128 == 0.
template <typename OUT>
__global__ void __launch_bounds__(256)
k_fp4_gemm_nt_pipe(Fp4Operand A, Fp4Operand B, int64_t K, const bf16_t* __restrict__ Aext,
                   const bf16_t* __restrict__ Bext, int Ke_all, float alpha, OUT* __restrict__ C, int64_t ldc, TileMap tmap,
                   int total_tiles, int tail_first, int tail_parts, float* __restrict__ partial) {
    constexpr int TM = 4, TN = 4, BM = 256, BN = 256, NT = 256, KS = G_KI / 16;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // LDS layout of a stage, chosen so that ONE 16-byte read per lane fetches the raw words of all four row
    // tiles of a wave (the wave issues an instruction only every ~9 clocks, so instructions, not bytes, count):
    // codes of an operand: planes (g = row / 128, step s, half) of 32 lanes x 4 tiles dwords,
    //   dword (g, s, half, l, i) = the 8 codes of row 128 g + 32 i + l at contraction 16 s + 8 half;
    // scales: planes (g, pair q of steps) of 32 x 4 dwords, dword (g, q, l, i) = the fp16 scales of blocks 2q, 2q+1.
    // A plane is 512 bytes, padded to 528 (planes of neighbouring 16-byte code segments then start in different banks).
    constexpr int PL = 528, CODES_OP = 2 * KS * 2 * PL, SC_OP = 2 * (KS / 2) * PL;
    constexpr int OFF_CB = CODES_OP, OFF_SA = 2 * CODES_OP, OFF_SB = OFF_SA + SC_OP, BUF = OFF_SB + SC_OP;
    static_assert(2 * BUF <= (int)gemm_lds_bytes<256, 256>(), "two stages fit the allocation");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // The tiles of the last, partly filled round of workgroups (launch positions tail_first ..) are cut along the
    // contraction into tail_parts workgroups each, which write fp32 partial tiles that a small kernel adds up:
    // the round then takes 1 / tail_parts of a tile's time instead of leaving most CUs idle for a whole one.
    int tile = (int)blockIdx.x, part = 0, parts = 1;
    if (tile >= tail_first) {
        const int idx = tile - tail_first;
        tile = tail_first + idx / tail_parts;
        part = idx - (tile - tail_first) * tail_parts;
        parts = tail_parts;
    }
    int tile_m, tile_n;
    tile_coords_of(tmap, tile, total_tiles, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
    const int li = lane & 31, half = lane >> 5;

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int niter_all = (int)(K / G_KI);
    const int it_begin = (int)((int64_t)part * niter_all / parts), it_end = (int)((int64_t)(part + 1) * niter_all / parts);
    const int niter = it_end - it_begin;                 // >= 1: the host keeps tail_parts <= K / 128
    const int Ke = part == 0 ? Ke_all : 0;               // the low-rank columns enter once
    // this thread's share of a stage: code vectors v = 0..3 of each operand (row tid/4 + 64 v, 16-byte
    // segment tid%4) and the scale rows tid (A) and tid (B); rows past the operand's end re-read its last row
    const uint8_t* pa[4];
    const uint8_t* pb[4];
    const int64_t cstride = K / 2, sstride = K / 16;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        int64_t ga = m0 + (tid >> 2) + 64 * v, gb = n0 + (tid >> 2) + 64 * v;
        if (ga >= A.rows) ga = A.rows - 1;
        if (gb >= B.rows) gb = B.rows - 1;
        pa[v] = A.codes + ga * cstride + 16 * (tid & 3) + (int64_t)it_begin * (G_KI / 2);
        pb[v] = B.codes + gb * cstride + 16 * (tid & 3) + (int64_t)it_begin * (G_KI / 2);
    }
    const uint8_t* psa;
    const uint8_t* psb;
    {
        int64_t ga = m0 + tid, gb = n0 + tid;
        if (ga >= A.rows) ga = A.rows - 1;
        if (gb >= B.rows) gb = B.rows - 1;
        psa = A.scales + ga * sstride + (int64_t)it_begin * (G_KI / 16);
        psb = B.scales + gb * sstride + (int64_t)it_begin * (G_KI / 16);
    }
    uint4 ra[4], rb[4];
    uint2 rsa, rsb;
    // st = stage index within this workgroup's range, clamped by the caller
    auto load_codes = [&](int st, int v) {
        ra[v] = *reinterpret_cast<const uint4*>(pa[v] + st * (G_KI / 2));
        rb[v] = *reinterpret_cast<const uint4*>(pb[v] + st * (G_KI / 2));
    };
    auto load_scales = [&](int st) {
        rsa = *reinterpret_cast<const uint2*>(psa + st * (G_KI / 16));
        rsb = *reinterpret_cast<const uint2*>(psb + st * (G_KI / 16));
    };
    auto load_stage = [&](int st) {
#pragma unroll
        for (int v = 0; v < 4; ++v) load_codes(st, v);
        load_scales(st);
    };
    // a 16-byte code vector = two steps (2 seg, 2 seg + 1) x two halves of one row: four dwords to four planes
    auto store_codes = [&](uint8_t* buf, int v) {
        const int e = tid + NT * v, row = e >> 2, seg = e & 3;
        const int off = (((row >> 7) * KS + 2 * seg) * 2) * PL + (row & 31) * 16 + ((row >> 5) & 3) * 4;
        uint8_t* da = buf + off;
        uint8_t* db = buf + OFF_CB + off;
        *reinterpret_cast<uint32_t*>(da) = ra[v].x;
        *reinterpret_cast<uint32_t*>(da + PL) = ra[v].y;
        *reinterpret_cast<uint32_t*>(da + 2 * PL) = ra[v].z;
        *reinterpret_cast<uint32_t*>(da + 3 * PL) = ra[v].w;
        *reinterpret_cast<uint32_t*>(db) = rb[v].x;
        *reinterpret_cast<uint32_t*>(db + PL) = rb[v].y;
        *reinterpret_cast<uint32_t*>(db + 2 * PL) = rb[v].z;
        *reinterpret_cast<uint32_t*>(db + 3 * PL) = rb[v].w;
    };
    auto store_scales = [&](uint8_t* buf) {
        const int off = ((tid >> 7) * (KS / 2)) * PL + (tid & 31) * 16 + ((tid >> 5) & 3) * 4;
        uint8_t* da = buf + OFF_SA + off;
        uint8_t* db = buf + OFF_SB + off;
        *reinterpret_cast<uint32_t*>(da) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsa.x, 1.0f, false));
        *reinterpret_cast<uint32_t*>(da + PL) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsa.x, 1.0f, true));
        *reinterpret_cast<uint32_t*>(da + 2 * PL) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsa.y, 1.0f, false));
        *reinterpret_cast<uint32_t*>(da + 3 * PL) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsa.y, 1.0f, true));
        *reinterpret_cast<uint32_t*>(db) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsb.x, 1.0f, false));
        *reinterpret_cast<uint32_t*>(db + PL) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsb.x, 1.0f, true));
        *reinterpret_cast<uint32_t*>(db + 2 * PL) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsb.y, 1.0f, false));
        *reinterpret_cast<uint32_t*>(db + 3 * PL) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(rsb.y, 1.0f, true));
    };
    load_stage(0);
#pragma unroll
    for (int v = 0; v < 4; ++v) store_codes(lds, v);
    store_scales(lds);
    __syncthreads();
    load_stage(niter > 1 ? 1 : 0);

    // per-lane byte offsets of this wave's planes inside a buffer (step 0 / pair 0)
    typedef uint32_t rawvec_t __attribute__((ext_vector_type(4)));
    const int oca = (((wave >> 1) * KS) * 2 + half) * PL + li * 16, ocb = OFF_CB + (((wave & 1) * KS) * 2 + half) * PL + li * 16;
    const int osa = OFF_SA + ((wave >> 1) * (KS / 2)) * PL + li * 16, osb = OFF_SB + ((wave & 1) * (KS / 2)) * PL + li * 16;
    uint32_t rawc[2][TM + TN], raws[2][TM + TN];
    half8_t frag[2][TM + TN];
    auto read_raw = [&](const uint8_t* buf, int s, int slot) {
        const rawvec_t ca = *reinterpret_cast<const rawvec_t*>(buf + oca + 2 * s * PL);
        const rawvec_t cb = *reinterpret_cast<const rawvec_t*>(buf + ocb + 2 * s * PL);
        const rawvec_t sa = *reinterpret_cast<const rawvec_t*>(buf + osa + (s >> 1) * PL);
        const rawvec_t sb = *reinterpret_cast<const rawvec_t*>(buf + osb + (s >> 1) * PL);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            rawc[slot][i] = ca[i];
            raws[slot][i] = sa[i];
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            rawc[slot][TM + j] = cb[j];
            raws[slot][TM + j] = sb[j];
        }
    };
    read_raw(lds, 0, 0);
    read_raw(lds, 1, 1);
#pragma unroll
    for (int t = 0; t < TM + TN; ++t) frag[0][t] = dequant8(rawc[0][t], raws[0][t], false);

#pragma unroll 1
    for (int it = 0; it < niter; ++it) {
        const uint8_t* bufc = lds + (it & 1) * BUF;
        uint8_t* bufn = lds + ((it & 1) ^ 1) * BUF;
        const int stn = it + 2 < niter ? it + 2 : niter - 1;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int c = s & 1, n = c ^ 1;
            if (s + 2 == KS) __syncthreads();     // next stage is in LDS, this stage's raw words are all read
            // expand step s+1 (its raw words arrived during step s-1), then refill that raw slot with s+2
#pragma unroll
            for (int t = 0; t < TM + TN; ++t) frag[n][t] = dequant8(rawc[n][t], raws[n][t], (s + 1) & 1);
            if (s + 2 < KS) read_raw(bufc, s + 2, c);
            else read_raw(bufn, s + 2 - KS, c);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(frag[c][i], frag[c][TM + j], acc[i][j], 0, 0, 0);
            // a staging register is refilled with the stage after next as soon as it has been written
            // to LDS, which gives every global load a whole stage to arrive
            if (s < 4) {
                store_codes(bufn, s);
                load_codes(stn, s);
            }
            if (s == 4) {
                store_scales(bufn);
                load_scales(stn);
            }
            // one MFMA, then its share of the other work: 4 of the 64 expansion ops, 1 of the 16 LDS reads,
            // and where the step has them an LDS write or a global load
#pragma unroll
            for (int m = 0; m < TM * TN; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (s <= 4) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                if (s <= 4 && m >= 8 && m < 10) {                      // the step's two global loads, after its LDS writes
                    __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
            }
        }
    }

    // low-rank terms: extra contraction columns in bf16, read straight from global memory, four steps
    // (64 columns) of fragments in flight at a time
    for (int ks = 0; ks < Ke; ks += 64) {
        BFrag fa[4][TM], fb[4][TN];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int kc = ks + 16 * u < Ke ? ks + 16 * u : ks;      // a short last batch re-reads its first step (unused)
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int64_t r = m0 + wm + 32 * i + li;
                if (r >= A.rows) r = A.rows - 1;
                fa[u][i].u = *reinterpret_cast<const uint4*>(Aext + r * Ke + kc + 8 * half);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int64_t r = n0 + wn + 32 * j + li;
                if (r >= B.rows) r = B.rows - 1;
                fb[u][j].u = *reinterpret_cast<const uint4*>(Bext + r * Ke + kc + 8 * half);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (ks + 16 * u < Ke) {                                   // uniform (kernel argument)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[u][i].v, fb[u][j].v, acc[i][j], 0, 0, 0);
            }
        }
    }
    // D layout 32x32: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
    if (parts > 1) {
        // partial tile, fp32, [tail tile][part][256][256]; bounds are applied when the parts are added up
        float* __restrict__ P = partial + ((size_t)(tile - tail_first) * parts + part) * (size_t)(BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    P[(wm + 32 * i + 4 * half + 8 * (v >> 2) + (v & 3)) * BN + wn + 32 * j + li] = alpha * acc[i][j][v];
        return;
    }
    const bool interior = m0 + BM <= A.rows && n0 + BN <= B.rows;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t c = n0 + wn + 32 * j + li;
            const int64_t rbase = m0 + wm + 32 * i + 4 * half;
            if (interior) {
                store_tile16<OUT>(C + rbase * ldc + c, ldc, acc[i][j], alpha);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t r = rbase + 8 * (v >> 2) + (v & 3);
                    if (r < A.rows && c < B.rows) store_out<OUT>(C + r * ldc + c, alpha * acc[i][j][v]);
                }
            }
        }
}

// adds the parts of the split tail tiles and writes them to C (see k_fp4_gemm_nt_pipe); one workgroup per 32 rows of a tile
template <typename OUT>
__global__ void __launch_bounds__(256)
k_gemm_tail_sum(const float* __restrict__ partial, int parts, int tail_first, int total_tiles, TileMap tmap, int64_t M,
                int64_t N, OUT* __restrict__ C, int64_t ldc) {
    const int tile = tail_first + (int)blockIdx.x / 8, rb = (int)blockIdx.x % 8;
    int tile_m, tile_n;
    tile_coords_of(tmap, tile, total_tiles, tile_m, tile_n);
    const float* __restrict__ P = partial + (size_t)(tile - tail_first) * parts * 65536;
    for (int e = threadIdx.x; e < 32 * 64; e += 256) {          // 32 rows x 64 float4
        const int r = 32 * rb + e / 64, c4 = (e % 64) * 4;
        float4 acc = *reinterpret_cast<const float4*>(P + r * 256 + c4);
        for (int p = 1; p < parts; ++p) {
            const float4 x = *reinterpret_cast<const float4*>(P + (size_t)p * 65536 + r * 256 + c4);
            acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
        }
        const int64_t gr = (int64_t)tile_m * 256 + r, gc = (int64_t)tile_n * 256 + c4;
        if (gr >= M) continue;
        const float v[4] = {acc.x, acc.y, acc.z, acc.w};
        for (int i = 0; i < 4; ++i)
            if (gc + i < N) store_out<OUT>(C + gr * ldc + gc + i, v[i]);
    }
}

// bytes of fp32 partial tiles the pipelined kernel wants for an M x N output (0: no tail split)
static size_t gemm_tail_bytes(int64_t M, int64_t N, int64_t K, int* parts_out = nullptr, int* tail_first_out = nullptr) {
    const int64_t tiles = ceil_div64(M, 256) * ceil_div64(N, 256);
    const int64_t tail = tiles % 256, niter = K / G_KI;
    int parts = tail > 0 ? (int)(256 / tail) : 1;
    if (parts > 4) parts = 4;
    if (parts > niter) parts = (int)niter;
    if (parts_out) *parts_out = parts;
    if (tail_first_out) *tail_first_out = (int)(tiles - tail);
    if (tail == 0 || parts < 2) return 0;
    return (size_t)tail * parts * 65536 * sizeof(float);
}

template <typename OUT>
int launch_gemm_pipe(hipStream_t s, const Fp4Operand& a, const Fp4Operand& b, int64_t K, const bf16_t* Aext,
                     const bf16_t* Bext, int Ke, float alpha, OUT* C, int64_t ldc, float* partial, size_t partial_bytes) {
    const int64_t tm = ceil_div64(a.rows, 256), tn = ceil_div64(b.rows, 256);
    if (tm * tn > 0x7FFFFFFF) return METIS_UNSUPPORTED;
    constexpr size_t lds = gemm_lds_bytes<256, 256>();
    const int total = (int)(tm * tn);
    int parts = 1, tail_first = total;
    const size_t want = gemm_tail_bytes(a.rows, b.rows, K, &parts, &tail_first);
    const bool split = want > 0 && partial && partial_bytes >= want;
    if (!split) { parts = 1; tail_first = total; }
    const int tail = total - tail_first;
    dim3 grid((unsigned)(tail_first + tail * parts));
    auto kern = k_fp4_gemm_nt_pipe<OUT>;
    static LdsLimitCache lds_set;
    if (!ensure_dyn_lds((const void*)kern, lds, lds_set)) return METIS_HIP_ERROR;
    const TileMap tmap = make_tile_map(tm, tn);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, tmap, total, tail_first, parts,
                       partial);
    METIS_LAUNCH_CHECK();
    if (split) {
        hipLaunchKernelGGL(k_gemm_tail_sum<OUT>, dim3((unsigned)(tail * 8)), dim3(256), 0, s, partial, parts, tail_first, total,
                           tmap, a.rows, b.rows, C, ldc);
        METIS_LAUNCH_CHECK();
    }
    return METIS_OK;
}

template <int TM, int TN, int WMW, int WNW, typename OUT>
int launch_gemm_tile(hipStream_t s, const Fp4Operand& a, const Fp4Operand& b, int64_t K, bool vec, const bf16_t* Aext,
                     const bf16_t* Bext, int Ke, float alpha, OUT* C, int64_t ldc, int ksplit = 1) {
    constexpr int BM = 32 * TM * WMW, BN = 32 * TN * WNW, NT = 64 * WMW * WNW;
    static_assert(BM * 4 >= NT && BN * 4 >= NT, "every thread stages at least one code vector");
    const int64_t tm = ceil_div64(a.rows, BM), tn = ceil_div64(b.rows, BN);
    if (tm * tn > 0x7FFFFFFF) return METIS_UNSUPPORTED;
    constexpr size_t lds = gemm_lds_bytes<BM, BN>();
    const int64_t niter = ceil_div64(K, G_KI);
    if (ksplit < 1 || sizeof(OUT) != 4) ksplit = 1;
    const int ips = (int)ceil_div64(niter, ksplit);
    dim3 grid((unsigned)(tm * tn), (unsigned)ceil_div64(niter, ips));
    if (vec) {
        auto kern = k_fp4_gemm_nt<TM, TN, WMW, WNW, true, OUT>;
        static LdsLimitCache lds_set;
        if (!ensure_dyn_lds((const void*)kern, lds, lds_set)) return METIS_HIP_ERROR;
        hipLaunchKernelGGL(kern, grid, dim3(NT), lds, s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, make_tile_map(tm, tn), ips);
    } else {
        auto kern = k_fp4_gemm_nt<TM, TN, WMW, WNW, false, OUT>;
        static LdsLimitCache lds_set;
        if (!ensure_dyn_lds((const void*)kern, lds, lds_set)) return METIS_HIP_ERROR;
        hipLaunchKernelGGL(kern, grid, dim3(NT), lds, s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, make_tile_map(tm, tn), ips);
    }
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

// ksplit > 1: C (fp32, zero on entry) accumulates the contraction splits with atomics
template <typename OUT>
int launch_gemm(hipStream_t s, const metis_fp4& A, const metis_fp4& B, const bf16_t* Aext, const bf16_t* Bext, int Ke,
                float alpha, OUT* C, int64_t ldc, int ksplit = 1, float* partial = nullptr, size_t partial_bytes = 0) {
    const int64_t M = A.rows, N = B.rows, K = A.cols;
    Fp4Operand a = {A.codes, A.scales, M}, b = {B.codes, B.scales, N};
    const bool vec = (K % G_KI) == 0 && reinterpret_cast<uintptr_t>(A.codes) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(B.codes) % 16 == 0 && reinterpret_cast<uintptr_t>(A.scales) % 8 == 0 &&
                     reinterpret_cast<uintptr_t>(B.scales) % 8 == 0;
    if (M >= 1024 && N >= 1024) {
        // 256x256 tile, 4 waves of 128x128, software-pipelined (needs whole 128-deep stages and aligned rows); the
        // tiles of a partly filled last round are cut along the contraction when the caller brought room for the parts
        const size_t tail_need = gemm_tail_bytes(M, N, K);
        const bool can_split = tail_need > 0 && partial && partial_bytes >= tail_need;
        if (vec && (can_split || ceil_div64(M, 256) * ceil_div64(N, 256) > 128))
            return launch_gemm_pipe<OUT>(s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, partial, partial_bytes);
        // an output of at most 128 tiles of 256 x 256 would leave half the CUs without work: 128 x 128 tiles
        // (four times as many workgroups, each less efficient) finish sooner
        if (ceil_div64(M, 256) * ceil_div64(N, 256) <= 128 && ksplit <= 1)
            return launch_gemm_tile<2, 2, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc, 1);
        if (vec) return launch_gemm_pipe<OUT>(s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, partial, partial_bytes);
        // otherwise 8 waves of 128x64 with bounds-checked staging
        return launch_gemm_tile<4, 2, 2, 4, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc);
    }
    if (N > 64 && M > 64) return launch_gemm_tile<2, 2, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc, ksplit);
    if (N <= 64) return launch_gemm_tile<2, 1, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc, ksplit);
    return launch_gemm_tile<1, 2, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc, ksplit);
}

// value of one FP4 element without the tensor scale: grid[code] * e4m3(scale)
__device__ __forceinline__ float fp4_elem_nog(const uint8_t* codes, const uint8_t* scales, int64_t cols, int64_t r,
                                              int64_t c) {
    uint32_t byte = codes[r * (cols / 2) + c / 2];
    uint32_t nib = (c & 1) ? (byte >> 4) : (byte & 15u);
    const float grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    float v = grid[nib & 7u] * e4m3_decode(scales[r * (cols / 16) + c / 16]);
    return (nib & 8u) ? -v : v;
}

// Extra contraction columns for Abar Bbar^T (see file header).  Column layout, Kep = padded kb+ka:
//   Aext[m, 0:kb]     = (T1[m,:] + sum_j Ua[m,j] Sa_j Mk[j,:]) * Sb * gUb / (gRa gRb)
//   Aext[m, kb:kb+ka] = Ua[m,:] without its tensor scale (exact in bf16)
//   Bext[n, 0:kb]     = Ub[n,:] without its tensor scale (exact in bf16)
//   Bext[n, kb:kb+ka] = E2[n,:] * Sa * gUa / (gRa gRb)
// Blocks [0, ceil(Ma/16)) build 16 rows of Aext each: the dequantized factor rows U_a S_a and the small
// matrix Mk sit in LDS, so the k_a-term sum of the first kb columns reads global memory once.  The
// remaining blocks build 16 rows of Bext each the same way.  (16 rows: several workgroups per CU; with 64
// the 8192 + 4096 rows of a layer gave fewer workgroups than CUs and the kernel took three times as long.)
#define AX_ROWS 16
__global__ void __launch_bounds__(256)
k_assemble_ext(int64_t Ma, int64_t Nb, int ka, int kb, int Kep, const float* __restrict__ T1,
               const float* __restrict__ Mk, const float* __restrict__ E2,
               const uint8_t* __restrict__ ua_codes, const uint8_t* __restrict__ ua_scales, float g_ua,
               const float* __restrict__ Sa, const uint8_t* __restrict__ ub_codes,
               const uint8_t* __restrict__ ub_scales, float g_ub, const float* __restrict__ Sb,
               float inv_grr, bf16_t* __restrict__ Aext, bf16_t* __restrict__ Bext) {
    extern __shared__ float ax_sm[];
    const int nblk_a = (int)((Ma + AX_ROWS - 1) / AX_ROWS);
    const int tid = threadIdx.x;
    if ((int)blockIdx.x < nblk_a) {
        float* ua = ax_sm;                          // [AX_ROWS][ka + 1]: factor entries without tensor scale
        float* mk = ax_sm + AX_ROWS * (ka + 1);     // [ka][kb]
        const int64_t r0 = (int64_t)blockIdx.x * AX_ROWS;
        for (int e = tid; e < AX_ROWS * ka; e += 256) {
            const int j = e / AX_ROWS, rr = e - j * AX_ROWS;      // consecutive threads walk along a stored factor row
            const int64_t row = r0 + rr;
            ua[rr * (ka + 1) + j] = row < Ma ? fp4_elem_nog(ua_codes, ua_scales, Ma, j, row) : 0.0f;
        }
        for (int e = tid; e < ka * kb; e += 256) mk[e] = Mk[e] * g_ua * Sa[e / kb];
        __syncthreads();
        for (int e = tid; e < AX_ROWS * Kep; e += 256) {
            const int rr = e / Kep, c = e - rr * Kep;
            const int64_t row = r0 + rr;
            if (row >= Ma) continue;
            float v = 0.0f;
            if (c < kb) {
                float acc = T1[row * kb + c];
                for (int j = 0; j < ka; ++j) acc += ua[rr * (ka + 1) + j] * mk[j * kb + c];
                v = acc * Sb[c] * g_ub * inv_grr;
            } else if (c < kb + ka) {
                v = ua[rr * (ka + 1) + (c - kb)];
            }
            Aext[row * Kep + c] = f32_to_bf16_rne(v);
        }
        return;
    }
    // Bext: 16 rows per block; the stored factor rows of U_b are decoded along their contiguous axis into LDS
    float* ub = ax_sm;                              // [AX_ROWS][kb + 1]
    const int64_t r0 = ((int64_t)blockIdx.x - nblk_a) * AX_ROWS;
    for (int e = tid; e < AX_ROWS * kb; e += 256) {
        const int j = e / AX_ROWS, rr = e - j * AX_ROWS;
        const int64_t row = r0 + rr;
        ub[rr * (kb + 1) + j] = row < Nb ? fp4_elem_nog(ub_codes, ub_scales, Nb, j, row) : 0.0f;
    }
    __syncthreads();
    for (int e = tid; e < AX_ROWS * Kep; e += 256) {
        const int rr = e / Kep, c = e - rr * Kep;
        const int64_t row = r0 + rr;
        if (row >= Nb) continue;
        float v = 0.0f;
        if (c < kb) {
            v = ub[rr * (kb + 1) + c];
        } else if (c < kb + ka) {
            const int j = c - kb;
            v = E2[row * ka + j] * Sa[j] * g_ua * inv_grr;
        }
        Bext[row * Kep + c] = f32_to_bf16_rne(v);
    }
}

__global__ void k_zero_f32(float* __restrict__ p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, st = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += st) p[i] = 0.0f;
}

struct NtOperand {            // one side of Abar Bbar^T: Abar = U diag(S) V^T + R, R [rows, Kc]
    metis_fp4 R, Ut, Vt;      // Ut [k, rows], Vt [k, Kc]
    const float* S;
    int k;
};

struct LinWs {
    size_t off_t1, off_mk, off_e2, off_aext, off_bext, off_tail, tail_bytes, total;
    int Kep;
};

LinWs lin_layout(int64_t Ma, int64_t Nb, int ka, int kb, int64_t Kc) {
    LinWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    w.Kep = (ka + kb + 15) / 16 * 16;
    w.off_t1 = take((size_t)Ma * (kb > 0 ? kb : 1) * 4);
    w.off_mk = take((size_t)(ka > 0 ? ka : 1) * (kb > 0 ? kb : 1) * 4);
    w.off_e2 = take((size_t)Nb * (ka > 0 ? ka : 1) * 4);
    w.off_aext = take((size_t)Ma * (w.Kep > 0 ? w.Kep : 16) * 2);
    w.off_bext = take((size_t)Nb * (w.Kep > 0 ? w.Kep : 16) * 2);
    w.tail_bytes = (Ma >= 1024 && Nb >= 1024 && Kc % G_KI == 0) ? gemm_tail_bytes(Ma, Nb, Kc) : 0;
    w.off_tail = take(w.tail_bytes);
    w.total = o;
    return w;
}

bool fp4_valid(const metis_fp4& f) { return f.codes && f.scales && f.rows > 0 && f.cols > 0 && f.cols % 16 == 0; }

int linear_nt(hipStream_t s, const NtOperand& a, const NtOperand& b, metis_mat* out, void* workspace,
              size_t workspace_bytes) {
    if (!out || !out->ptr) return METIS_INVALID_ARG;
    if (!fp4_valid(a.R) || !fp4_valid(b.R) || a.R.cols != b.R.cols) return METIS_BAD_SHAPE;
    const int64_t Ma = a.R.rows, Nb = b.R.rows, Kc = a.R.cols;
    if (out->rows != Ma || out->cols != Nb || out->ld < Nb) return METIS_BAD_SHAPE;
    if (out->dtype != METIS_BF16 && out->dtype != METIS_F32) return METIS_INVALID_ARG;
    const int ka = a.k, kb = b.k;
    if (ka < 0 || kb < 0 || ka > 128 || kb > 128) return METIS_UNSUPPORTED;
    if (ka > 0 && (!a.S || !fp4_valid(a.Ut) || !fp4_valid(a.Vt) || a.Ut.rows != ka || a.Ut.cols != Ma ||
                   a.Vt.rows != ka || a.Vt.cols != Kc)) return METIS_BAD_SHAPE;
    if (kb > 0 && (!b.S || !fp4_valid(b.Ut) || !fp4_valid(b.Vt) || b.Ut.rows != kb || b.Ut.cols != Nb ||
                   b.Vt.rows != kb || b.Vt.cols != Kc)) return METIS_BAD_SHAPE;
    const float grr = a.R.tscale * b.R.tscale;
    int Ke = 0;
    const bf16_t *Aext = nullptr, *Bext = nullptr;
    int st;
    if (ka > 0 || kb > 0) {
        const LinWs w = lin_layout(Ma, Nb, ka, kb, Kc);
        if (!workspace || workspace_bytes < w.off_tail) return METIS_WORKSPACE_TOO_SMALL;   // the tail region is optional
        if (reinterpret_cast<uintptr_t>(workspace) % 16) return METIS_INVALID_ARG;
        char* ws = (char*)workspace;
        float* T1 = (float*)(ws + w.off_t1);
        float* Mk = (float*)(ws + w.off_mk);
        float* E2 = (float*)(ws + w.off_e2);
        bf16_t* ae = (bf16_t*)(ws + w.off_aext);
        bf16_t* be = (bf16_t*)(ws + w.off_bext);
        // skinny products: few output tiles, long contraction -> split it over workgroups
        auto splits = [&](int64_t rows, int64_t cols) {
            int64_t tiles = ceil_div64(rows, 128) * ceil_div64(cols, 64), iters = ceil_div64(Kc, G_KI);
            int64_t want = ceil_div64(256, tiles), maxs = iters / 2 > 0 ? iters / 2 : 1;
            return (int)(want < maxs ? want : maxs);
        };
        // (the k_a x k_b product Mk is a single output tile: without a split one workgroup would walk the whole
        // contraction alone, ~100 us at 14336 columns)
        const int s1 = kb > 0 ? splits(Ma, kb) : 1, s2 = ka > 0 ? splits(Nb, ka) : 1;
        const int s3 = ka > 0 && kb > 0 ? splits(ka, kb) : 1;
        if (s1 > 1 || s2 > 1 || s3 > 1) {     // T1, Mk, E2 are contiguous at the start of the workspace
            hipLaunchKernelGGL(k_zero_f32, dim3(256), dim3(256), 0, s, (float*)ws, w.off_aext / 4);
            METIS_LAUNCH_CHECK();
        }
        if (kb > 0 && (st = launch_gemm<float>(s, a.R, b.Vt, nullptr, nullptr, 0, a.R.tscale * b.Vt.tscale, T1, kb, s1)))
            return st;
        if (ka > 0 && (st = launch_gemm<float>(s, b.R, a.Vt, nullptr, nullptr, 0, b.R.tscale * a.Vt.tscale, E2, ka, s2)))
            return st;
        if (ka > 0 && kb > 0 &&
            (st = launch_gemm<float>(s, a.Vt, b.Vt, nullptr, nullptr, 0, a.Vt.tscale * b.Vt.tscale, Mk, kb, s3)))
            return st;
        const int64_t nblk = ceil_div64(Ma, AX_ROWS) + ceil_div64(Nb, AX_ROWS);
        const size_t ax_lds = ((size_t)AX_ROWS * ((ka > kb ? ka : kb) + 1) + (size_t)ka * kb) * sizeof(float);
        static LdsLimitCache ax_set;
        if (ax_lds > 48 * 1024 && !ensure_dyn_lds((const void*)k_assemble_ext, ax_lds, ax_set)) return METIS_HIP_ERROR;
        hipLaunchKernelGGL(k_assemble_ext, dim3((unsigned)nblk), dim3(256), ax_lds, s, Ma, Nb, ka, kb, w.Kep,
                           T1, Mk, E2, a.Ut.codes, a.Ut.scales, ka > 0 ? a.Ut.tscale : 1.0f, a.S, b.Ut.codes,
                           b.Ut.scales, kb > 0 ? b.Ut.tscale : 1.0f, b.S, 1.0f / grr, ae, be);
        METIS_LAUNCH_CHECK();
        Ke = w.Kep;
        Aext = ae;
        Bext = be;
    }
    // room for the partial tiles of a split last round, when the workspace has it
    float* partial = nullptr;
    size_t partial_bytes = 0;
    {
        const LinWs w = lin_layout(Ma, Nb, ka, kb, Kc);
        if (w.tail_bytes > 0 && workspace && workspace_bytes >= w.total && reinterpret_cast<uintptr_t>(workspace) % 16 == 0) {
            partial = (float*)((char*)workspace + w.off_tail);
            partial_bytes = w.tail_bytes;
        }
    }
    const int pi = metis_prof_begin(METIS_PROF_GEMM, s);
    if (out->dtype == METIS_BF16)
        st = launch_gemm<bf16_t>(s, a.R, b.R, Aext, Bext, Ke, grr, (bf16_t*)out->ptr, out->ld, 1, partial, partial_bytes);
    else
        st = launch_gemm<float>(s, a.R, b.R, Aext, Bext, Ke, grr, (float*)out->ptr, out->ld, 1, partial, partial_bytes);
    metis_prof_end(METIS_PROF_GEMM, pi, s);
    return st;
}

NtOperand nt(const metis_fp4& R, const metis_fp4& Ut, const metis_fp4& Vt, const float* S, int k) {
    NtOperand o;
    o.R = R; o.Ut = Ut; o.Vt = Vt; o.S = S; o.k = k;
    return o;
}

}  // namespace

extern "C" size_t metis_linear_workspace_bytes(int64_t L, int64_t N, int64_t K, int k) {
    if (L < 1 || N < 1 || K < 1 || k < 0) return 0;
    size_t a = lin_layout(L, N, k, k, K).total, b = lin_layout(L, K, k, k, N).total, c = lin_layout(N, K, k, k, L).total;
    return a > b ? (a > c ? a : c) : (b > c ? b : c);
}

// Y[L,N] = Xbar Wbar^T: contraction over K
extern "C" int metis_fp4_linear_fwd(void* stream, const metis_split* X, const metis_split* W, metis_mat* Y,
                                    void* workspace, size_t workspace_bytes) {
    if (!X || !W) return METIS_INVALID_ARG;
    return linear_nt((hipStream_t)stream, nt(X->R, X->Ut, X->Vt, X->S, X->k), nt(W->R, W->Ut, W->Vt, W->S, W->k), Y,
                     workspace, workspace_bytes);
}

// dX[L,K] = Gbar Wbar: contraction over N; Wbar^T [K,N] = Vw Sw Uw^T + Rw^T
extern "C" int metis_fp4_linear_dgrad(void* stream, const metis_split* G, const metis_split* W, metis_mat* dX,
                                      void* workspace, size_t workspace_bytes) {
    if (!G || !W) return METIS_INVALID_ARG;
    return linear_nt((hipStream_t)stream, nt(G->R, G->Ut, G->Vt, G->S, G->k), nt(W->Rt, W->Vt, W->Ut, W->S, W->k), dX,
                     workspace, workspace_bytes);
}

// dW[N,K] = Gbar^T Xbar: contraction over L; Gbar^T [N,L] = Vg Sg Ug^T + Rg^T, Xbar^T [K,L] likewise
extern "C" int metis_fp4_linear_wgrad(void* stream, const metis_split* G, const metis_split* X, metis_mat* dW,
                                      void* workspace, size_t workspace_bytes) {
    if (!G || !X) return METIS_INVALID_ARG;
    return linear_nt((hipStream_t)stream, nt(G->Rt, G->Vt, G->Ut, G->S, G->k), nt(X->Rt, X->Vt, X->Ut, X->S, X->k), dW,
                     workspace, workspace_bytes);
}
