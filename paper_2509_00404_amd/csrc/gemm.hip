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

// The extra contraction columns (bf16, Ke % 16 == 0) are stored in the order the matrix instruction wants them:
// element (row r, column c) at (((r/32 * Ke/16 + c/16) * 2 + (c%16)/8) * 32 + r%32) * 8 + c%8, rows padded to a
// multiple of 32 -- the 64 lanes' 16-byte operands of one 32-row block and 16-column step are 1 KiB of
// consecutive memory (read row-major, one such load touched 32 cache lines and used a quarter of each).
__host__ __device__ __forceinline__ int64_t ext_chunk(int64_t row_block, int step, int half, int li, int nsteps) {
    return (((row_block * nsteps + step) * 2 + half) * 32 + li) * 8;
}

// One output tile by a workgroup of WMW x WNW waves, each wave TM x TN tiles of 32x32 (BM = 32 TM WMW,
// BN = 32 TN WNW), over the contraction stages [it0, niter).
template <int TM, int TN, int WMW, int WNW, bool VEC, typename OUT>
__device__ __forceinline__ void
gemm_nt_tile(const Fp4Operand& A, const Fp4Operand& B, int64_t K, const bf16_t* __restrict__ Aext,
             const bf16_t* __restrict__ Bext, int Ke, float alpha, OUT* __restrict__ C, int64_t ldc, int tile_m, int tile_n,
             int64_t it0, int64_t niter) {
    constexpr int BM = 32 * TM * WMW, BN = 32 * TN * WNW, NT = 64 * WMW * WNW;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // LDS: [buffer][codes A | codes B | scales A | scales B]
    constexpr int OFF_CB = BM * G_CROW, OFF_SA = (BM + BN) * G_CROW, OFF_SB = OFF_SA + BM * G_SROW,
                  BUF = OFF_SB + BN * G_SROW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    // this workgroup's stages of the contraction: [it0, niter)
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
    if (Ke > 0) {
        const int nks = Ke >> 4;
        const int64_t rba_max = (A.rows + 31) / 32 - 1, rbb_max = (B.rows + 31) / 32 - 1;
        for (int ks = 0; ks < nks; ++ks) {
            BFrag fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int64_t rb = (m0 + wm) / 32 + i;
                if (rb > rba_max) rb = rba_max;
                fa[i].u = *reinterpret_cast<const uint4*>(Aext + ext_chunk(rb, ks, half, li, nks));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int64_t rb = (n0 + wn) / 32 + j;
                if (rb > rbb_max) rb = rbb_max;
                fb[j].u = *reinterpret_cast<const uint4*>(Bext + ext_chunk(rb, ks, half, li, nks));
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
                if (r < A.rows && c < B.rows) store_out<OUT>(C + r * ldc + c, alpha * acc[i][j][v]);
            }
        }
}

// 1-D grid of ceil(M / BM) * ceil(N / BN) workgroups; workgroup -> tile by TileMap
template <int TM, int TN, int WMW, int WNW, bool VEC, typename OUT>
__global__ void __launch_bounds__(64 * WMW * WNW)
k_fp4_gemm_nt(Fp4Operand A, Fp4Operand B, int64_t K, const bf16_t* __restrict__ Aext,
              const bf16_t* __restrict__ Bext, int Ke, float alpha, OUT* __restrict__ C, int64_t ldc, TileMap tmap) {
    int tile_m, tile_n;
    tile_coords(tmap, tile_m, tile_n);
    gemm_nt_tile<TM, TN, WMW, WNW, VEC, OUT>(A, B, K, Aext, Bext, Ke, alpha, C, ldc, tile_m, tile_n, 0, (K + G_KI - 1) / G_KI);
}

// Up to three skinny products in one launch, each cut along the contraction into `splits` parts that are written
// side by side (part z of problem q at P + z rows_a rows_b, plain stores): the consumer adds the parts in a fixed
// order, so the result does not depend on the order in which workgroups finish.  128 x 64 tiles, 4 waves.
struct SkinnyProblem {
    Fp4Operand A, B;         // C = alpha A B^T, [A.rows, B.rows]
    float alpha;
    float* P;
    int tiles_n, tiles;      // tiles along B.rows, tiles in all
    int ips;                 // stages per part
    int first;               // first workgroup of this problem
};
struct SkinnyBatch {
    SkinnyProblem p[3];
    int count;
};

template <bool VEC>
__global__ void __launch_bounds__(256)
k_fp4_skinny_batch(SkinnyBatch batch, int64_t K) {
    int q = 0;
#pragma unroll
    for (int i = 1; i < 3; ++i)
        if (i < batch.count && (int)blockIdx.x >= batch.p[i].first) q = i;
    SkinnyProblem pr = batch.p[0];
    if (q == 1) pr = batch.p[1];
    if (q == 2) pr = batch.p[2];
    const int local = (int)blockIdx.x - pr.first, z = local / pr.tiles, t = local - z * pr.tiles;
    const int64_t niter_all = (K + G_KI - 1) / G_KI;
    const int64_t it0 = (int64_t)z * pr.ips;
    const int64_t niter = it0 + pr.ips < niter_all ? it0 + pr.ips : niter_all;
    gemm_nt_tile<2, 1, 2, 2, VEC, float>(pr.A, pr.B, K, nullptr, nullptr, 0, pr.alpha,
                                         pr.P + (size_t)z * pr.A.rows * pr.B.rows, pr.B.rows, t / pr.tiles_n, t % pr.tiles_n,
                                         it0, niter);
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
                   int total_tiles, int tail_first, int tail_parts, float* __restrict__ partial, int total_items) {
    constexpr int TM = 4, TN = 4, BM = 256, BN = 256, NT = 256, KS = G_KI / 16;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // LDS layout of a stage, chosen so that ONE 16-byte read per lane fetches the raw words of all four row
    // tiles of a wave (a lone wave per SIMD is bound by the number of instructions it issues, so instructions, not bytes, count):
    // codes of an operand: planes (g = row / 128, step s, half) of 32 lanes x 4 tiles dwords,
    //   dword (g, s, half, l, i) = the 8 codes of row 128 g + 32 i + l at contraction 16 s + 8 half;
    // scales: planes (g, pair q of steps) of 32 x 4 dwords, dword (g, q, l, i) = the fp16 scales of blocks 2q, 2q+1.
    // A plane is 512 bytes, padded to 528 (planes of neighbouring 16-byte code segments then start in different banks).
    constexpr int PL = 528, CODES_OP = 2 * KS * 2 * PL, SC_OP = 2 * (KS / 2) * PL;
    constexpr int OFF_CB = CODES_OP, OFF_SA = 2 * CODES_OP, OFF_SB = OFF_SA + SC_OP, BUF = OFF_SB + SC_OP;
    static_assert(2 * BUF <= (int)gemm_lds_bytes<256, 256>(), "two stages fit the allocation");
    // The tiles of the last, partly filled round of workgroups (launch positions tail_first ..) are cut along the
    // contraction into tail_parts workgroups each, which write fp32 partial tiles that a small kernel adds up:
    // the round then takes 1 / tail_parts of a tile's time instead of leaving most CUs idle for a whole one.
    // A workgroup walks the launch positions blockIdx.x, blockIdx.x + gridDim.x, ... itself (one workgroup per CU):
    // the stores of a finished tile drain while the next tile's contraction runs, and no CU waits for a dispatch.
    // (No barrier between tiles is needed: after the barrier in the last stage every LDS read fetches words
    // that are never used, and the next tile's first reads come after the barrier of its own first stage.)
    for (int pos = (int)blockIdx.x; pos < total_items; pos += (int)gridDim.x) {
    // (the thread index passes through an empty asm in every round, so that nothing derived from it counts as
    // loop-invariant: hoisted out of this loop, the per-lane offsets of all phases would be live at once and spill)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = tid >> 6;
    int tile = pos, part = 0, parts = 1;
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
    // (in the order the stage loop issues and consumes them -- scheduling fences keep it: the wait in front of the
    // loop's first LDS write is computed over both ways into the loop, and with this order reversed here it has to
    // wait for every load in flight instead of the oldest pair)
    {
        const int st1 = niter > 1 ? 1 : 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            load_codes(st1, v);
            __builtin_amdgcn_sched_barrier(0);
        }
        load_scales(st1);
        __builtin_amdgcn_sched_barrier(0);
    }

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
            // one MFMA, then its share of the other work: 4 of the 64 expansion ops (5 early in a staging step: the
            // address arithmetic of the LDS writes and the loads needs slots too, or it drifts to the end of the
            // stage and takes the loads with it), 1 of the 16 LDS reads, and where the step has them an LDS write
            // or a global load.  Four load slots per staging step, right behind its LDS writes: with two, half of
            // the loads were issued a third of a stage later, and a load has to be back one stage after its issue.
#pragma unroll
            for (int m = 0; m < TM * TN; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (s <= 4 && m < 12) __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                else __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (s <= 4) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                if (s <= 4 && m >= 6 && m < 10) {                      // the step's global loads, after its LDS writes
                    __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
            }
        }
    }

    // low-rank terms: extra contraction columns in bf16, read straight from global memory; three steps of
    // fragments in flight, a step's registers are refilled with the step three ahead as soon as it is used
    const int nks = Ke >> 4;
    if (nks > 0) {
        const bf16_t* ea[TM];
        const bf16_t* eb[TN];
        const int64_t rba_max = (A.rows + 31) / 32 - 1, rbb_max = (B.rows + 31) / 32 - 1;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int64_t rb = (m0 + wm) / 32 + i;
            if (rb > rba_max) rb = rba_max;
            ea[i] = Aext + ext_chunk(rb, 0, half, li, nks);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int64_t rb = (n0 + wn) / 32 + j;
            if (rb > rbb_max) rb = rbb_max;
            eb[j] = Bext + ext_chunk(rb, 0, half, li, nks);
        }
        constexpr int EXT_DEPTH = 3;      // four fit the registers only with spills, and run no faster
        BFrag f[EXT_DEPTH][TM + TN];
        auto load_ext = [&](int step, int slot) {
#pragma unroll
            for (int i = 0; i < TM; ++i) f[slot][i].u = *reinterpret_cast<const uint4*>(ea[i] + step * 512);
#pragma unroll
            for (int j = 0; j < TN; ++j) f[slot][TM + j].u = *reinterpret_cast<const uint4*>(eb[j] + step * 512);
        };
#pragma unroll
        for (int u = 0; u < EXT_DEPTH; ++u)
            if (u < nks) load_ext(u, u);
        for (int ks = 0; ks < nks; ks += EXT_DEPTH) {
#pragma unroll
            for (int u = 0; u < EXT_DEPTH; ++u) {
                if (ks + u < nks) {                                   // uniform (kernel argument)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[u][i].v, f[u][TM + j].v, acc[i][j], 0, 0, 0);
                    if (ks + u + EXT_DEPTH < nks) load_ext(ks + u + EXT_DEPTH, u);
                }
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
        continue;
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
    const int items = tail_first + tail * parts;
    const int cus = device_cu_count();
    if (cus < 1) return METIS_HIP_ERROR;
    dim3 grid((unsigned)(items < cus ? items : cus));
    auto kern = k_fp4_gemm_nt_pipe<OUT>;
    static LdsLimitCache lds_set;
    if (!ensure_dyn_lds((const void*)kern, lds, lds_set)) return METIS_HIP_ERROR;
    const TileMap tmap = make_tile_map(tm, tn);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, tmap, total, tail_first, parts,
                       partial, items);
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
                     const bf16_t* Bext, int Ke, float alpha, OUT* C, int64_t ldc) {
    constexpr int BM = 32 * TM * WMW, BN = 32 * TN * WNW, NT = 64 * WMW * WNW;
    static_assert(BM * 4 >= NT && BN * 4 >= NT, "every thread stages at least one code vector");
    const int64_t tm = ceil_div64(a.rows, BM), tn = ceil_div64(b.rows, BN);
    if (tm * tn > 0x7FFFFFFF) return METIS_UNSUPPORTED;
    constexpr size_t lds = gemm_lds_bytes<BM, BN>();
    dim3 grid((unsigned)(tm * tn));
    if (vec) {
        auto kern = k_fp4_gemm_nt<TM, TN, WMW, WNW, true, OUT>;
        static LdsLimitCache lds_set;
        if (!ensure_dyn_lds((const void*)kern, lds, lds_set)) return METIS_HIP_ERROR;
        hipLaunchKernelGGL(kern, grid, dim3(NT), lds, s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, make_tile_map(tm, tn));
    } else {
        auto kern = k_fp4_gemm_nt<TM, TN, WMW, WNW, false, OUT>;
        static LdsLimitCache lds_set;
        if (!ensure_dyn_lds((const void*)kern, lds, lds_set)) return METIS_HIP_ERROR;
        hipLaunchKernelGGL(kern, grid, dim3(NT), lds, s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, make_tile_map(tm, tn));
    }
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

template <typename OUT>
int launch_gemm(hipStream_t s, const metis_fp4& A, const metis_fp4& B, const bf16_t* Aext, const bf16_t* Bext, int Ke,
                float alpha, OUT* C, int64_t ldc, float* partial = nullptr, size_t partial_bytes = 0) {
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
        if (ceil_div64(M, 256) * ceil_div64(N, 256) <= 128)
            return launch_gemm_tile<2, 2, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc);
        if (vec) return launch_gemm_pipe<OUT>(s, a, b, K, Aext, Bext, Ke, alpha, C, ldc, partial, partial_bytes);
        // otherwise 8 waves of 128x64 with bounds-checked staging
        return launch_gemm_tile<4, 2, 2, 4, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc);
    }
    if (N > 64 && M > 64) return launch_gemm_tile<2, 2, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc);
    if (N <= 64) return launch_gemm_tile<2, 1, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc);
    return launch_gemm_tile<1, 2, 2, 2, OUT>(s, a, b, K, vec, Aext, Bext, Ke, alpha, C, ldc);
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
// T1, E2 and Mk arrive as n1, n2, n3 contraction parts that are added here in ascending order.
// Blocks [0, ceil(Ma/32)) build 32 rows of Aext each: the dequantized factor rows U_a and the small matrix
// Sa Mk sit in LDS; thread (row t/8, column group t%8) owns the columns 64 h + 8 (t%8) + 0..7 of its row.  The
// remaining blocks build 32 rows of Bext each the same way.  The kernel moves little data and is bound by
// load latency, so every global load of a thread is issued before the first use: parts are read four at a time.
#define AX_ROWS 32

// acc[i] += sum over parts p < n of base[p * pstride + off + i], i < cnt <= 8 (vec: cnt = 8 and 16-byte aligned).
// Four parts per round, loaded before any is used; a round's missing parts re-read the last one with weight 0.
__device__ __forceinline__ void sum_parts8(const float* __restrict__ base, size_t pstride, int n, size_t off, int cnt,
                                           bool vec, float (&acc)[8]) {
    for (int p0 = 0; p0 < n; p0 += 4) {
        float x[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int p = p0 + u < n ? p0 + u : n - 1;
            const float* q = base + (size_t)p * pstride + off;
            if (vec) {
                const float4 lo = *reinterpret_cast<const float4*>(q), hi = *reinterpret_cast<const float4*>(q + 4);
                x[u][0] = lo.x; x[u][1] = lo.y; x[u][2] = lo.z; x[u][3] = lo.w;
                x[u][4] = hi.x; x[u][5] = hi.y; x[u][6] = hi.z; x[u][7] = hi.w;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) x[u][i] = i < cnt ? q[i] : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = p0 + u < n ? 1.0f : 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = fmaf(w, x[u][i], acc[i]);
        }
    }
}

// Rows r0 .. r0 + 31 of a factor stored transposed in FP4 (codes [k, rows], rows % 16 == 0), without the tensor
// scale, into dst[32][k + 1]: a thread decodes 8 consecutive rows of one stored row j (4 code bytes, one scale).
__device__ __forceinline__ void decode_factor_rows(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                   int64_t rows, int k, int64_t r0, float* dst, int tid) {
    const float grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    const int q = tid & 3;
    const int64_t r = r0 + 8 * q;
    for (int j = tid >> 2; j < k; j += 64) {
        uint32_t by[4] = {0, 0, 0, 0};
        float sc = 0.0f;
        if (r < rows) {
            const uint8_t* c = codes + (int64_t)j * (rows / 2) + r / 2;
#pragma unroll
            for (int i = 0; i < 4; ++i) by[i] = c[i];
            sc = e4m3_decode(scales[(int64_t)j * (rows / 16) + r / 16]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t nib = (i & 1) ? (by[i >> 1] >> 4) : (by[i >> 1] & 15u);
            const float v = grid[nib & 7u] * sc;
            dst[(8 * q + i) * (k + 1) + j] = (nib & 8u) ? -v : v;
        }
    }
}

__device__ __forceinline__ uint4 pack8_bf16(const float (&v)[8]) {
    uint4 o;
    o.x = (uint32_t)f32_to_bf16_rne(v[0]) | (uint32_t)f32_to_bf16_rne(v[1]) << 16;
    o.y = (uint32_t)f32_to_bf16_rne(v[2]) | (uint32_t)f32_to_bf16_rne(v[3]) << 16;
    o.z = (uint32_t)f32_to_bf16_rne(v[4]) | (uint32_t)f32_to_bf16_rne(v[5]) << 16;
    o.w = (uint32_t)f32_to_bf16_rne(v[6]) | (uint32_t)f32_to_bf16_rne(v[7]) << 16;
    return o;
}

// NCH = ceil(kb / 64): column groups of a row that hold T1-type columns
template <int NCH>
__global__ void __launch_bounds__(256)
k_assemble_ext(int64_t Ma, int64_t Nb, int ka, int kb, int Kep, const float* __restrict__ T1, int n1,
               const float* __restrict__ Mk, int n3, const float* __restrict__ E2, int n2,
               const uint8_t* __restrict__ ua_codes, const uint8_t* __restrict__ ua_scales, float g_ua,
               const float* __restrict__ Sa, const uint8_t* __restrict__ ub_codes,
               const uint8_t* __restrict__ ub_scales, float g_ub, const float* __restrict__ Sb,
               float inv_grr, bf16_t* __restrict__ Aext, bf16_t* __restrict__ Bext) {
    extern __shared__ __attribute__((aligned(16))) float ax_sm[];
    const int nblk_a = (int)((Ma + AX_ROWS - 1) / AX_ROWS);
    const int tid = threadIdx.x, rr = tid >> 3, cg = tid & 7;
    if ((int)blockIdx.x < nblk_a) {
        float* ua = ax_sm;                                          // [AX_ROWS][ka + 1]
        float* mk = ax_sm + (AX_ROWS * (ka + 1) + 3) / 4 * 4;       // [ka][kb] (+ 8 floats of slack)
        const int64_t r0 = (int64_t)blockIdx.x * AX_ROWS, row = r0 + rr;
        const bool in = row < Ma;
        const int64_t lrow = in ? row : Ma - 1;
        // this thread's sums of the T1 parts
        float t1[NCH][8];
#pragma unroll
        for (int h = 0; h < NCH; ++h) {
#pragma unroll
            for (int i = 0; i < 8; ++i) t1[h][i] = 0.0f;
            const int c0 = 64 * h + 8 * cg;
            if (c0 < kb && n1 > 0) {
                const int cnt = kb - c0 < 8 ? kb - c0 : 8;
                sum_parts8(T1, (size_t)Ma * kb, n1, (size_t)lrow * kb + c0, cnt, cnt == 8 && kb % 4 == 0, t1[h]);
            }
        }
        // Sa Mk (with U_a's tensor scale) into LDS, the parts added on the way
        const int nmk = ka * kb;
        for (int e0 = 8 * tid; e0 < nmk; e0 += 8 * 256) {
            float m[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
            const int cnt = nmk - e0 < 8 ? nmk - e0 : 8;
            sum_parts8(Mk, (size_t)nmk, n3, (size_t)e0, cnt, cnt == 8 && nmk % 4 == 0, m);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < cnt) mk[e0 + i] = m[i] * g_ua * Sa[(e0 + i) / kb];
        }
        decode_factor_rows(ua_codes, ua_scales, Ma, ka, r0, ua, tid);
        __syncthreads();
        if (!in) return;
        const bool vecmk = kb % 4 == 0;
        const float gs = g_ub * inv_grr;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int c0 = 64 * h + 8 * cg;
            if (c0 >= Kep) continue;
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = c0 + i;
                v[i] = (c >= kb && c < kb + ka) ? ua[rr * (ka + 1) + c - kb] : 0.0f;
            }
            if (h < NCH && c0 < kb) {
                float acc[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = t1[h < NCH ? h : 0][i];
                for (int j = 0; j < ka; ++j) {
                    const float u = ua[rr * (ka + 1) + j];
                    const float* mrow = mk + j * kb + c0;
                    if (vecmk) {
                        const float4 lo = *reinterpret_cast<const float4*>(mrow), hi = *reinterpret_cast<const float4*>(mrow + 4);
                        acc[0] = fmaf(u, lo.x, acc[0]); acc[1] = fmaf(u, lo.y, acc[1]);
                        acc[2] = fmaf(u, lo.z, acc[2]); acc[3] = fmaf(u, lo.w, acc[3]);
                        acc[4] = fmaf(u, hi.x, acc[4]); acc[5] = fmaf(u, hi.y, acc[5]);
                        acc[6] = fmaf(u, hi.z, acc[6]); acc[7] = fmaf(u, hi.w, acc[7]);
                    } else {
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[i] = fmaf(u, mrow[i], acc[i]);
                    }
                }
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (c0 + i < kb) v[i] = acc[i] * Sb[c0 + i] * gs;
            }
            *reinterpret_cast<uint4*>(Aext + ext_chunk(row >> 5, c0 >> 4, (c0 >> 3) & 1, rr, Kep >> 4)) = pack8_bf16(v);
        }
        return;
    }
    // Bext rows
    float* ub = ax_sm;                              // [AX_ROWS][kb + 1]
    const int64_t r0 = ((int64_t)blockIdx.x - nblk_a) * AX_ROWS, row = r0 + rr;
    const bool in = row < Nb;
    const int64_t lrow = in ? row : Nb - 1;
    float e2[4][8];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
#pragma unroll
        for (int i = 0; i < 8; ++i) e2[h][i] = 0.0f;
        // the E2-type columns of this group: c in [max(c0, kb), min(c0 + 8, kb + ka)) <-> E2 columns c - kb
        const int c0 = 64 * h + 8 * cg;
        const int lo = c0 > kb ? c0 : kb, hi = c0 + 8 < kb + ka ? c0 + 8 : kb + ka;
        if (lo < hi && n2 > 0) {
            const int cnt = hi - lo;
            sum_parts8(E2, (size_t)Nb * ka, n2, (size_t)lrow * ka + (lo - kb), cnt,
                       cnt == 8 && ka % 4 == 0 && (lo - kb) % 4 == 0, e2[h]);
        }
    }
    decode_factor_rows(ub_codes, ub_scales, Nb, kb, r0, ub, tid);
    __syncthreads();
    if (!in) return;
    const float gs = g_ua * inv_grr;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        const int c0 = 64 * h + 8 * cg;
        if (c0 >= Kep) continue;
        const int lo = c0 > kb ? c0 : kb;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = c0 + i;
            float x = 0.0f;
            if (c < kb) x = ub[rr * (kb + 1) + c];
            else if (c < kb + ka) {
                // e2[h] holds the group's E2-type columns from index 0 on
                float t = 0.0f;
#pragma unroll
                for (int z = 0; z < 8; ++z) t = (c - lo == z) ? e2[h][z] : t;
                x = t * Sa[c - kb] * gs;
            }
            v[i] = x;
        }
        *reinterpret_cast<uint4*>(Bext + ext_chunk(row >> 5, c0 >> 4, (c0 >> 3) & 1, rr, Kep >> 4)) = pack8_bf16(v);
    }
}

struct NtOperand {            // one side of Abar Bbar^T: Abar = U diag(S) V^T + R, R [rows, Kc]
    metis_fp4 R, Ut, Vt;      // Ut [k, rows], Vt [k, Kc]
    const float* S;
    int k;
};

struct LinWs {
    size_t off_t1, off_mk, off_e2, off_aext, off_bext, off_tail, tail_bytes, total;
    int Kep;
    int s1, s2, s3;          // contraction parts of T1, E2, Mk
};

// Parts of a skinny product with rows x cols outputs: few output tiles, long contraction -> cut it so that about
// 256 workgroups share the work, each with at least two stages.
int skinny_parts(int64_t rows, int64_t cols, int64_t Kc, int64_t cap) {
    const int64_t tiles = ceil_div64(rows, 128) * ceil_div64(cols, 64), iters = ceil_div64(Kc, G_KI);
    int64_t want = ceil_div64(256, tiles);
    const int64_t maxs = iters / 2 > 0 ? iters / 2 : 1;
    if (want > maxs) want = maxs;
    if (want > cap) want = cap;
    const int64_t ips = ceil_div64(iters, want);
    return (int)ceil_div64(iters, ips);           // no empty part
}

LinWs lin_layout(int64_t Ma, int64_t Nb, int ka, int kb, int64_t Kc) {
    LinWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    w.Kep = (ka + kb + 15) / 16 * 16;
    // (the assembly kernel adds the parts up, two rounds of four loads at most)
    w.s1 = kb > 0 ? skinny_parts(Ma, kb, Kc, 8) : 1;
    w.s2 = ka > 0 ? skinny_parts(Nb, ka, Kc, 8) : 1;
    w.s3 = ka > 0 && kb > 0 ? skinny_parts(ka, kb, Kc, 8) : 1;
    w.off_t1 = take((size_t)w.s1 * Ma * (kb > 0 ? kb : 1) * 4);
    w.off_mk = take((size_t)w.s3 * (ka > 0 ? ka : 1) * (kb > 0 ? kb : 1) * 4);
    w.off_e2 = take((size_t)w.s2 * Nb * (ka > 0 ? ka : 1) * 4);
    w.off_aext = take((size_t)((Ma + 31) / 32 * 32) * (w.Kep > 0 ? w.Kep : 16) * 2);       // rows padded to whole 32-row blocks
    w.off_bext = take((size_t)((Nb + 31) / 32 * 32) * (w.Kep > 0 ? w.Kep : 16) * 2);
    w.tail_bytes = (Ma >= 1024 && Nb >= 1024 && Kc % G_KI == 0) ? gemm_tail_bytes(Ma, Nb, Kc) : 0;
    w.off_tail = take(w.tail_bytes);
    w.total = o;
    return w;
}

bool fp4_valid(const metis_fp4& f) { return f.codes && f.scales && f.rows > 0 && f.cols > 0 && f.cols % 16 == 0; }

// phase: METIS_LINEAR_ALL, or only the pre-pass (PREPARE: fills the workspace) / only the main kernel (APPLY)
int linear_nt(hipStream_t s, const NtOperand& a, const NtOperand& b, metis_mat* out, void* workspace,
              size_t workspace_bytes, int phase = METIS_LINEAR_ALL) {
    const bool do_pre = phase != METIS_LINEAR_APPLY, do_main = phase != METIS_LINEAR_PREPARE;
    if (do_main && (!out || !out->ptr)) return METIS_INVALID_ARG;
    if (!fp4_valid(a.R) || !fp4_valid(b.R) || a.R.cols != b.R.cols) return METIS_BAD_SHAPE;
    const int64_t Ma = a.R.rows, Nb = b.R.rows, Kc = a.R.cols;
    if (do_main) {
        if (out->rows != Ma || out->cols != Nb || out->ld < Nb) return METIS_BAD_SHAPE;
        if (out->dtype != METIS_BF16 && out->dtype != METIS_F32) return METIS_INVALID_ARG;
    }
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
        if (do_pre) {
            // the skinny products T1 = R_a V_b^T, E2 = R_b V_a^T and Mk = V_a V_b^T in one launch, cut along the contraction
            // (Mk is a single output tile: alone, one workgroup would walk the whole contraction, ~100 us at 14336 columns)
            SkinnyBatch sb;
            sb.count = 0;
            int wgs = 0;
            const int64_t iters = ceil_div64(Kc, G_KI);
            bool vec = Kc % G_KI == 0;
            auto add = [&](const metis_fp4& X, const metis_fp4& Y, float* P, int parts) {
                SkinnyProblem& q = sb.p[sb.count++];
                q.A = {X.codes, X.scales, X.rows};
                q.B = {Y.codes, Y.scales, Y.rows};
                q.alpha = X.tscale * Y.tscale;
                q.P = P;
                q.tiles_n = (int)ceil_div64(Y.rows, 64);
                q.tiles = (int)ceil_div64(X.rows, 128) * q.tiles_n;
                q.ips = (int)ceil_div64(iters, parts);
                q.first = wgs;
                wgs += q.tiles * parts;
                vec = vec && reinterpret_cast<uintptr_t>(X.codes) % 16 == 0 && reinterpret_cast<uintptr_t>(Y.codes) % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(X.scales) % 8 == 0 && reinterpret_cast<uintptr_t>(Y.scales) % 8 == 0;
            };
            if (ceil_div64(Ma, 128) * 64 * w.s1 + ceil_div64(Nb, 128) * 64 * w.s2 > 0x3FFFFFFF) return METIS_UNSUPPORTED;
            if (kb > 0) add(a.R, b.Vt, T1, w.s1);
            if (ka > 0) add(b.R, a.Vt, E2, w.s2);
            if (ka > 0 && kb > 0) add(a.Vt, b.Vt, Mk, w.s3);
            for (int i = sb.count; i < 3; ++i) sb.p[i] = sb.p[0];
            {
                constexpr size_t lds = gemm_lds_bytes<128, 64>();
                if (vec) {
                    static LdsLimitCache lds_set;
                    if (!ensure_dyn_lds((const void*)k_fp4_skinny_batch<true>, lds, lds_set)) return METIS_HIP_ERROR;
                    hipLaunchKernelGGL(k_fp4_skinny_batch<true>, dim3((unsigned)wgs), dim3(256), lds, s, sb, Kc);
                } else {
                    static LdsLimitCache lds_set;
                    if (!ensure_dyn_lds((const void*)k_fp4_skinny_batch<false>, lds, lds_set)) return METIS_HIP_ERROR;
                    hipLaunchKernelGGL(k_fp4_skinny_batch<false>, dim3((unsigned)wgs), dim3(256), lds, s, sb, Kc);
                }
                METIS_LAUNCH_CHECK();
            }
            const int64_t nblk = ceil_div64(Ma, AX_ROWS) + ceil_div64(Nb, AX_ROWS);
            const size_t ax_lds = ((size_t)(AX_ROWS * ((ka > kb ? ka : kb) + 1) + 3) / 4 * 4 + (size_t)ka * kb + 8) * sizeof(float);
            auto assemble = kb > 64 ? k_assemble_ext<2> : k_assemble_ext<1>;
            static LdsLimitCache ax_set[2];
            if (ax_lds > 48 * 1024 && !ensure_dyn_lds((const void*)assemble, ax_lds, ax_set[kb > 64])) return METIS_HIP_ERROR;
            hipLaunchKernelGGL(assemble, dim3((unsigned)nblk), dim3(256), ax_lds, s, Ma, Nb, ka, kb, w.Kep,
                               T1, w.s1, Mk, w.s3, E2, w.s2, a.Ut.codes, a.Ut.scales, ka > 0 ? a.Ut.tscale : 1.0f, a.S, b.Ut.codes,
                               b.Ut.scales, kb > 0 ? b.Ut.tscale : 1.0f, b.S, 1.0f / grr, ae, be);
            METIS_LAUNCH_CHECK();
        }
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
    if (!do_main) return METIS_OK;
    const int pi = metis_prof_begin(METIS_PROF_GEMM, s);
    if (out->dtype == METIS_BF16)
        st = launch_gemm<bf16_t>(s, a.R, b.R, Aext, Bext, Ke, grr, (bf16_t*)out->ptr, out->ld, partial, partial_bytes);
    else
        st = launch_gemm<float>(s, a.R, b.R, Aext, Bext, Ke, grr, (float*)out->ptr, out->ld, partial, partial_bytes);
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

extern "C" int metis_fp4_linear_phase(void* stream, int product, int phase, const metis_split* a, const metis_split* b,
                                      metis_mat* out, void* workspace, size_t workspace_bytes) {
    if (!a || !b || phase < METIS_LINEAR_ALL || phase > METIS_LINEAR_APPLY) return METIS_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    switch (product) {
        case METIS_LINEAR_FWD:        // a = X, b = W
            return linear_nt(s, nt(a->R, a->Ut, a->Vt, a->S, a->k), nt(b->R, b->Ut, b->Vt, b->S, b->k), out, workspace,
                             workspace_bytes, phase);
        case METIS_LINEAR_DGRAD:      // a = G, b = W
            return linear_nt(s, nt(a->R, a->Ut, a->Vt, a->S, a->k), nt(b->Rt, b->Vt, b->Ut, b->S, b->k), out, workspace,
                             workspace_bytes, phase);
        case METIS_LINEAR_WGRAD:      // a = G, b = X
            return linear_nt(s, nt(a->Rt, a->Vt, a->Ut, a->S, a->k), nt(b->Rt, b->Vt, b->Ut, b->S, b->k), out, workspace,
                             workspace_bytes, phase);
        default: return METIS_INVALID_ARG;
    }
}
