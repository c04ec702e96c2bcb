// metis_split_quantize: R = A - U diag(S) V^T fused with the NVFP4 quantizer (Sec. 3.2:
// the split; Q_b applied to U, V and R separately; Sec. 2.3: the quantizer).
//
// The low-rank product runs on the bf16 matrix cores with both factors split in two bf16
// parts (hi*hi + hi*lo + lo*hi, ~2^-16 relative), fp32 accumulation; A is streamed once and
// the fp32 residual tile is quantized along both axes before it leaves the workgroup.
#include "splitq.h"
#include "quant_dev.h"
#include <type_traits>

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

namespace {

union Frag {
    uint4 u;
    bf16x8_t v;
};

// -(U diag(S)) and V as bf16 hi/lo, row-major with the rank padded to kp (a multiple of 16)
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
        if (c < k) x = -(U[row * k + c] * S[c]);
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

// 16 bytes of codes (two neighbouring blocks) to an 8-byte aligned address in one store
typedef uint32_t uvec4_a8 __attribute__((ext_vector_type(4), aligned(8)));
__device__ __forceinline__ void store_codes16(uint8_t* p, uint2 c0, uint2 c1) {
    uvec4_a8 v = {c0.x, c0.y, c1.x, c1.y};
    *reinterpret_cast<uvec4_a8*>(p) = v;
}
// the scale bytes of two neighbouring blocks: one 16-bit store where the address allows it
__device__ __forceinline__ void store_scale_pair(uint8_t* p, uint32_t s0, uint32_t s1) {
    if ((reinterpret_cast<uintptr_t>(p) & 1) == 0) {
        *reinterpret_cast<uint16_t*>(p) = (uint16_t)((s0 & 0xFFu) | ((s1 & 0xFFu) << 8));
    } else {
        p[0] = (uint8_t)s0;
        p[1] = (uint8_t)s1;
    }
}

#define RQ_ROWS 128              // rows per workgroup (4 waves x 32)
#define RQ_COLS 64               // columns per step
#define RQ_LDR 68                // padded fp32 row of the per-wave residual tile (16-byte aligned rows)

typedef uint32_t uvec4_t __attribute__((ext_vector_type(4)));   // native vector: selects and arrays stay in registers

// Residual + quantize.  One workgroup = 4 waves = 128 rows x a run of 64-column steps.
// Per step and wave: R[32 x 64] = A + (-U S) V^T entirely on the matrix cores (A enters through an
// identity operand, so the bf16 values are added exactly into the fp32 accumulators); the
// -U S fragments of the wave's rows stay in registers for the whole run, V is staged through
// LDS, A and V for the next step are in flight while the current one is processed.
// Blocks along the rows of A (transposed output, WT) are quantized straight from the accumulators
// after a half-wave swap; blocks along the columns go through a per-wave LDS tile.
// Every global load is unconditional (a lane with nothing to read loads the first 16 bytes of the
// array and its value is replaced by zero on the way into LDS).  A workgroup whose rows and steps
// are all whole runs a step body without any branch around its loads and stores: the compiler can
// then count them and wait for the loads of the next step only, not for this step's stores, whose
// round trip would otherwise stall every step.
// grid: (ceil(M/128), csplit); block 256.  KS = kp / 16.
template <int KS, bool SR, bool WT>
__global__ void __launch_bounds__(256, KS <= 4 ? 2 : 1)
k_residual_quant(const bf16_t* __restrict__ A, int64_t lda, int64_t M, int64_t N, int64_t cchunk,
                 const bf16_t* __restrict__ us_hi, const bf16_t* __restrict__ us_lo,
                 const bf16_t* __restrict__ v_hi, const bf16_t* __restrict__ v_lo, QuantParams qp,
                 uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, uint8_t* __restrict__ codes_t,
                 uint8_t* __restrict__ scales_t, float* __restrict__ R_debug, uint64_t seed, int64_t Mt, int64_t row_off) {
    // A may be a band of rows of a taller matrix: Mt = rows of the whole matrix (row length of the transposed
    // outputs, whose pointers already point at this band's first row), row_off = the band's first row (only the
    // stochastic-rounding word index needs it)
    constexpr int KP = 16 * KS, LDV = KP + 8;
    constexpr int VVEC = 2 * RQ_COLS * (KP / 8) / 256;                          // 16-byte V vectors per thread
    static_assert(VVEC * 256 == 2 * RQ_COLS * (KP / 8), "a V stage is a whole number of vectors per thread");
    // one V stage (hi and lo): a second buffer saves a barrier per step but measured slower
    __shared__ __attribute__((aligned(16))) bf16_t Vs[2][RQ_COLS][LDV];         // [hi/lo][column][k]
    __shared__ __attribute__((aligned(16))) float Rt[4][32][RQ_LDR];           // per-wave residual tile
    // per-wave bf16 slice of A, overlaid on the wave's residual tile: it is consumed (operand reads)
    // before the tile is written and refilled after the tile has been read
    typedef bf16_t ASlice[32][RQ_COLS + 8];
    static_assert(sizeof(ASlice) <= sizeof(float) * 32 * RQ_LDR, "A slice must fit in the residual tile");
    // Output staging of the whole-workgroup path.  Scattered 16-byte and 2-byte stores make the memory
    // system request-bound, so the codes leave as whole lines: a wave collects four steps of its 32 rows
    // (128 bytes of codes and 16 bytes of scales per row), the workgroup collects one step of the
    // transposed copy (64 bytes of codes and 8 bytes of scales per column of A).
    __shared__ __attribute__((aligned(16))) uvec4_t Cst[4][32][9];              // [wave][row][16-byte piece], padded
    __shared__ __attribute__((aligned(4))) uint16_t Sst[4][32][8];              // [wave][row][2 * step + half]
    __shared__ __attribute__((aligned(16))) uvec4_t Tst[WT ? RQ_COLS : 1][5];   // [column][wave], padded
    __shared__ __attribute__((aligned(2))) uint16_t Tsc[WT ? RQ_COLS : 1][4];   // [column][wave]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, half = lane >> 5;
    const int64_t wr0 = (int64_t)blockIdx.x * RQ_ROWS + 32 * wave;
    const int64_t cbeg = (int64_t)blockIdx.y * cchunk;
    const int64_t cend = cbeg + cchunk < N ? cbeg + cchunk : N;
    if (cbeg >= N) return;
    int64_t arow = wr0 + li;
    if (arow >= M) arow = M - 1;              // in-bounds loads; results for such rows are not stored

    // persistent -U S fragments of this wave's 32 rows
    Frag ush[KS], usl[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        ush[ks].u = *reinterpret_cast<const uint4*>(us_hi + arow * KP + 16 * ks + 8 * half);
        usl[ks].u = *reinterpret_cast<const uint4*>(us_lo + arow * KP + 16 * ks + 8 * half);
    }
    // identity operand: contraction slot (step s, half h, element e) stands for column 16s + 8h + e of a tile
    Frag idf[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
        uint32_t w[4] = {0, 0, 0, 0};
        int e = li - 16 * s2 - 8 * half;
        if (e >= 0 && e < 8) w[e >> 1] = (e & 1) ? 0x3F800000u : 0x00003F80u;
        idf[s2].u = make_uint4(w[0], w[1], w[2], w[3]);
    }
    // A is read with coalesced 16-byte loads (8 lanes cover the 128 bytes one row contributes to a
    // step) and reaches the MFMA operand layout through the wave's LDS slice
    const int lrow = lane >> 3, piece = lane & 7;
    const bf16_t* aptr[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int64_t r = wr0 + 8 * q + lrow;
        aptr[q] = A + (r < M ? r : M - 1) * lda + 8 * piece;
    }
    const uvec4_t zero4 = {0u, 0u, 0u, 0u};
    ASlice& aslice = *reinterpret_cast<ASlice*>(&Rt[wave][0][0]);
    // `live` = the step exists; columns at or past cend read nothing
    auto load_a = [&](int64_t n0, bool live, uvec4_t (&a)[4]) {
        const bool in = live && n0 + 8 * piece < cend;
#pragma unroll
        for (int q = 0; q < 4; ++q) a[q] = *reinterpret_cast<const uvec4_t*>(in ? aptr[q] + n0 : A);
    };
    auto store_a = [&](const uvec4_t (&a)[4], int64_t n0, bool live, bool whole) {
        const bool in = whole || (live && n0 + 8 * piece < cend);
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<uvec4_t*>(&aslice[8 * q + lrow][8 * piece]) = in ? a[q] : zero4;
    };
    auto load_v = [&](int64_t n0, bool live, uvec4_t (&b)[VVEC]) {
#pragma unroll
        for (int v = 0; v < VVEC; ++v) {
            int e = tid + 256 * v;
            int part = e / (RQ_COLS * (KP / 8));
            int r = e % (RQ_COLS * (KP / 8));
            int c = r / (KP / 8), seg = r % (KP / 8);
            const bool in = live && n0 + c < cend;
            b[v] = *reinterpret_cast<const uvec4_t*>(in ? (part ? v_lo : v_hi) + (n0 + c) * KP + seg * 8 : v_hi);
        }
    };
    auto store_v = [&](const uvec4_t (&b)[VVEC], int64_t n0, bool live, bool whole) {
#pragma unroll
        for (int v = 0; v < VVEC; ++v) {
            int e = tid + 256 * v;
            int part = e / (RQ_COLS * (KP / 8));
            int r = e % (RQ_COLS * (KP / 8));
            int c = r / (KP / 8), seg = r % (KP / 8);
            const bool in = whole || (live && n0 + c < cend);
            *reinterpret_cast<uvec4_t*>(&Vs[part][c][seg * 8]) = in ? b[v] : zero4;
        }
    };

    uvec4_t a_nxt[4];
    uvec4_t v_nxt[VVEC];
    load_a(cbeg, true, a_nxt);
    load_v(cbeg, true, v_nxt);
    store_a(a_nxt, cbeg, true, false);
    store_v(v_nxt, cbeg, true, false);
    __syncthreads();

    // one 64-column step; WHOLE = every row, column and step of this workgroup exists and the scale rows
    // start on even addresses (no bounds checks, no branches around loads and stores)
    // the four finished steps of this wave's rows (cnt < 4: the last, shorter group) as whole lines
    auto flush_rows = [&](int64_t gn0, int cnt) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = 8 * q + lrow;
            if (piece < 2 * cnt)
                *reinterpret_cast<uvec4_t*>(codes + (wr0 + row) * (N / 2) + gn0 / 2 + 16 * piece) = Cst[wave][row][piece];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int w = 2 * half + j;       // the scale bytes of step w of the group: one dword per row
            if (w < cnt)
                *reinterpret_cast<uint32_t*>(scales + (wr0 + li) * (N / 16) + gn0 / 16 + 4 * w) =
                    *reinterpret_cast<const uint32_t*>(&Sst[wave][li][2 * w]);
        }
    };
    const int64_t brow0 = (int64_t)blockIdx.x * RQ_ROWS;

    auto step = [&](auto WHOLE_C, int64_t n0, int g) {
        constexpr bool WHOLE = decltype(WHOLE_C)::value;
        const bool more = n0 + RQ_COLS < cend;
        // a finished group leaves before the next loads are issued: the wait for those loads then never
        // includes these stores
        if (WHOLE && g == 0 && n0 > cbeg) flush_rows(n0 - 4 * RQ_COLS, 4);
        load_a(n0 + RQ_COLS, more, a_nxt);
        load_v(n0 + RQ_COLS, more, v_nxt);
        float16_t acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
            Frag a0, a1;
            a0.u = *reinterpret_cast<const uint4*>(&aslice[li][32 * t + 8 * half]);
            a1.u = *reinterpret_cast<const uint4*>(&aslice[li][32 * t + 16 + 8 * half]);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, idf[0].v, acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, idf[1].v, acc[t], 0, 0, 0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                Frag bh, bl;
                bh.u = *reinterpret_cast<const uint4*>(&Vs[0][32 * t + li][16 * ks + 8 * half]);
                bl.u = *reinterpret_cast<const uint4*>(&Vs[1][32 * t + li][16 * ks + 8 * half]);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ush[ks].v, bh.v, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ush[ks].v, bl.v, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(usl[ks].v, bh.v, acc[t], 0, 0, 0);
            }
        }
        // accumulator layout: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32 of tile t
        // ---- blocks along the columns: through the wave's LDS tile (this overwrites the A slice) ----
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) Rt[wave][8 * (v >> 2) + 4 * half + (v & 3)][32 * t + li] = acc[t][v];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        {
            const int64_t m = wr0 + li;
            uint2 cc[2] = {make_uint2(0, 0), make_uint2(0, 0)};
            uint32_t ss[2] = {0, 0};
#pragma unroll
            for (int bb = 0; bb < 2; ++bb) {
                const int blk = 2 * half + bb;
                const int64_t n = n0 + 16 * blk;
                float x[16];
                const float4* src = reinterpret_cast<const float4*>(&Rt[wave][li][16 * blk]);
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    float4 f = src[q4];
                    x[4 * q4] = f.x; x[4 * q4 + 1] = f.y; x[4 * q4 + 2] = f.z; x[4 * q4 + 3] = f.w;
                }
                if (WHOLE || (m < M && n < cend)) {
                    // stochastic rounding draws: stream 3, word = row-major position in R
                    ss[bb] = SR ? quantize_block16_sr(x, qp, cc[bb], seed, 3u, (uint64_t)((row_off + m) * N + n))
                                : quantize_block16(x, qp, cc[bb]);
                    if (!WHOLE && R_debug) {
                        float4* dst = reinterpret_cast<float4*>(R_debug + m * N + n);
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) dst[q4] = make_float4(x[4 * q4], x[4 * q4 + 1], x[4 * q4 + 2], x[4 * q4 + 3]);
                    }
                }
            }
            // the lane's two blocks are neighbours in the row: one 16-byte and one 2-byte store (scattered
            // narrow stores, not the bytes, are what this kernel's output costs)
            const int64_t na = n0 + 32 * half;
            uint8_t* cp = codes + m * (N / 2) + na / 2;
            uint8_t* sp = scales + m * (N / 16) + na / 16;
            if (WHOLE) {
                const uvec4_t cv = {cc[0].x, cc[0].y, cc[1].x, cc[1].y};
                Cst[wave][li][2 * g + half] = cv;
                Sst[wave][li][2 * g + half] = (uint16_t)((ss[0] & 0xFFu) | ((ss[1] & 0xFFu) << 8));
            } else if (m < M && na < cend) {
                if (na + 16 < cend) {
                    store_codes16(cp, cc[0], cc[1]);
                    store_scale_pair(sp, ss[0], ss[1]);
                } else {
                    *reinterpret_cast<uint2*>(cp) = cc[0];
                    sp[0] = (uint8_t)ss[0];
                }
            }
        }
        // ---- blocks along the rows (transposed output): half-wave swap, then in-lane ----
        if (WT) {
            uint2 ct[2] = {make_uint2(0, 0), make_uint2(0, 0)};
            uint32_t st[2] = {0, 0};
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                float x[16];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    // swap the upper half of element i with the lower half of element i+8
                    auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[t][i]), __float_as_uint(acc[t][i + 8]), false, false);
                    // lower lanes: rows 0-15 of the tile, upper lanes: rows 16-31
                    x[(i & 3) + 8 * (i >> 2)] = __uint_as_float(sw[0]);
                    x[(i & 3) + 8 * (i >> 2) + 4] = __uint_as_float(sw[1]);
                }
                const int64_t n = n0 + 32 * t + li, m = wr0 + 16 * half;
                if (WHOLE || (n < cend && m < M)) {
                    // transposed copy: stream 4, word = row-major position in R^T
                    st[t] = SR ? quantize_block16_sr(x, qp, ct[t], seed, 4u, (uint64_t)(n * Mt + row_off + m))
                               : quantize_block16(x, qp, ct[t]);
                }
            }
            // second swap: the lower lanes end up with both 16-row blocks of column li of tile 0, the upper
            // lanes with those of tile 1 (element 0 = rows 0-15, element 1 = rows 16-31), 16 bytes in a row
            auto sx = __builtin_amdgcn_permlane32_swap(ct[0].x, ct[1].x, false, false);
            auto sy = __builtin_amdgcn_permlane32_swap(ct[0].y, ct[1].y, false, false);
            auto sq = __builtin_amdgcn_permlane32_swap(st[0], st[1], false, false);
            const int64_t n = n0 + 32 * half + li;
            uint8_t* cp = codes_t + n * (Mt / 2) + wr0 / 2;
            uint8_t* sp = scales_t + n * (Mt / 16) + wr0 / 16;
            if (WHOLE) {
                const uvec4_t cv = {sx[0], sy[0], sx[1], sy[1]};
                Tst[32 * half + li][wave] = cv;
                Tsc[32 * half + li][wave] = (uint16_t)((sq[0] & 0xFFu) | ((sq[1] & 0xFFu) << 8));
            } else if (n < cend && wr0 < M) {
                if (wr0 + 16 < M) {
                    store_codes16(cp, make_uint2(sx[0], sy[0]), make_uint2(sx[1], sy[1]));
                    store_scale_pair(sp, sq[0], sq[1]);
                } else {
                    *reinterpret_cast<uint2*>(cp) = make_uint2(sx[0], sy[0]);
                    sp[0] = (uint8_t)sq[0];
                }
            }
        }
        __syncthreads();                      // everybody has finished reading the V stage
        if (WHOLE && WT) {
            // four lanes cover the 64 bytes one column of A gets from this workgroup's 128 rows
            const int nl = tid >> 2, w = tid & 3;
            *reinterpret_cast<uvec4_t*>(codes_t + (n0 + nl) * (Mt / 2) + brow0 / 2 + 16 * w) = Tst[nl][w];
            *reinterpret_cast<uint16_t*>(scales_t + (n0 + nl) * (Mt / 16) + brow0 / 16 + 2 * w) = Tsc[nl][w];
        }
        store_v(v_nxt, n0 + RQ_COLS, more, WHOLE);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        store_a(a_nxt, n0 + RQ_COLS, more, WHOLE);
        __syncthreads();
    };

    // whole: all 128 rows and every step exist, and rows of the outputs start where 16-byte code stores and
    // 4-byte (transposed copy: 2-byte) scale stores are aligned
    const bool whole = !R_debug && brow0 + RQ_ROWS <= M && (cend - cbeg) % RQ_COLS == 0 && N % 64 == 0 &&
                       reinterpret_cast<uintptr_t>(codes) % 16 == 0 && reinterpret_cast<uintptr_t>(scales) % 4 == 0 &&
                       (!WT || (M % 32 == 0 && Mt % 32 == 0 && reinterpret_cast<uintptr_t>(codes_t) % 16 == 0 &&
                                reinterpret_cast<uintptr_t>(scales_t) % 2 == 0));
    if (whole) {
        int g = 0;
        for (int64_t n0 = cbeg; n0 < cend; n0 += RQ_COLS, g = (g + 1) & 3) step(std::true_type{}, n0, g);
        const int cnt = g == 0 ? 4 : g;       // steps in the last group
        flush_rows(cend - (int64_t)cnt * RQ_COLS, cnt);
    } else {
        for (int64_t n0 = cbeg; n0 < cend; n0 += RQ_COLS) step(std::false_type{}, n0, 0);
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

namespace {
// C = sum of the partial products (fp64 sum in part order, rounded once: the same sum the Gram kernel takes of
// separate parts), -C as bf16 hi / lo with the rank padded to kp
__global__ void __launch_bounds__(256)
k_band_factors(const float* __restrict__ parts, int nparts, int64_t part_stride, int64_t rows, int k, int kp,
               float* __restrict__ C_out, bf16_t* __restrict__ us_hi, bf16_t* __restrict__ us_lo) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * kp) return;
    const int64_t row = t / kp;
    const int c = (int)(t - row * kp);
    float x = 0.0f;
    if (c < k) {
        double acc = 0.0;
        for (int p = 0; p < nparts; ++p) acc += (double)parts[p * part_stride + row * k + c];
        x = (float)acc;
        C_out[row * k + c] = x;
        x = -x;
    }
    const bf16_t h = f32_to_bf16_rne(x);
    us_hi[row * kp + c] = h;
    us_lo[row * kp + c] = f32_to_bf16_rne(x - bf16_to_f32(h));
}
}  // namespace

int launch_v_factors(hipStream_t s, const float* V, int64_t N, int k, int kp, bf16_t* v_hi, bf16_t* v_lo) {
    hipLaunchKernelGGL(k_split_factors, dim3((unsigned)ceil_div64(N * kp, 256)), dim3(256), 0, s, (const float*)nullptr,
                       (const float*)nullptr, V, (int64_t)0, N, k, kp, (bf16_t*)nullptr, (bf16_t*)nullptr, v_hi, v_lo,
                       (float*)nullptr);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

int launch_band_factors(hipStream_t s, const float* parts, int nparts, int64_t part_stride, int64_t rows, int k, int kp,
                        float* C_out, bf16_t* us_hi, bf16_t* us_lo) {
    hipLaunchKernelGGL(k_band_factors, dim3((unsigned)ceil_div64(rows * kp, 256)), dim3(256), 0, s, parts, nparts, part_stride,
                       rows, k, kp, C_out, us_hi, us_lo);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

int check_split_out(int64_t M, int64_t N, int k, const metis_split* out) {
    if (!out || k < 1 || out->k != k || !out->S) return METIS_INVALID_ARG;
    if (k > 128) return METIS_UNSUPPORTED;
    if (N % 16) return METIS_BAD_SHAPE;
    const bool want_t = out->Rt.codes != nullptr;
    if (!fp4_ok(out->R, M, N)) return METIS_BAD_SHAPE;
    if (want_t && (!fp4_ok(out->Rt, N, M) || out->Rt.tscale != out->R.tscale)) return METIS_BAD_SHAPE;
    if (!fp4_ok(out->Ut, k, M) || !fp4_ok(out->Vt, k, N)) return METIS_BAD_SHAPE;
    return METIS_OK;
}


// Launch of the fused residual + quantize kernel on A [M rows, N] (possibly a band of rows of a matrix with Mt
// rows, starting at row row_off; the transposed outputs then point at the band's first row).
int launch_residual_quant(hipStream_t s, const bf16_t* Ap, int64_t lda, int64_t M, int64_t N, int64_t Mt, int64_t row_off,
                          const bf16_t* us_hi, const bf16_t* us_lo, const bf16_t* v_hi, const bf16_t* v_lo, int kp, float g,
                          uint8_t* codes, uint8_t* scales, uint8_t* ct, uint8_t* st_, float* R_debug, bool sr, uint64_t seed) {
    // two workgroups per CU at a time; every workgroup walks at least four 64-column steps; the number of column
    // chunks that fills the last round of workgroups best
    const int64_t row_blocks = ceil_div64(M, RQ_ROWS);
    const int64_t want = balanced_split(row_blocks, ceil_div64(N, 4 * RQ_COLS), 512);
    int64_t cchunk = ceil_div64(ceil_div64(N, want), RQ_COLS) * RQ_COLS;
    if (cchunk < 4 * RQ_COLS) cchunk = 4 * RQ_COLS;
    dim3 grid((unsigned)row_blocks, (unsigned)ceil_div64(N, cchunk));
    const QuantParams qp = make_quant_params(g);
    const bool want_t = ct != nullptr;
    const int pi = metis_prof_begin(METIS_PROF_RESIDUAL_QUANT, s);
#define RQ_LAUNCH3(KS_, SR_, WT_)                                                                                       \
    hipLaunchKernelGGL((k_residual_quant<KS_, SR_, WT_>), grid, dim3(256), 0, s, Ap, lda, M, N, cchunk, us_hi, us_lo,   \
                       v_hi, v_lo, qp, codes, scales, ct, st_, R_debug, seed, Mt, row_off)
#define RQ_LAUNCH(KS_, WT_) do { if (sr) RQ_LAUNCH3(KS_, true, WT_); else RQ_LAUNCH3(KS_, false, WT_); } while (0)
    switch (kp / 16) {
        case 1: if (want_t) RQ_LAUNCH(1, true); else RQ_LAUNCH(1, false); break;
        case 2: if (want_t) RQ_LAUNCH(2, true); else RQ_LAUNCH(2, false); break;
        case 4: if (want_t) RQ_LAUNCH(4, true); else RQ_LAUNCH(4, false); break;
        default: if (want_t) RQ_LAUNCH(8, true); else RQ_LAUNCH(8, false); break;
    }
#undef RQ_LAUNCH
#undef RQ_LAUNCH3
    metis_prof_end(METIS_PROF_RESIDUAL_QUANT, pi, s);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

int padded_rank(int k) { return k <= 16 ? 16 : k <= 32 ? 32 : k <= 64 ? 64 : 128; }

extern "C" size_t metis_split_workspace_bytes(int64_t M, int64_t N, int k) {
    if (M < 1 || N < 1 || k < 1 || k > 128) return 0;
    int64_t kp = padded_rank(k);
    return align_up((size_t)M * kp * 2, 256) * 2 + align_up((size_t)N * kp * 2, 256) * 2;
}

extern "C" int metis_quantize_sr(void* stream, const metis_mat* A, uint64_t seed, metis_fp4* out, metis_fp4* out_t);

extern "C" int metis_quantize(void* stream, const metis_mat* A, metis_fp4* out, metis_fp4* out_t);

int quantize_factors(hipStream_t s, const float* U, const float* S, const float* V, int64_t M, int64_t N, int k,
                     metis_split* out, bool sr, uint64_t seed) {
    // factors: Q(U^T) [k,M], Q(V^T) [k,N], blocks along the long axis; with stochastic rounding the two draw under
    // their own keys so that no two tensors share draws
    return launch_quantize_factors_t(s, U, M, V, N, k, out->Ut, out->Vt, sr, seed + 1, seed + 2,
                                     S && out->S != S ? S : nullptr, out->S);
}

template <bool SR>
static int split_quantize_impl(void* stream, const metis_mat* A, const float* U, const float* S, const float* V,
                               int k, uint64_t seed, metis_split* out, float* R_debug, void* workspace,
                               size_t workspace_bytes) {
    if (!A || !A->ptr || !U || !S || !V || !out || !workspace) return METIS_INVALID_ARG;
    if (k < 1 || out->k != k || !out->S) return METIS_INVALID_ARG;
    if (A->dtype != METIS_BF16 || k > 128) return METIS_UNSUPPORTED;
    const int64_t M = A->rows, N = A->cols;
    if (M < 1 || N < 1 || A->ld < N) return METIS_BAD_SHAPE;
    if (N % 16 || A->ld % 8 || reinterpret_cast<uintptr_t>(A->ptr) % 16) return METIS_BAD_SHAPE;   // 16-byte row loads
    const bool want_t = out->Rt.codes != nullptr;
    if (!fp4_ok(out->R, M, N)) return METIS_BAD_SHAPE;
    if (want_t && (!fp4_ok(out->Rt, N, M) || out->Rt.tscale != out->R.tscale)) return METIS_BAD_SHAPE;
    if (!fp4_ok(out->Ut, k, M) || !fp4_ok(out->Vt, k, N)) return METIS_BAD_SHAPE;
    if (workspace_bytes < metis_split_workspace_bytes(M, N, k)) return METIS_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16) return METIS_INVALID_ARG;

    hipStream_t s = (hipStream_t)stream;
    const int kp = padded_rank(k);
    char* ws = (char*)workspace;
    const size_t ub = align_up((size_t)M * kp * 2, 256), vb = align_up((size_t)N * kp * 2, 256);
    bf16_t* us_hi = (bf16_t*)ws;
    bf16_t* us_lo = (bf16_t*)(ws + ub);
    bf16_t* v_hi = (bf16_t*)(ws + 2 * ub);
    bf16_t* v_lo = (bf16_t*)(ws + 2 * ub + vb);
    int64_t tot = (M + N) * kp;
    hipLaunchKernelGGL(k_split_factors, dim3((unsigned)ceil_div64(tot, 256)), dim3(256), 0, s, U, S, V, M, N, k, kp,
                       us_hi, us_lo, v_hi, v_lo, out->S);
    const bf16_t* Ap = (const bf16_t*)A->ptr;
    uint8_t* ct = want_t ? out->Rt.codes : nullptr;
    uint8_t* st_ = want_t ? out->Rt.scales : nullptr;
    {
        const int rs = launch_residual_quant(s, Ap, A->ld, M, N, M, 0, us_hi, us_lo, v_hi, v_lo, kp, out->R.tscale,
                                             out->R.codes, out->R.scales, ct, st_, R_debug, SR, seed);
        if (rs != METIS_OK) return rs;
    }
    return quantize_factors(s, U, nullptr, V, M, N, k, out, SR, seed);
}

extern "C" int metis_split_quantize(void* stream, const metis_mat* A, const float* U, const float* S, const float* V,
                                    int k, metis_split* out, float* R_debug, void* workspace,
                                    size_t workspace_bytes) {
    return split_quantize_impl<false>(stream, A, U, S, V, k, 0, out, R_debug, workspace, workspace_bytes);
}

extern "C" int metis_split_quantize_sr(void* stream, const metis_mat* A, const float* U, const float* S, const float* V,
                                       int k, uint64_t seed, metis_split* out, float* R_debug, void* workspace,
                                       size_t workspace_bytes) {
    return split_quantize_impl<true>(stream, A, U, S, V, k, seed, out, R_debug, workspace, workspace_bytes);
}

// ---- variant for callers that cannot allocate ---------------------------------------------------------------
// Same kernels; the bf16 factor staging lives in a file-scope device array instead of a caller workspace.  Each
// GPU holds its own copy of the array at its own address: the address is looked up once per device (with that
// device current) and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[METIS_SPLIT_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[64];          // per device; a race between first calls only repeats the lookup

extern "C" int metis_split_quantize_static(void* stream, const metis_mat* A, const float* U, const float* S,
                                           const float* V, int k, metis_split* out, float* R_debug) {
    if (!A || k < 1 || k > 128) return METIS_INVALID_ARG;
    const size_t need = metis_split_workspace_bytes(A->rows, A->cols, k);
    if (need == 0) return METIS_BAD_SHAPE;
    if (need > (size_t)METIS_SPLIT_STATIC_SCRATCH_BYTES) return METIS_SCRATCH_TOO_SMALL;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return METIS_HIP_ERROR;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return METIS_HIP_ERROR;
        g_scratch_ptr[dev] = ptr;
    }
    // every byte the kernels read is rewritten by k_split_factors first: nothing has to start at zero
    return split_quantize_impl<false>(stream, A, U, S, V, k, 0, out, R_debug, g_scratch_ptr[dev], need);
}

// Split of a weight whose factors and residual are stored variables (Sec. 3.2): nothing is subtracted,
// the three parts go through the quantizer as they are and S is copied.
template <bool SR>
static int split_from_parts_impl(void* stream, const metis_mat* W_R, const float* U, const float* S, const float* V,
                                 int k, uint64_t seed, metis_split* out) {
    if (!W_R || !W_R->ptr || !U || !S || !V || !out) return METIS_INVALID_ARG;
    if (k < 1 || k > 128 || out->k != k || !out->S) return METIS_INVALID_ARG;
    const int64_t M = W_R->rows, N = W_R->cols;
    const bool want_t = out->Rt.codes != nullptr;
    if (!fp4_ok(out->R, M, N)) return METIS_BAD_SHAPE;
    if (want_t && (!fp4_ok(out->Rt, N, M) || out->Rt.tscale != out->R.tscale)) return METIS_BAD_SHAPE;
    if (!fp4_ok(out->Ut, k, M) || !fp4_ok(out->Vt, k, N)) return METIS_BAD_SHAPE;
    metis_fp4* rt = want_t ? &out->Rt : nullptr;
    int st = SR ? metis_quantize_sr(stream, W_R, seed, &out->R, rt) : metis_quantize(stream, W_R, &out->R, rt);
    if (st != METIS_OK) return st;
    return quantize_factors((hipStream_t)stream, U, S, V, M, N, k, out, SR, seed);
}

extern "C" int metis_split_from_parts(void* stream, const metis_mat* W_R, const float* U, const float* S,
                                      const float* V, int k, metis_split* out) {
    return split_from_parts_impl<false>(stream, W_R, U, S, V, k, 0, out);
}

extern "C" int metis_split_from_parts_sr(void* stream, const metis_mat* W_R, const float* U, const float* S,
                                         const float* V, int k, uint64_t seed, metis_split* out) {
    return split_from_parts_impl<true>(stream, W_R, U, S, V, k, seed, out);
}
