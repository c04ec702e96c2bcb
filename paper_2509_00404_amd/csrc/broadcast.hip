// Broadcast of the sampled subspace to the full batch (Sec. 3.1): C = A V0 over ALL rows of
// A, streamed once from HBM, on the bf16 matrix cores with fp32 accumulation.  V0 is given
// as two bf16 parts (hi + lo, ~16 significant bits) stored transposed [k][N], so the
// contraction runs twice per tile.  By-product: max|A|.
//
// One workgroup = 8 waves = 256 rows of A and one contraction range; each wave keeps its
// 32 rows x 128 contraction elements of A for the NEXT stage in flight (registers) while it
// multiplies the current one; the V0 stage is shared through double-buffered LDS.
#include "broadcast.h"

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

#define BC_WAVES 8
#define BC_ROWS (32 * BC_WAVES)   // rows per workgroup
#define BC_NC 128                 // contraction elements per stage
#define BC_LDB (BC_NC + 8)        // padded LDS row (bf16 elements): +16 B keeps b128 reads conflict-free
#define BC_KS (BC_NC / 16)        // MFMA steps per stage

union Frag {
    uint4 u;
    bf16x8_t v;
};

__device__ __forceinline__ uint32_t pk_umax16(uint32_t a, uint32_t b) {
    uint32_t lo = (a & 0xFFFFu) > (b & 0xFFFFu) ? (a & 0xFFFFu) : (b & 0xFFFFu);
    uint32_t hi = (a >> 16) > (b >> 16) ? (a >> 16) : (b >> 16);
    return lo | (hi << 16);
}

// grid: (ceil(M/256), nsplit); block 512.  KT = number of 32-column tiles of V0 (k <= 32*KT).
template <int KT>
__global__ void __launch_bounds__(64 * BC_WAVES)
k_broadcast(const bf16_t* __restrict__ A, int64_t lda, int64_t M, int64_t N, const bf16_t* __restrict__ V0hi,
            const bf16_t* __restrict__ V0lo, int k, int64_t nchunk, float* __restrict__ C,
            uint32_t* __restrict__ amax_bits) {
    constexpr int NT = 64 * BC_WAVES;
    constexpr int BVEC = (2 * 32 * KT * (BC_NC / 8) + NT - 1) / NT;          // 16-byte V0 vectors per thread
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][2][32 * KT][BC_LDB];  // [buffer][hi/lo][column][n]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * BC_ROWS + wave * 32;
    const int64_t nbeg = (int64_t)blockIdx.y * nchunk;
    const int64_t nend = nbeg + nchunk < N ? nbeg + nchunk : N;
    const int half = lane >> 5;
    int64_t row = row0 + (lane & 31);
    const bool row_ok = row < M;
    if (!row_ok) row = M - 1;                 // keep loads in bounds, result discarded
    const bf16_t* arow = A + row * lda + (BC_NC / 2) * half;   // each lane reads BC_NC bytes contiguous per stage

    float16_t acc[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    uint32_t amax2 = 0;                       // two 15-bit magnitudes tracked as packed u16 maxima

    // this lane's BC_KS x 16 B of A per stage: contraction slots of half h are n0 + 64h + 8s .. +7
    auto load_a = [&](int64_t n0, Frag (&a)[BC_KS]) {
#pragma unroll
        for (int s = 0; s < BC_KS; ++s) {
            int64_t n = n0 + (BC_NC / 2) * half + 8 * s;
            a[s].u = n < nend ? *reinterpret_cast<const uint4*>(arow + n0 + 8 * s) : make_uint4(0, 0, 0, 0);
        }
    };
    auto load_b = [&](int64_t n0, uint4 (&b)[BVEC]) {
#pragma unroll
        for (int v = 0; v < BVEC; ++v) {
            int e = tid + NT * v;
            int part = e / (32 * KT * (BC_NC / 8));
            int r = e % (32 * KT * (BC_NC / 8));
            int c = r / (BC_NC / 8), seg = r % (BC_NC / 8);
            int64_t n = n0 + seg * 8;
            b[v] = make_uint4(0, 0, 0, 0);
            if (part < 2 && c < k && n < nend)
                b[v] = *reinterpret_cast<const uint4*>((part ? V0lo : V0hi) + (int64_t)c * N + n);
        }
    };
    auto store_b = [&](int buf, const uint4 (&b)[BVEC]) {
#pragma unroll
        for (int v = 0; v < BVEC; ++v) {
            int e = tid + NT * v;
            int part = e / (32 * KT * (BC_NC / 8));
            int r = e % (32 * KT * (BC_NC / 8));
            int c = r / (BC_NC / 8), seg = r % (BC_NC / 8);
            if (part < 2) *reinterpret_cast<uint4*>(&Bs[buf][part][c][seg * 8]) = b[v];
        }
    };

    Frag a_cur[BC_KS], a_nxt[BC_KS];
    uint4 b_nxt[BVEC];
    load_a(nbeg, a_cur);
    load_b(nbeg, b_nxt);
    store_b(0, b_nxt);
    __syncthreads();
    int buf = 0;
    for (int64_t n0 = nbeg; n0 < nend; n0 += BC_NC) {
        const bool more = n0 + BC_NC < nend;
        if (more) {
            load_a(n0 + BC_NC, a_nxt);
            load_b(n0 + BC_NC, b_nxt);
        }
#pragma unroll
        for (int s = 0; s < BC_KS; ++s) {
            amax2 = pk_umax16(amax2, a_cur[s].u.x & 0x7FFF7FFFu);
            amax2 = pk_umax16(amax2, a_cur[s].u.y & 0x7FFF7FFFu);
            amax2 = pk_umax16(amax2, a_cur[s].u.z & 0x7FFF7FFFu);
            amax2 = pk_umax16(amax2, a_cur[s].u.w & 0x7FFF7FFFu);
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                Frag bh, bl;
                bh.u = *reinterpret_cast<const uint4*>(&Bs[buf][0][32 * t + (lane & 31)][(BC_NC / 2) * half + 8 * s]);
                bl.u = *reinterpret_cast<const uint4*>(&Bs[buf][1][32 * t + (lane & 31)][(BC_NC / 2) * half + 8 * s]);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur[s].v, bh.v, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur[s].v, bl.v, acc[t], 0, 0, 0);
            }
        }
        if (more) {
            store_b(buf ^ 1, b_nxt);
#pragma unroll
            for (int s = 0; s < BC_KS; ++s) a_cur[s] = a_nxt[s];
        }
        __syncthreads();
        buf ^= 1;
    }
    // D layout 32x32: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        int c = 32 * t + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int64_t r = row0 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (r < M && c < k) unsafeAtomicAdd(&C[r * k + c], acc[t][v]);
        }
    }
    if (amax_bits) {
        uint32_t m = (amax2 & 0xFFFFu) > (amax2 >> 16) ? (amax2 & 0xFFFFu) : (amax2 >> 16);
        if (!row_ok) m = 0;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            uint32_t other = __shfl_xor(m, o);
            m = other > m ? other : m;
        }
        if (lane == 0) atomicMax(amax_bits, m << 16);     // fp32 bit pattern of the bf16 magnitude
    }
}

int launch_broadcast(hipStream_t s, const bf16_t* A, int64_t lda, int64_t M, int64_t N, const bf16_t* V0hi,
                     const bf16_t* V0lo, int k, float* C, uint32_t* amax_bits) {
    const int kt = (k + 31) / 32;
    int64_t row_blocks = ceil_div64(M, BC_ROWS);
    // about 1.5 workgroups (12 waves) per CU, but at least four stages per workgroup: every extra
    // contraction split costs one more fp32 atomic per output element
    int64_t want = ceil_div64(384, row_blocks);
    int64_t nchunk = ceil_div64(ceil_div64(N, want), BC_NC) * BC_NC;
    if (nchunk < 4 * BC_NC) nchunk = 4 * BC_NC;
    int nsplit = (int)ceil_div64(N, nchunk);
    dim3 grid((unsigned)row_blocks, (unsigned)nsplit);
    dim3 block(64 * BC_WAVES);
    switch (kt) {
        case 1: hipLaunchKernelGGL(k_broadcast<1>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        case 2: hipLaunchKernelGGL(k_broadcast<2>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        case 3: hipLaunchKernelGGL(k_broadcast<3>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        case 4: hipLaunchKernelGGL(k_broadcast<4>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        default: return METIS_UNSUPPORTED;
    }
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
