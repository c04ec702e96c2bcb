// Broadcast of the sampled subspace to the full batch (Sec. 3.1): C = A V0 over ALL rows of
// A, streamed once from HBM, on the bf16 matrix cores with fp32 accumulation.  V0 is given
// as two bf16 parts (hi + lo, ~16 significant bits) stored transposed [k][N], so the
// contraction runs twice per tile.  By-product: max|A|.
#include "broadcast.h"

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

#define BC_ROWS 128           // rows per workgroup (4 waves x 32)
#define BC_NC 64              // contraction elements per LDS stage
#define BC_LDB (BC_NC + 8)    // padded LDS row (bf16 elements): 144 B keeps b128 reads conflict-free

union Frag {
    uint4 u;
    bf16x8_t v;
};

// grid: (ceil(M/128), nsplit); block 256.  KT = number of 32-column tiles of V0 (k <= 32*KT).
template <int KT>
__global__ void __launch_bounds__(256)
k_broadcast(const bf16_t* __restrict__ A, int64_t lda, int64_t M, int64_t N, const bf16_t* __restrict__ V0hi,
            const bf16_t* __restrict__ V0lo, int k, int64_t nchunk, float* __restrict__ C,
            uint32_t* __restrict__ amax_bits) {
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][32 * KT][BC_LDB];   // [hi/lo][column c][n]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * BC_ROWS + wave * 32;
    const int64_t nbeg = (int64_t)blockIdx.y * nchunk;
    const int64_t nend = nbeg + nchunk < N ? nbeg + nchunk : N;
    const int half = lane >> 5;
    int64_t row = row0 + (lane & 31);
    const bool row_ok = row < M;
    if (!row_ok) row = M - 1;                 // keep loads in bounds, result discarded
    const bf16_t* arow = A + row * lda;

    float16_t acc[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    uint32_t amax2 = 0;                       // two 15-bit magnitudes tracked as packed u16 maxima

    for (int64_t n0 = nbeg; n0 < nend; n0 += BC_NC) {
        // stage V0 hi/lo for this chunk: 32*KT columns x 64 n, 16 B per thread and part
        for (int e = tid; e < 32 * KT * (BC_NC / 8); e += 256) {
            int c = e / (BC_NC / 8), seg = e % (BC_NC / 8);
            int64_t n = n0 + seg * 8;
            uint4 h = {0, 0, 0, 0}, l = {0, 0, 0, 0};
            if (c < k && n < nend) {
                h = *reinterpret_cast<const uint4*>(V0hi + (int64_t)c * N + n);
                l = *reinterpret_cast<const uint4*>(V0lo + (int64_t)c * N + n);
            }
            *reinterpret_cast<uint4*>(&Bs[0][c][seg * 8]) = h;
            *reinterpret_cast<uint4*>(&Bs[1][c][seg * 8]) = l;
        }
        // this lane's 4 x 16 B of A: contraction slots of half h are n0 + 32h + 8s .. +7
        Frag a[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            int64_t n = n0 + 32 * half + 8 * s;
            if (n < nend) a[s].u = *reinterpret_cast<const uint4*>(arow + n);
            else a[s].u = make_uint4(0, 0, 0, 0);
            uint32_t w[4] = {a[s].u.x, a[s].u.y, a[s].u.z, a[s].u.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t m = w[i] & 0x7FFF7FFFu;
                uint32_t lo = (m & 0xFFFFu) > (amax2 & 0xFFFFu) ? (m & 0xFFFFu) : (amax2 & 0xFFFFu);
                uint32_t hi = (m >> 16) > (amax2 >> 16) ? (m >> 16) : (amax2 >> 16);
                amax2 = lo | (hi << 16);
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                Frag bh, bl;
                bh.u = *reinterpret_cast<const uint4*>(&Bs[0][32 * t + (lane & 31)][32 * half + 8 * s]);
                bl.u = *reinterpret_cast<const uint4*>(&Bs[1][32 * t + (lane & 31)][32 * half + 8 * s]);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s].v, bh.v, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s].v, bl.v, acc[t], 0, 0, 0);
            }
        }
        __syncthreads();
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
    // enough workgroups to fill 256 CUs a few times over; contraction chunk a multiple of 64
    int64_t want = 1024 / (row_blocks > 1024 ? 1024 : row_blocks);
    if (want < 1) want = 1;
    int64_t nchunk = ceil_div64(ceil_div64(N, want), BC_NC) * BC_NC;
    if (nchunk < 256) nchunk = 256;
    int nsplit = (int)ceil_div64(N, nchunk);
    dim3 grid((unsigned)row_blocks, (unsigned)nsplit);
    switch (kt) {
        case 1: hipLaunchKernelGGL(k_broadcast<1>, grid, dim3(256), 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        case 2: hipLaunchKernelGGL(k_broadcast<2>, grid, dim3(256), 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        case 3: hipLaunchKernelGGL(k_broadcast<3>, grid, dim3(256), 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        case 4: hipLaunchKernelGGL(k_broadcast<4>, grid, dim3(256), 0, s, A, lda, M, N, V0hi, V0lo, k, nchunk, C, amax_bits); break;
        default: return METIS_UNSUPPORTED;
    }
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
