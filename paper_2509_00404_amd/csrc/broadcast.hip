// Broadcast of the sampled subspace to the full batch (Sec. 3.1): C = A V0 over ALL rows of
// A, streamed once from HBM, on the bf16 matrix cores with fp32 accumulation.  V0 is given
// as two bf16 parts (hi + lo, ~16 significant bits) stored transposed [k][N], so the
// contraction runs twice per tile.  By-product: max|A|.
//
// One workgroup = 8 waves = 256 rows of A and one contraction range; each wave keeps its
// 32 rows x 64 contraction elements of A for the NEXT stage in flight (registers) while it
// multiplies the current one; the V0 stage is shared through double-buffered LDS.
#include "broadcast.h"

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

#define BC_WAVES 8
#define BC_ROWS (32 * BC_WAVES)   // rows per workgroup
#define BC_NC 64                  // contraction elements per stage
#define BC_LDB (BC_NC + 8)        // padded LDS row (bf16 elements): 144 B keeps b128 accesses conflict-free
#define BC_KS (BC_NC / 16)        // MFMA steps per stage

// native vector (a HIP uint4 is a struct: arrays of it, and selects between two of them, end up in scratch)
typedef uint32_t uvec4_t __attribute__((ext_vector_type(4)));

union Frag {
    uvec4_t u;
    bf16x8_t v;
};

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
// max of two packed pairs of 16-bit magnitudes: one v_pk_max_u16
__device__ __forceinline__ uint32_t pk_umax16(uint32_t a, uint32_t b) {
    ushort2_t r = __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a), __builtin_bit_cast(ushort2_t, b));
    return __builtin_bit_cast(uint32_t, r);
}

// grid: (ceil(M/256), nsplit); block 512.  KT = number of 32-column tiles of V0 (k <= 32*KT).
// A is read with fully coalesced 16-byte loads (8 lanes cover one 128-byte row piece) and passes
// through a per-wave LDS slice to reach the MFMA operand layout; loading each lane's operand
// fragment directly would touch every cache line 4-8 times with 16 bytes each.
template <int KT>
__global__ void __launch_bounds__(64 * BC_WAVES)
k_broadcast(const bf16_t* __restrict__ A, int64_t lda, int64_t M, int64_t N, const bf16_t* __restrict__ V0hi,
            const bf16_t* __restrict__ V0lo, int k, float* __restrict__ Cpart, uint32_t* __restrict__ amax_bits) {
    constexpr int NT = 64 * BC_WAVES;
    constexpr int BVEC = 2 * 32 * KT * (BC_NC / 8) / NT;                     // 16-byte V0 vectors per thread
    static_assert(BVEC * NT == 2 * 32 * KT * (BC_NC / 8), "a V0 stage is a whole number of vectors per thread");
    constexpr int BC_DEPTH = KT <= 2 ? 3 : 2;                                // stages of A and V0 kept in flight in registers
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][2][32 * KT][BC_LDB];  // [buffer][hi/lo][column][n]
    __shared__ __attribute__((aligned(16))) bf16_t As[BC_WAVES][32][BC_LDB];   // per-wave slice of A
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * BC_ROWS + wave * 32;
    // contraction stages are dealt round-robin to the gridDim.y workgroups of a row block, so that the
    // workgroups running side by side read neighbouring pieces of the same rows (DRAM page locality)
    const int64_t nstride = (int64_t)gridDim.y * BC_NC;
    const int64_t nbeg = (int64_t)blockIdx.y * BC_NC;
    const int li = lane & 31, half = lane >> 5;
    const int lrow = lane >> 3, piece = lane & 7;           // coalesced load: 8 rows x 128 B per instruction

    float16_t acc[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    uint32_t amax2 = 0;                       // two 15-bit magnitudes tracked as packed u16 maxima

    const bf16_t* aptr[4];
    bool aok[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int64_t r = row0 + 8 * q + lrow;
        aok[q] = r < M;
        aptr[q] = A + (aok[q] ? r : M - 1) * lda + 8 * piece;
    }
    const int64_t nst = nbeg < N ? (N - nbeg + nstride - 1) / nstride : 0;     // stages of this workgroup
    // Every load is unconditional, so that the compiler can count the loads in flight and wait for
    // exactly the stage it needs: a lane with nothing to read (row or column past the end, stage past
    // the last) loads the first 16 bytes of the array instead, and its value becomes zero on the way
    // into LDS.
    const uvec4_t zero4 = {0u, 0u, 0u, 0u};
    auto a_valid = [&](int64_t i) { return i < nst && nbeg + i * nstride + 8 * piece < N; };
    auto load_a = [&](int64_t i, uvec4_t (&a)[4]) {
        const bool in = a_valid(i);
        const int64_t n0 = nbeg + i * nstride;
#pragma unroll
        for (int q = 0; q < 4; ++q) a[q] = *reinterpret_cast<const uvec4_t*>((in && aok[q]) ? aptr[q] + n0 : A);
    };
    auto load_b = [&](int64_t i, uvec4_t (&b)[BVEC]) {
        const int64_t n0 = nbeg + i * nstride;
#pragma unroll
        for (int v = 0; v < BVEC; ++v) {
            int e = tid + NT * v;
            int part = e / (32 * KT * (BC_NC / 8));
            int r = e % (32 * KT * (BC_NC / 8));
            int c = r / (BC_NC / 8), seg = r % (BC_NC / 8);
            int64_t n = n0 + seg * 8;
            const bool ok = c < k && i < nst && n < N;
            b[v] = *reinterpret_cast<const uvec4_t*>(ok ? (part ? V0lo : V0hi) + (int64_t)c * N + n : V0hi);
        }
    };
    auto store_b = [&](int buf, const uvec4_t (&b)[BVEC], int64_t i) {
        const int64_t n0 = nbeg + i * nstride;
#pragma unroll
        for (int v = 0; v < BVEC; ++v) {
            int e = tid + NT * v;
            int part = e / (32 * KT * (BC_NC / 8));
            int r = e % (32 * KT * (BC_NC / 8));
            int c = r / (BC_NC / 8), seg = r % (BC_NC / 8);
            const bool ok = c < k && i < nst && n0 + seg * 8 < N;
            *reinterpret_cast<uvec4_t*>(&Bs[buf][part][c][seg * 8]) = ok ? b[v] : zero4;
        }
    };
    auto store_a = [&](const uvec4_t (&a)[4], int64_t i) {
        const bool in = a_valid(i);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uvec4_t x = (in && aok[q]) ? a[q] : zero4;
            *reinterpret_cast<uvec4_t*>(&As[wave][8 * q + lrow][8 * piece]) = x;
            // |x| as 15-bit patterns, compared as unsigned 16-bit integers
            amax2 = pk_umax16(amax2, pk_umax16(x.x & 0x7FFF7FFFu, x.y & 0x7FFF7FFFu));
            amax2 = pk_umax16(amax2, pk_umax16(x.z & 0x7FFF7FFFu, x.w & 0x7FFF7FFFu));
        }
    };
    int buf = 0;
    // one stage: multiply what is in LDS, then move the next stage from its registers into LDS
    auto multiply = [&]() {
#pragma unroll
        for (int s = 0; s < BC_KS; ++s) {
            Frag a;
            a.u = *reinterpret_cast<const uvec4_t*>(&As[wave][li][16 * s + 8 * half]);
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                Frag bh, bl;
                bh.u = *reinterpret_cast<const uvec4_t*>(&Bs[buf][0][32 * t + li][16 * s + 8 * half]);
                bl.u = *reinterpret_cast<const uvec4_t*>(&Bs[buf][1][32 * t + li][16 * s + 8 * half]);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bh.v, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bl.v, acc[t], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    // Register ring: the loads of stages i+1 .. i+BC_DEPTH are in flight while stage i is multiplied.
    uvec4_t ra[BC_DEPTH][4], rb[BC_DEPTH][BVEC];
#pragma unroll
    for (int j = 0; j < BC_DEPTH; ++j) {
        load_a(j, ra[j]);
        load_b(j, rb[j]);
    }
    store_a(ra[0], 0);
    store_b(0, rb[0], 0);
    __syncthreads();
    // whole groups of BC_DEPTH stages, branch-free (a stage past the last is stored as zeros and never used)
    int64_t base = 0;
    for (; base + BC_DEPTH <= nst; base += BC_DEPTH) {
#pragma unroll
        for (int j = 0; j < BC_DEPTH; ++j) {
            const int64_t i = base + j;
            // slot j held stage i (now in LDS): refill it with stage i + BC_DEPTH
            load_a(i + BC_DEPTH, ra[j]);
            load_b(i + BC_DEPTH, rb[j]);
            multiply();
            store_a(ra[(j + 1) % BC_DEPTH], i + 1);
            store_b(buf ^ 1, rb[(j + 1) % BC_DEPTH], i + 1);
            __syncthreads();
            buf ^= 1;
        }
    }
    // the last nst % BC_DEPTH stages: everything they need is already in registers or in LDS
#pragma unroll
    for (int j = 0; j < BC_DEPTH - 1; ++j) {
        const int64_t i = base + j;
        if (i < nst) {
            multiply();
            store_a(ra[j + 1], i + 1);
            store_b(buf ^ 1, rb[j + 1], i + 1);
            __syncthreads();
            buf ^= 1;
        }
    }
    // D layout 32x32: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32.
    // Each contraction split writes its own partial C (plain stores); the consumers add the parts.
    float* __restrict__ P = Cpart + (size_t)blockIdx.y * (size_t)M * k;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        int c = 32 * t + li;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int64_t r = row0 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (r < M && c < k) P[r * k + c] = acc[t][v];
        }
    }
    if (amax_bits) {                          // kernel argument: the branch is uniform
        uint32_t m = (amax2 & 0xFFFFu) > (amax2 >> 16) ? (amax2 & 0xFFFFu) : (amax2 >> 16);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            uint32_t other = __shfl_xor(m, o);
            m = other > m ? other : m;
        }
        // One atomic per workgroup at most, and none when the stored maximum already covers it: thousands
        // of atomics on one address at the end of the kernel take longer than the whole pass over A.
        __shared__ uint32_t wmax[BC_WAVES];
        if (lane == 0) wmax[wave] = m;
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 1; w < BC_WAVES; ++w) m = wmax[w] > m ? wmax[w] : m;
            const uint32_t bits = m << 16;        // fp32 bit pattern of the bf16 magnitude
            if (bits > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_bits, bits);
        }
    }
}

int broadcast_splits(int64_t M, int64_t N) {
    const int64_t row_blocks = ceil_div64(M, BC_ROWS);
    // one workgroup (8 waves) per CU at a time; every workgroup at least two stages deep, at most 16 partial
    // results; the number of contraction splits that fills the last round of workgroups best
    const int64_t stages = ceil_div64(N, BC_NC);
    int64_t max_split = stages / 2;
    if (max_split > 16) max_split = 16;
    return (int)balanced_split(row_blocks, max_split, 256);
}

int launch_broadcast(hipStream_t s, const bf16_t* A, int64_t lda, int64_t M, int64_t N, const bf16_t* V0hi,
                     const bf16_t* V0lo, int k, float* Cpart, uint32_t* amax_bits) {
    const int kt = (k + 31) / 32;
    dim3 grid((unsigned)ceil_div64(M, BC_ROWS), (unsigned)broadcast_splits(M, N));
    dim3 block(64 * BC_WAVES);
    switch (kt) {
        case 1: hipLaunchKernelGGL(k_broadcast<1>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, Cpart, amax_bits); break;
        case 2: hipLaunchKernelGGL(k_broadcast<2>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, Cpart, amax_bits); break;
        case 3: hipLaunchKernelGGL(k_broadcast<3>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, Cpart, amax_bits); break;
        case 4: hipLaunchKernelGGL(k_broadcast<4>, grid, block, 0, s, A, lda, M, N, V0hi, V0lo, k, Cpart, amax_bits); break;
        default: return METIS_UNSUPPORTED;
    }
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}
