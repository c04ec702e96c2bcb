// Small fp64 GEMM on the f64 matrix cores (v_mfma_f64_16x16x4_f64), used for the
// sample-stage contractions of the decomposition (Sec. 3.1), whose conditioning needs
// fp64 accumulation.  C[m,n] (+)= sum_k A(m,k) B(n,k) with freely strided / gathered
// operands of type bf16, fp32 or fp64; several epilogues.
#pragma once
#include "common.h"
#include <vector>

typedef double double4_t __attribute__((ext_vector_type(4)));

struct DOperand {
    const void* p;
    int64_t s_outer;             // element stride between consecutive m (resp. n)
    int64_t s_k;                 // element stride between consecutive k
    const uint32_t* map_outer;   // optional gather on the outer index
    const uint32_t* map_k;       // optional gather on the contraction index
    int nparts;                  // the operand is the sum of nparts arrays ...
    int64_t part_stride;         // ... part_stride elements apart (nparts <= 1: a single array)
};

// PART_F64: contraction chunk z stores its partial product at c + z * part_stride (no atomics: the parts are added
// afterwards in a fixed order, k_sum_parts_batch, so a result does not depend on the order workgroups finish in)
enum { EPI_STORE_F64 = 0, EPI_PART_F64 = 1, EPI_STORE_F32 = 2, EPI_STORE_SPLIT_T = 3 };

struct DEpilogue {
    void* c;                     // F64 / F32 output, element (m,n) at c[m*ldc + n]
    int64_t ldc;
    bf16_t* hi_t;                // SPLIT_T: bf16 hi/lo parts stored transposed, (m,n) at [n*ld_t + m]
    bf16_t* lo_t;
    int64_t ld_t;
    const int32_t* skip;         // optional device flag: nonzero -> the kernel returns at once
    int64_t part_stride;         // PART_F64: elements between the partial products of consecutive chunks
};

template <typename T> __device__ __forceinline__ double dload(const void* p, int64_t off);
template <> __device__ __forceinline__ double dload<bf16_t>(const void* p, int64_t off) {
    return (double)bf16_to_f32(((const bf16_t*)p)[off]);
}
template <> __device__ __forceinline__ double dload<float>(const void* p, int64_t off) {
    return (double)((const float*)p)[off];
}
template <> __device__ __forceinline__ double dload<double>(const void* p, int64_t off) {
    return ((const double*)p)[off];
}

template <typename T>
__device__ __forceinline__ double dload_sum(const DOperand& o, int64_t off) {
    double v = dload<T>(o.p, off);
    for (int p = 1; p < o.nparts; ++p) v += dload<T>(o.p, off + p * o.part_stride);
    return v;
}

#define DG_BM 32
#define DG_BN 32
#define DG_BK 32
#define DG_PAD 2

// one 32 x 32 output tile of one contraction chunk: block (bx, by, bz) of a (ceil(N/32), ceil(M/32), ksplit) grid;
// 256 threads (4 waves, each a 16x16 sub-tile)
template <typename TA, typename TB, int EPI>
__device__ __forceinline__ void dgemm_tile(const DOperand& A, const DOperand& B, int64_t M, int64_t N, int64_t K,
                                           int64_t kchunk, const DEpilogue& ep, uint32_t bx, uint32_t by, uint32_t bz) {
    __shared__ double As[DG_BK][DG_BM + DG_PAD];
    __shared__ double Bs[DG_BK][DG_BN + DG_PAD];
    if (ep.skip && *ep.skip) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t m0 = (int64_t)by * DG_BM, n0 = (int64_t)bx * DG_BN;
    const int64_t kbeg = (int64_t)bz * kchunk;
    const int64_t kend = kbeg + kchunk < K ? kbeg + kchunk : K;
    const int wm = (wave >> 1) * 16, wn = (wave & 1) * 16;
    double4_t acc = {0.0, 0.0, 0.0, 0.0};
    const bool a_kfast = A.s_k == 1 && !A.map_k, b_kfast = B.s_k == 1 && !B.map_k;

    // per-thread element slots of a stage: the outer-index part of every address is fixed for the whole
    // contraction, only the k part moves (unless k is gathered)
    int a_mm[4], a_kk[4], b_nn[4], b_kk[4];
    int64_t a_off[4], b_off[4];
    bool a_ok[4], b_ok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = tid + 256 * i;
        a_mm[i] = a_kfast ? e >> 5 : e & 31;
        a_kk[i] = a_kfast ? e & 31 : e >> 5;
        b_nn[i] = b_kfast ? e >> 5 : e & 31;
        b_kk[i] = b_kfast ? e & 31 : e >> 5;
        const int64_t m = m0 + a_mm[i], n = n0 + b_nn[i];
        a_ok[i] = m < M;
        b_ok[i] = n < N;
        const int64_t mo = a_ok[i] ? (A.map_outer ? (int64_t)A.map_outer[m] : m) : 0;
        const int64_t no = b_ok[i] ? (B.map_outer ? (int64_t)B.map_outer[n] : n) : 0;
        a_off[i] = mo * A.s_outer;
        b_off[i] = no * B.s_outer;
    }
    for (int64_t kt = kbeg; kt < kend; kt += DG_BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            {
                const int64_t k = kt + a_kk[i];
                double v = 0.0;
                if (a_ok[i] && k < kend) {
                    const int64_t ko = A.map_k ? (int64_t)A.map_k[k] : k;
                    v = dload_sum<TA>(A, a_off[i] + ko * A.s_k);
                }
                As[a_kk[i]][a_mm[i]] = v;
            }
            {
                const int64_t k = kt + b_kk[i];
                double v = 0.0;
                if (b_ok[i] && k < kend) {
                    const int64_t ko = B.map_k ? (int64_t)B.map_k[k] : k;
                    v = dload_sum<TB>(B, b_off[i] + ko * B.s_k);
                }
                Bs[b_kk[i]][b_nn[i]] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < DG_BK / 4; ++s) {
            double a = As[4 * s + (lane >> 4)][wm + (lane & 15)];
            double b = Bs[4 * s + (lane >> 4)][wn + (lane & 15)];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    // D layout of the 16x16x4 f64 instruction: lane l, element v -> row 4*v + l/16, column l%16
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        int64_t m = m0 + wm + 4 * v + (lane >> 4), n = n0 + wn + (lane & 15);
        if (m >= M || n >= N) continue;
        double x = acc[v];
        if (EPI == EPI_STORE_F64) {
            ((double*)ep.c)[m * ep.ldc + n] = x;
        } else if (EPI == EPI_PART_F64) {
            ((double*)ep.c)[(int64_t)bz * ep.part_stride + m * ep.ldc + n] = x;
        } else if (EPI == EPI_STORE_F32) {
            ((float*)ep.c)[m * ep.ldc + n] = (float)x;
        } else {
            float f = (float)x;
            bf16_t hi = f32_to_bf16_rne(f);
            float rem = f - bf16_to_f32(hi);
            bf16_t lo = f32_to_bf16_rne(rem);
            ep.hi_t[n * ep.ld_t + m] = hi;
            ep.lo_t[n * ep.ld_t + m] = lo;
            ((float*)ep.c)[m * ep.ldc + n] = bf16_to_f32(hi) + bf16_to_f32(lo);
        }
    }
}

template <typename TA, typename TB, int EPI>
__global__ void __launch_bounds__(256)
k_dgemm(DOperand A, DOperand B, int64_t M, int64_t N, int64_t K, int64_t kchunk, DEpilogue ep) {
    dgemm_tile<TA, TB, EPI>(A, B, M, N, K, kchunk, ep, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Several independent small products in one launch (the same step of several decompositions): the calls travel
// by value in the kernel arguments, call c owns the blocks [off[c], off[c+1]) of a one-dimensional grid.
#define DG_MAX_BATCH 16
struct DgemmCall {
    DOperand A, B;
    int64_t M, N, K, kchunk;
    DEpilogue ep;
    uint32_t gx, gy, gz;
};
struct DgemmBatch {
    int n;
    uint32_t off[DG_MAX_BATCH + 1];
    DgemmCall c[DG_MAX_BATCH];
};

template <typename TA, typename TB, int EPI>
__global__ void __launch_bounds__(256)
k_dgemm_batch(const DgemmBatch b) {
    const uint32_t blk = blockIdx.x;
    int c = 0;
    while (c + 1 < b.n && blk >= b.off[c + 1]) ++c;
    const DgemmCall& call = b.c[c];
    const uint32_t local = blk - b.off[c];
    const uint32_t bx = local % call.gx, by = (local / call.gx) % call.gy, bz = local / (call.gx * call.gy);
    dgemm_tile<TA, TB, EPI>(call.A, call.B, call.M, call.N, call.K, call.kchunk, call.ep, bx, by, bz);
}

// Epilogue shared by both kernels.
template <int EPI>
__device__ __forceinline__ void dgemm_store(const DEpilogue& ep, int64_t m, int64_t n, double x, uint32_t z) {
    if (EPI == EPI_STORE_F64) {
        ((double*)ep.c)[m * ep.ldc + n] = x;
    } else if (EPI == EPI_PART_F64) {
        ((double*)ep.c)[(int64_t)z * ep.part_stride + m * ep.ldc + n] = x;
    } else if (EPI == EPI_STORE_F32) {
        ((float*)ep.c)[m * ep.ldc + n] = (float)x;
    } else {
        float f = (float)x;
        bf16_t hi = f32_to_bf16_rne(f);
        float rem = f - bf16_to_f32(hi);
        bf16_t lo = f32_to_bf16_rne(rem);
        ep.hi_t[n * ep.ld_t + m] = hi;
        ep.lo_t[n * ep.ld_t + m] = lo;
        ((float*)ep.c)[m * ep.ldc + n] = bf16_to_f32(hi) + bf16_to_f32(lo);
    }
}

// Larger variant for the two contractions that touch every sampled row (sketch, projection):
// 64x64 block tile, each of the 4 waves a 32x32 tile (2x2 MFMA tiles), 32-deep stages, the next
// stage's operands in flight (registers) while the current one is multiplied, double-buffered LDS.
#define DGB_T 64
#define DGB_K 32
template <typename TA, typename TB, int EPI>
__global__ void __launch_bounds__(256)
k_dgemm_big(DOperand A, DOperand B, int64_t M, int64_t N, int64_t K, int64_t kchunk, DEpilogue ep) {
    __shared__ double As[2][DGB_K][DGB_T + DG_PAD];
    __shared__ double Bs[2][DGB_K][DGB_T + DG_PAD];
    if (ep.skip && *ep.skip) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t m0 = (int64_t)blockIdx.y * DGB_T, n0 = (int64_t)blockIdx.x * DGB_T;
    const int64_t kbeg = (int64_t)blockIdx.z * kchunk;
    const int64_t kend = kbeg + kchunk < K ? kbeg + kchunk : K;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
    double4_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (double4_t){0.0, 0.0, 0.0, 0.0};
    const bool a_kfast = A.s_k == 1 && !A.map_k, b_kfast = B.s_k == 1 && !B.map_k;
    // element e of a 64 x 32 stage: (outer, k) = (e/32, e%32) when k is the contiguous axis, else (e%64, e/64)
    double ra[8], rb[8];
    auto fetch = [&](int64_t kt) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int e = tid + 256 * i;
            {
                int mm = a_kfast ? e >> 5 : e & 63, kk = a_kfast ? e & 31 : e >> 6;
                int64_t m = m0 + mm, k = kt + kk;
                double v = 0.0;
                if (m < M && k < kend) {
                    int64_t mo = A.map_outer ? (int64_t)A.map_outer[m] : m;
                    int64_t ko = A.map_k ? (int64_t)A.map_k[k] : k;
                    v = dload_sum<TA>(A, mo * A.s_outer + ko * A.s_k);
                }
                ra[i] = v;
            }
            {
                int nn = b_kfast ? e >> 5 : e & 63, kk = b_kfast ? e & 31 : e >> 6;
                int64_t n = n0 + nn, k = kt + kk;
                double v = 0.0;
                if (n < N && k < kend) {
                    int64_t no = B.map_outer ? (int64_t)B.map_outer[n] : n;
                    int64_t ko = B.map_k ? (int64_t)B.map_k[k] : k;
                    v = dload_sum<TB>(B, no * B.s_outer + ko * B.s_k);
                }
                rb[i] = v;
            }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int e = tid + 256 * i;
            As[buf][a_kfast ? e & 31 : e >> 6][a_kfast ? e >> 5 : e & 63] = ra[i];
            Bs[buf][b_kfast ? e & 31 : e >> 6][b_kfast ? e >> 5 : e & 63] = rb[i];
        }
    };
    fetch(kbeg);
    stash(0);
    __syncthreads();
    int buf = 0;
    for (int64_t kt = kbeg; kt < kend; kt += DGB_K) {
        const bool more = kt + DGB_K < kend;
        if (more) fetch(kt + DGB_K);
#pragma unroll
        for (int s = 0; s < DGB_K / 4; ++s) {
            const int kr = 4 * s + (lane >> 4);
            double a0 = As[buf][kr][wm + (lane & 15)], a1 = As[buf][kr][wm + 16 + (lane & 15)];
            double b0 = Bs[buf][kr][wn + (lane & 15)], b1 = Bs[buf][kr][wn + 16 + (lane & 15)];
            acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                int64_t m = m0 + wm + 16 * i + 4 * v + (lane >> 4), n = n0 + wn + 16 * j + (lane & 15);
                if (m < M && n < N) dgemm_store<EPI>(ep, m, n, acc[i][j][v], blockIdx.z);
            }
}

static inline bool dgemm_is_big(int64_t M, int64_t N, int64_t K) { return M * N * K >= ((int64_t)1 << 26) && M >= 48 && N >= 48; }

// contraction chunk and number of chunks a product is launched with (ksplit = the caller's wish; only the
// PART_F64 epilogue may split)
template <int EPI>
static inline int dgemm_parts(int64_t M, int64_t N, int64_t K, int ksplit, int64_t* kchunk_out = nullptr) {
    if (ksplit < 1 || EPI != EPI_PART_F64) ksplit = 1;
    int64_t kchunk;
    if (dgemm_is_big(M, N, K)) {
        // split the contraction only as far as needed for ~512 workgroups
        const int64_t tiles = ceil_div64(M, DGB_T) * ceil_div64(N, DGB_T);
        if (EPI == EPI_PART_F64) {
            const int64_t want = ceil_div64(512, tiles), maxs = K / 128 > 0 ? K / 128 : 1;
            ksplit = (int)(want < maxs ? want : maxs);
        }
        kchunk = ceil_div64(ceil_div64(K, ksplit), DGB_K) * DGB_K;
    } else {
        kchunk = ceil_div64(ceil_div64(K, ksplit), DG_BK) * DG_BK;
    }
    if (kchunk_out) *kchunk_out = kchunk;
    return (int)ceil_div64(K, kchunk);
}

template <typename TA, typename TB, int EPI>
static inline void launch_dgemm(hipStream_t s, DOperand A, DOperand B, int64_t M, int64_t N, int64_t K,
                                int ksplit, DEpilogue ep) {
    int64_t kchunk;
    ksplit = dgemm_parts<EPI>(M, N, K, ksplit, &kchunk);
    if (dgemm_is_big(M, N, K)) {
        dim3 grid((unsigned)ceil_div64(N, DGB_T), (unsigned)ceil_div64(M, DGB_T), (unsigned)ksplit);
        hipLaunchKernelGGL((k_dgemm_big<TA, TB, EPI>), grid, dim3(256), 0, s, A, B, M, N, K, kchunk, ep);
        return;
    }
    dim3 grid((unsigned)ceil_div64(N, DG_BN), (unsigned)ceil_div64(M, DG_BM), (unsigned)ksplit);
    hipLaunchKernelGGL((k_dgemm<TA, TB, EPI>), grid, dim3(256), 0, s, A, B, M, N, K, kchunk, ep);
}


// A list of products of one kind: the small ones go out in launches of up to DG_MAX_BATCH calls, a large one
// (see launch_dgemm) on its own.
template <typename TA, typename TB, int EPI>
struct DgemmList {
    struct Item { DOperand A, B; int64_t M, N, K; int ksplit; DEpilogue ep; };
    std::vector<Item> items;
    void add(DOperand A, DOperand B, int64_t M, int64_t N, int64_t K, int ksplit, DEpilogue ep) {
        items.push_back({A, B, M, N, K, ksplit, ep});
    }
    void launch(hipStream_t s) {
        DgemmBatch b;
        b.n = 0;
        b.off[0] = 0;
        auto flush = [&]() {
            if (b.n == 0) return;
            for (int i = b.n; i < DG_MAX_BATCH; ++i) { b.c[i] = b.c[0]; b.off[i + 1] = b.off[b.n]; }
            hipLaunchKernelGGL((k_dgemm_batch<TA, TB, EPI>), dim3(b.off[b.n]), dim3(256), 0, s, b);
            b.n = 0;
        };
        for (const Item& it : items) {
            if (dgemm_is_big(it.M, it.N, it.K)) {
                launch_dgemm<TA, TB, EPI>(s, it.A, it.B, it.M, it.N, it.K, it.ksplit, it.ep);
                continue;
            }
            int64_t kchunk;
            const int ksplit = dgemm_parts<EPI>(it.M, it.N, it.K, it.ksplit, &kchunk);
            DgemmCall& c = b.c[b.n];
            c.A = it.A; c.B = it.B; c.M = it.M; c.N = it.N; c.K = it.K; c.kchunk = kchunk; c.ep = it.ep;
            c.gx = (uint32_t)ceil_div64(it.N, DG_BN);
            c.gy = (uint32_t)ceil_div64(it.M, DG_BM);
            c.gz = (uint32_t)ksplit;
            b.off[b.n + 1] = b.off[b.n] + c.gx * c.gy * c.gz;
            if (++b.n == DG_MAX_BATCH) flush();
        }
        flush();
        items.clear();
    }
};

// Sum of partial arrays in a fixed order: out[i] = sum_p parts[p * stride + i], i < n, for several independent
// calls in one launch.  Two shapes of work.  Many parts of a small array (the Gram matrices: up to a few hundred
// parts of r x r): a workgroup owns 32 consecutive elements, its 8 thread groups each add a contiguous range of the
// parts in ascending order and the 8 subtotals are added in ascending order.  Few parts of a large array (sketch,
// projection): a thread owns two consecutive elements and adds the parts in ascending order, eight loads in
// flight.  Either way the result is a function of the parts alone.
#define SUM_EB 32
#define SUM_PG 8
#define SUM_WIDE 512             // elements per workgroup in the few-parts shape
#define SUM_MAX_BATCH 24
struct SumCall {
    const double* parts;
    double* out;
    int64_t n, stride;
    int nparts;
    int wide;                    // 1: few parts of a large array
    const int32_t* skip;         // optional device flag: nonzero -> nothing is written
};
struct SumBatch {
    int n;
    uint32_t off[SUM_MAX_BATCH + 1];
    SumCall c[SUM_MAX_BATCH];
};

static __global__ void __launch_bounds__(256)
k_sum_parts_batch(const SumBatch b) {
    __shared__ double red[SUM_PG][SUM_EB];
    const uint32_t blk = blockIdx.x;
    int c = 0;
    while (c + 1 < b.n && blk >= b.off[c + 1]) ++c;
    const SumCall& call = b.c[c];
    if (call.skip && *call.skip) return;
    if (call.wide) {
        const int64_t i = ((int64_t)(blk - b.off[c]) * 256 + threadIdx.x) * 2;
        if (i >= call.n) return;
        const double* __restrict__ src = call.parts + i;
        double a0 = 0.0, a1 = 0.0;
        if (i + 1 < call.n && (call.stride & 1) == 0) {          // 16-byte loads (parts and out are 16-byte aligned)
#pragma unroll 8
            for (int p = 0; p < call.nparts; ++p) {
                const double2 v = *reinterpret_cast<const double2*>(src + (int64_t)p * call.stride);
                a0 += v.x;
                a1 += v.y;
            }
            *reinterpret_cast<double2*>(call.out + i) = make_double2(a0, a1);
        } else {
            const bool two = i + 1 < call.n;
#pragma unroll 4
            for (int p = 0; p < call.nparts; ++p) {
                a0 += src[(int64_t)p * call.stride];
                if (two) a1 += src[(int64_t)p * call.stride + 1];
            }
            call.out[i] = a0;
            if (two) call.out[i + 1] = a1;
        }
        return;
    }
    const int e = threadIdx.x % SUM_EB, g = threadIdx.x / SUM_EB;
    const int64_t i = (int64_t)(blk - b.off[c]) * SUM_EB + e;
    const int per = (call.nparts + SUM_PG - 1) / SUM_PG;
    const int p0 = g * per, p1 = p0 + per < call.nparts ? p0 + per : call.nparts;
    double acc = 0.0;
    if (i < call.n) {
        const double* __restrict__ src = call.parts + i;
#pragma unroll 4
        for (int p = p0; p < p1; ++p) acc += src[(int64_t)p * call.stride];
    }
    red[g][e] = acc;
    __syncthreads();
    if (g == 0 && i < call.n) {
        double t = red[0][e];
#pragma unroll
        for (int q = 1; q < SUM_PG; ++q) t += red[q][e];
        call.out[i] = t;
    }
}

struct SumList {
    std::vector<SumCall> items;
    void add(const double* parts, int nparts, int64_t stride, int64_t n, double* out, const int32_t* skip = nullptr) {
        // few parts of a large array: one thread adds them all; many parts: thread groups share them
        const int wide = nparts <= 24 || n >= ((int64_t)1 << 18);
        items.push_back({parts, out, n, stride, nparts, wide, skip});
    }
    void launch(hipStream_t s) {
        SumBatch b;
        b.n = 0;
        b.off[0] = 0;
        auto flush = [&]() {
            if (b.n == 0) return;
            for (int i = b.n; i < SUM_MAX_BATCH; ++i) { b.c[i] = b.c[0]; b.off[i + 1] = b.off[b.n]; }
            hipLaunchKernelGGL(k_sum_parts_batch, dim3(b.off[b.n]), dim3(256), 0, s, b);
            b.n = 0;
        };
        for (const SumCall& it : items) {
            b.c[b.n] = it;
            b.off[b.n + 1] = b.off[b.n] + (uint32_t)ceil_div64(it.n, it.wide ? SUM_WIDE : SUM_EB);
            if (++b.n == SUM_MAX_BATCH) flush();
        }
        flush();
        items.clear();
    }
};
