// Shared device/host helpers of the HIP path (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/metis.h"

#define METIS_WAVE 64

#define METIS_LAUNCH_CHECK()                                   \
    do {                                                       \
        if (hipGetLastError() != hipSuccess) return METIS_HIP_ERROR; \
    } while (0)

typedef uint16_t bf16_t;   // raw bfloat16 bits

// ---- optional event bracketing of the hot kernels (see metis_profile_events) ----
enum { METIS_PROF_GEMM = 0, METIS_PROF_BROADCAST = 1, METIS_PROF_RESIDUAL_QUANT = 2, METIS_PROF_QUANTIZE = 3,
       METIS_PROF_COUNT = 4 };
struct MetisProfSlot {
    hipEvent_t* start;
    hipEvent_t* stop;
    int n, next;
};
extern MetisProfSlot g_metis_prof[METIS_PROF_COUNT];
static inline int metis_prof_begin(int id, hipStream_t s) {
    MetisProfSlot& p = g_metis_prof[id];
    if (p.n <= 0) return -1;
    int i = p.next % p.n;
    (void)hipEventRecord(p.start[i], s);
    return i;
}
static inline void metis_prof_end(int id, int i, hipStream_t s) {
    if (i < 0) return;
    MetisProfSlot& p = g_metis_prof[id];
    (void)hipEventRecord(p.stop[i], s);
    p.next++;
}

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// low / high half of a dword holding two bf16
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16, round to nearest even (finite inputs)
__device__ __forceinline__ bf16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Raising a kernel's dynamic LDS limit is a driver call of tens of microseconds: remember, per device, the largest
// value already set for that kernel (one zero-initialised cache per call site).  Races only repeat the call.
struct LdsLimitCache { int bytes[16]; };
static inline bool ensure_dyn_lds(const void* fn, size_t bytes, LdsLimitCache& c) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const bool slot = dev >= 0 && dev < 16;
    if (slot && c.bytes[dev] >= (int)bytes) return true;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return false;
    if (slot) c.bytes[dev] = (int)bytes;
    return true;
}

// compute units of the current device (cached per device), 0 on error
static inline int device_cu_count() {
    static int cached[16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    const bool slot = dev >= 0 && dev < 16;
    if (slot && cached[dev] > 0) return cached[dev];
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (slot) cached[dev] = n;
    return n;
}

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// How many ways to cut the second grid dimension (1 .. max_split) when `blocks` workgroups exist along the first and
// the GPU runs `slots` workgroups at a time: the cut whose last round of workgroups is fullest, among those that
// reach at least one full round when possible; ties go to the fewest cuts (longer runs per workgroup).
static inline int64_t balanced_split(int64_t blocks, int64_t max_split, int64_t slots) {
    if (max_split < 1) max_split = 1;
    int64_t best = 1;
    double best_eff = -1.0;
    for (int64_t s = 1; s <= max_split; ++s) {
        const int64_t wgs = blocks * s, rounds = ceil_div64(wgs, slots);
        const double eff = (double)wgs / (double)(rounds * slots);
        if (eff > best_eff + 1e-9) { best_eff = eff; best = s; }
    }
    return best;
}
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- Philox4x32-10 (Salmon et al., SC'11), written from the published round function ----
struct u32x4 { uint32_t x, y, z, w; };

__host__ __device__ __forceinline__ u32x4 philox4x32_10(u32x4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32 x 32 -> 64 bit product per multiplier (a single v_mad_u64_u32) instead of separate high and
        // low halves: integer multiplies run at a quarter of the vector rate and dominate the generator
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c.x, p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c.z;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0, hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        u32x4 n;
        n.x = hi1 ^ c.y ^ k0;
        n.y = lo1;
        n.z = hi0 ^ c.w ^ k1;
        n.w = lo0;
        c = n;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

// word `w` of stream `t` under `seed`: lane w%4 of block w/4, counter (blk lo, blk hi, t, 0)
__host__ __device__ __forceinline__ u32x4 philox_block(uint64_t seed, uint32_t stream, uint64_t blk) {
    u32x4 c = {(uint32_t)blk, (uint32_t)(blk >> 32), stream, 0u};
    return philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// ---- FP8 E4M3 (bias 7, no inf, max 448) for non-negative block scales ----
__device__ __forceinline__ float e4m3_decode(uint32_t b) {
    return b >= 8u ? __uint_as_float((b + (120u << 3)) << 20) : (float)b * 0.001953125f;
}
