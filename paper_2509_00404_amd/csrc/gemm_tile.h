// Pieces shared by the matrix-core GEMM kernels: the 32x32 accumulator tile's epilogue and the
// XCD-aware workgroup -> output tile map.
#pragma once
#include "common.h"

typedef float float16_t __attribute__((ext_vector_type(16)));

namespace {

template <typename T> __device__ __forceinline__ void store_out(T* p, float v);
template <> __device__ __forceinline__ void store_out<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_out<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16_rne(v); }

// one lane's 16 values of a 32x32 accumulator tile: rows 8 (v/4) + v%4 from p, one column
template <typename T> __device__ __forceinline__ void store_tile16(T* p, int64_t ldc, const float16_t& a, float alpha);
template <> __device__ __forceinline__ void store_tile16<float>(float* p, int64_t ldc, const float16_t& a, float alpha) {
#pragma unroll
    for (int v = 0; v < 16; ++v) p[(8 * (v >> 2) + (v & 3)) * ldc] = alpha * a[v];
}
template <> __device__ __forceinline__ void store_tile16<bf16_t>(bf16_t* p, int64_t ldc, const float16_t& a, float alpha) {
    typedef __bf16 bf2_t __attribute__((ext_vector_type(2)));
    typedef float f2_t __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
        // hardware packed conversion (round to nearest even), then the two halves go to consecutive rows
        const f2_t x = {alpha * a[v], alpha * a[v + 1]};
        const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf2_t));
        bf16_t* q = p + (8 * (v >> 2) + (v & 3)) * ldc;
        q[0] = (bf16_t)(w & 0xFFFFu);
        q[ldc] = (bf16_t)(w >> 16);
    }
}

// Workgroup ids are dealt round-robin to the 8 XCDs by the hardware, and each XCD has its own L2.
// XCD x therefore gets one RM x RN region of the tile grid (when the grid splits that way) and walks it
// row-major, so the ~32 tiles it runs at a time form a block of few distinct A and B panels; without a
// fitting region every XCD takes a contiguous run of row-major tiles.
struct TileMap {
    int tiles_n;     // tiles along N
    int rm, rn;      // region shape in tiles, 0 = no regions
};

static inline TileMap make_tile_map(int64_t tiles_m, int64_t tiles_n) {
    TileMap t = {(int)tiles_n, 0, 0};
    const int64_t total = tiles_m * tiles_n;
    if (total % 8) return t;
    const int64_t per = total / 8;
    int64_t best = 0;
    for (int64_t rn = 1; rn <= tiles_n; ++rn) {          // the most square region that tiles the grid
        if (per % rn || tiles_n % rn) continue;
        const int64_t rm = per / rn;
        if (tiles_m % rm) continue;
        const int64_t cur = rn < rm ? rn : rm;
        if (cur > best) { best = cur; t.rm = (int)rm; t.rn = (int)rn; }
    }
    return t;
}

__device__ __forceinline__ void tile_coords_of(const TileMap& t, int b, int total, int& tm, int& tn);
__device__ __forceinline__ void tile_coords(const TileMap& t, int& tm, int& tn) {
    tile_coords_of(t, (int)blockIdx.x, (int)gridDim.x, tm, tn);
}
// b = position in launch order among `total` tiles
__device__ __forceinline__ void tile_coords_of(const TileMap& t, int b, int total, int& tm, int& tn) {
    if (t.rm > 0) {
        const int xcd = b & 7, local = b >> 3, regions_n = t.tiles_n / t.rn;
        tm = (xcd / regions_n) * t.rm + local / t.rn;
        tn = (xcd % regions_n) * t.rn + local % t.rn;
    } else {
        int tile = b;
        if ((total & 7) == 0) tile = (b & 7) * (total >> 3) + (b >> 3);
        tm = tile / t.tiles_n;
        tn = tile % t.tiles_n;
    }
}

}  // namespace
