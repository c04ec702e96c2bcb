// NVFP4 block quantizer (Sec. 2.3; value set App. C.1), device side.
// One block = 16 values held by one lane; every comparison is exact in fp32 because
// 6*s, midpoint*s need at most 7 significand bits and the tensor scale g is a power of two.
#pragma once
#include "common.h"

struct QuantParams {
    float g;        // per-tensor scale (power of two)
    float inv6g;    // ~ 1/(6 g): only used for a first guess of the block scale
};

static inline QuantParams make_quant_params(float g) {
    QuantParams q;
    q.g = g;
    q.inv6g = 1.0f / (6.0f * g);
    return q;
}

// smallest E4M3 byte c (0..126) with 6*e4m3(c)*g >= amax, saturating at 126 (=448)
__device__ __forceinline__ uint32_t e4m3_scale_round_up(float amax, QuantParams qp) {
    float q = amax * qp.inv6g;
    uint32_t c;
    if (q >= 0.015625f) {                       // normal range: keep 3 mantissa bits, round up
        uint32_t u = __float_as_uint(q) + 0xFFFFFu;
        uint32_t e = u >> 23;                   // biased fp32 exponent (q > 0: sign bit clear)
        c = e >= 120u + 16u ? 126u : ((e - 120u) << 3) | ((u >> 20) & 7u);
        c = c > 126u ? 126u : c;
    } else {                                    // subnormal range: steps of 2^-9
        c = (uint32_t)ceilf(q * 512.0f);
    }
    // the guess came from an inexact product: settle it with exact comparisons
    if (c < 126u && 6.0f * e4m3_decode(c) * qp.g < amax) ++c;
    else if (c > 0u && 6.0f * e4m3_decode(c - 1u) * qp.g >= amax) --c;
    return c;
}

// magnitude code 0..7 of |x| for block step `step` (= e4m3(scale)*g), ties to the even code
__device__ __forceinline__ uint32_t e2m1_code(float a, float step) {
    uint32_t c = (a > 0.25f * step) ? 1u : 0u;
    c += (a >= 0.75f * step) ? 1u : 0u;
    c += (a > 1.25f * step) ? 1u : 0u;
    c += (a >= 1.75f * step) ? 1u : 0u;
    c += (a > 2.5f * step) ? 1u : 0u;
    c += (a >= 3.5f * step) ? 1u : 0u;
    c += (a > 5.0f * step) ? 1u : 0u;
    return c;
}

// Quantize 16 values; returns the scale byte, writes 8 code bytes (low nibble = even element).
__device__ __forceinline__ uint32_t quantize_block16(const float (&v)[16], QuantParams qp, uint2& codes) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
    uint32_t sc = e4m3_scale_round_up(amax, qp);
    float step = e4m3_decode(sc) * qp.g;
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        uint32_t mag = sc == 0u ? 0u : e2m1_code(fabsf(v[i]), step);
        uint32_t nib = ((__float_as_uint(v[i]) >> 28) & 8u) | mag;
        w[i >> 3] |= nib << (4 * (i & 7));
    }
    codes.x = w[0];
    codes.y = w[1];
    return sc;
}
