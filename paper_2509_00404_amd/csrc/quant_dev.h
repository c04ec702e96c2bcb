// NVFP4 block quantizer (Sec. 2.3; value set App. C.1), device side.
// One block = 16 values held by one lane.  The scale choice compares exactly (6*s needs at
// most 6 significand bits and the tensor scale g is a power of two).  The element rule is
// round(e / (s g)) in real arithmetic, ties to the even code.  It is met through the correctly
// rounded fp32 quotient y = fl32(e / step), step = s g: rounding is monotone and the seven
// midpoints m are fp32 values, so y can only mislead by landing ON a midpoint while e != m step.
// That needs |e - m step| / (m step) <= 2^-24 / significand(m), whereas two distinct fp32 values
// near T = m step differ by at least 2^-23 / significand(T) of T (2^-24 just below a power of
// two): impossible unless T is a power of two with significand(m) = 1, i.e. m = 0.25 and step a
// power of two, where the division is exact anyway.  So no input changes a decision.
#pragma once
#include "common.h"

struct QuantParams {
    float g;        // per-tensor scale (power of two)
    float inv6g;    // ~ 1/(6 g): only used for a first guess of the block scale
};

static inline QuantParams make_quant_params(float g) {
    QuantParams q;
    q.g = g;
    q.inv6g = (1.0f / (6.0f * g)) * (1.0f - 4.0f * 1.1920929e-07f);   // biased low: see e4m3_scale_round_up
    return q;
}

// smallest E4M3 byte c (0..126) with 6*e4m3(c)*g >= amax, saturating at 126 (=448)
__device__ __forceinline__ uint32_t e4m3_scale_round_up(float amax, QuantParams qp) {
    // first guess from a product that is biased low by a few ulp: rounding up is monotone, so the guess
    // is the answer or one below it, and a single exact comparison settles it
    float q = amax * qp.inv6g;
    uint32_t c;
    if (q >= 0.015625f) {                       // normal range: keep 3 mantissa bits, round up
        uint32_t u = __float_as_uint(q) + 0xFFFFFu;
        uint32_t e = u >> 23;                   // biased fp32 exponent (q > 0: sign bit clear)
        c = ((e - 120u) << 3) | ((u >> 20) & 7u);
        c = e >= 136u ? 126u : (c > 126u ? 126u : c);
    } else {                                    // subnormal range: steps of 2^-9
        c = (uint32_t)ceilf(q * 512.0f);
    }
    if (c < 126u && 6.0f * e4m3_decode(c) * qp.g < amax) ++c;
    return c;
}

// fl32(1/step), correctly rounded, from the hardware reciprocal and one fma correction
// (step has at most 4 significant bits; checked against IEEE division for every scale in the tests)
__device__ __forceinline__ float recip_rn(float step) {
    float r0 = __builtin_amdgcn_rcpf(step);
    float e = __builtin_fmaf(-step, r0, 1.0f);
    return __builtin_fmaf(e, r0, r0);
}

// y = fl32(x / step), correctly rounded, from r = fl32(1/step): one product, the exact remainder by
// fma, one correction (Markstein: correct unless the divisor's significand is all ones; a step has
// at most 4 significant bits).  Keeps the sign of x for zeros and for r = 0 without a separate sign
// copy: the remainder is taken as d = q step - x, which is +0 whenever it vanishes (round to nearest
// gives +0 for every exact cancellation, and for x = -+0 the two terms are zeros of opposite sign),
// so the correction term d (-r) is -0 there and q - 0 keeps the sign q took from x.
__device__ __forceinline__ float quot_rn(float x, float step, float r) {
    float q = x * r;
    float d = __builtin_fmaf(q, step, -x);
    return __builtin_fmaf(d, -r, q);
}

// Quantize 16 values; returns the scale byte, writes 8 code bytes (low nibble = even element).
// Element rule: code = nearest E2M1 value of x / (e4m3(scale) * g), ties to the even code, magnitudes
// above 6 saturate, sign bit of x kept (also for zeros); taken on the correctly rounded fp32 quotient,
// which decides exactly as real arithmetic does (see the head of this file).
// The packed converter of gfx950 does the rounding, saturation and nibble packing for two values.
__device__ __forceinline__ uint32_t quantize_block16(const float (&v)[16], QuantParams qp, uint2& codes) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; i += 2) amax = fmaxf(amax, fmaxf(fabsf(v[i]), fabsf(v[i + 1])));
    const uint32_t sc = e4m3_scale_round_up(amax, qp);
    // an all-zero block (scale byte 0) keeps only the signs: r = 0 maps every element to +-0
    const float step = e4m3_decode(sc) * qp.g;
    const float r = sc == 0u ? 0.0f : recip_rn(step);
    float y[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) y[i] = quot_rn(v[i], step, r);
    uint32_t w0 = 0u, w1 = 0u;
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[0], y[1], 1.0f, 0);
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[2], y[3], 1.0f, 1);
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[4], y[5], 1.0f, 2);
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[6], y[7], 1.0f, 3);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[8], y[9], 1.0f, 0);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[10], y[11], 1.0f, 1);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[12], y[13], 1.0f, 2);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[14], y[15], 1.0f, 3);
    codes.x = w0;
    codes.y = w1;
    return sc;
}

// Stochastically rounded variant (Sec. 4, FP4 Training).  Same block scale; a = min(|x| / step, 6) in real
// arithmetic lies between two neighbouring E2M1 magnitudes lo <= a < hi and goes up with probability
// t = (a - lo) / (hi - lo): up iff u < t, u = (word >> 8) * 2^-24, word = Philox word `first_word + i` of
// `stream` for element i.  Evaluated without rounding error: the correctly rounded quotient y locates lo
// (the E2M1 spacing around y is w = 2^(max(exponent(y), 0) - 1): 0.5 below 2, then 1, then 2, and
// lo = floor(y / w) w); rem = |x| - lo step is exact in fp32 (lo step has at most 6 significant bits and
// |x| < 2 lo step) and never negative: by the argument at the head of this file y reaches a grid point only
// when the true quotient is that grid point.  Then u < t  <=>  u w step < rem, decided by the sign of one
// fused multiply-add, which is exact.  The chosen neighbour is a grid value, which the packed converter
// encodes exactly.
__device__ __forceinline__ float sr_pick(float x, float y, float step, uint32_t word) {
    const float ax = fabsf(x);
    const float a = fminf(fabsf(y), 6.0f);
    int e = (int)((__float_as_uint(a) >> 23) & 0xFFu) - 127;                   // floor(log2 a) for normal a; a < 1 -> e = 0
    e = e < 0 ? 0 : e;
    const float w = __uint_as_float((uint32_t)(126 + e) << 23);  // 2^(e-1)
    const float winv = __uint_as_float((uint32_t)(128 - e) << 23);   // 2^(1-e)
    const float lo = floorf(a * winv) * w;
    const float rem = __builtin_fmaf(-lo, step, ax);
    const float u = (float)(word >> 8) * 5.9604644775390625e-08f;    // 2^-24, exact
    const bool up = __builtin_fmaf(-(u * w), step, rem) > 0.0f;
    const float v = fminf(lo + (up ? w : 0.0f), 6.0f);           // at lo = 6 there is nowhere to go
    return __builtin_copysignf(v, y);
}

__device__ __forceinline__ uint32_t quantize_block16_sr(const float (&v)[16], QuantParams qp, uint2& codes, uint64_t seed,
                                                        uint32_t stream, uint64_t first_word /* multiple of 4 */) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; i += 2) amax = fmaxf(amax, fmaxf(fabsf(v[i]), fabsf(v[i + 1])));
    const uint32_t sc = e4m3_scale_round_up(amax, qp);
    const float step = e4m3_decode(sc) * qp.g;
    const float r = sc == 0u ? 0.0f : recip_rn(step);
    float y[16];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const u32x4 rw = philox_block(seed, stream, (first_word >> 2) + b);
        y[4 * b + 0] = sr_pick(v[4 * b + 0], quot_rn(v[4 * b + 0], step, r), step, rw.x);
        y[4 * b + 1] = sr_pick(v[4 * b + 1], quot_rn(v[4 * b + 1], step, r), step, rw.y);
        y[4 * b + 2] = sr_pick(v[4 * b + 2], quot_rn(v[4 * b + 2], step, r), step, rw.z);
        y[4 * b + 3] = sr_pick(v[4 * b + 3], quot_rn(v[4 * b + 3], step, r), step, rw.w);
    }
    uint32_t w0 = 0u, w1 = 0u;
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[0], y[1], 1.0f, 0);
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[2], y[3], 1.0f, 1);
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[4], y[5], 1.0f, 2);
    w0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w0, y[6], y[7], 1.0f, 3);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[8], y[9], 1.0f, 0);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[10], y[11], 1.0f, 1);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[12], y[13], 1.0f, 2);
    w1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w1, y[14], y[15], 1.0f, 3);
    codes.x = w0;
    codes.y = w1;
    return sc;
}
