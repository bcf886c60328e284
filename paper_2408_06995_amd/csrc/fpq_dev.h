// Device-side pieces shared by the libfpq kernels: format parameters and the ExMy encoder.
// Section / equation numbers refer to "Low-Bitwidth Floating Point Quantization for Efficient
// High-Quality Diffusion Models" (Section IV-B: Eq. (5)-(9); Section V-B: Eq. (12)).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fpq.h"

namespace fpq {

// Quantizer parameters as the kernels take them.
struct QParams {
    int m;    // mantissa bits
    int b;    // integer bias
    int em;   // e + m (position of the sign bit)
    float c;  // max magnitude (a grid value)
};

// Code (without sign) of a clipped magnitude 0 <= a <= c, round-to-nearest, ties to even.
//
// P = max(floor(log2 a) + b, 1) is the exponent field the value falls in and s = 2^(P-b-m) the
// step of Eq. (9).  Adding C = 2^23 * s to a in fp32 makes the hardware's round-to-nearest-even
// land on a multiple of s (ulp(C) = s and a < C), so the low bits of a + C hold n = rne(a / s)
// directly (Eq. (8)).  n runs over [0, 2^m) for subnormals and [2^m, 2^(m+1)] for normals, and
// (P-1) << m plus n is the code in both cases, including the carry into the next binade.
// The outer clamp of Eq. (8) is already satisfied: a <= c, c is a grid value and rounding is
// monotone.
__device__ __forceinline__ uint32_t encode_magnitude(float a, const QParams& q)
{
    uint32_t ab = __float_as_uint(a);
    int P = max((int)(ab >> 23) - 127 + q.b, 1);
    uint32_t Cb = (uint32_t)(P - q.b - q.m + 150) << 23;
    float t = __fadd_rn(a, __uint_as_float(Cb));
    uint32_t n = __float_as_uint(t) - Cb;
    return ((uint32_t)(P - 1) << q.m) + n;
}

// Eq. (6), (9), (8) on y = fl32(x * r), r = fl32(1 / scale).  The sign bit of y (that of x) is
// kept even when the magnitude rounds to zero.  NaN is clamped to c by v_min_f32.
__device__ __forceinline__ uint32_t quantize_nearest(float x, float r, const QParams& q)
{
    float y = __fmul_rn(x, r);
    uint32_t yb = __float_as_uint(y);
    float a = fminf(__uint_as_float(yb & 0x7fffffffu), q.c);
    return ((yb >> 31) << q.em) | encode_magnitude(a, q);
}

// Eq. (12) with a fixed rounding decision h: floor towards minus infinity on the step of the
// clipped, unrounded weight, plus h steps, then the clamp.  The result is always a grid value,
// so the nearest-value encoder above returns its code unchanged.
__device__ __forceinline__ uint32_t quantize_mask(float w, float r, uint32_t h, const QParams& q)
{
    float y = __fmul_rn(w, r);
    float yc = fminf(fmaxf(y, -q.c), q.c);
    uint32_t ab = __float_as_uint(yc) & 0x7fffffffu;
    int P = max((int)(ab >> 23) - 127 + q.b, 1);
    int es = P - q.b - q.m;                                   // s = 2^es
    float s = __uint_as_float((uint32_t)(127 + es) << 23);
    float inv_s = __uint_as_float((uint32_t)(127 - es) << 23);
    float n = floorf(__fmul_rn(yc, inv_s)) + (h ? 1.0f : 0.0f);  // exact: |yc / s| < 2^(m+1)
    float qv = fminf(fmaxf(__fmul_rn(n, s), -q.c), q.c);
    uint32_t neg = (qv < 0.0f || (qv == 0.0f && (__float_as_uint(w) >> 31))) ? 1u : 0u;
    return (neg << q.em) | encode_magnitude(fabsf(qv), q);
}

// r = fl32(1 / scale) with the scale taken from device memory when a pointer is given.
__device__ __forceinline__ float inv_scale(float scale, const float* scale_dev)
{
    float s = scale_dev ? scale_dev[0] : scale;
    return __fdiv_rn(1.0f, s);
}

// Where a quantize kernel takes its per-tensor scale from: a host value, a device value, or (dynamic
// scale) the per-block partial maxima of |x| that absmax_partial_kernel left behind, in which case every
// block folds them again and derives scale = absmax / maxval itself (no launch of its own for that),
// and the first block publishes [scale, absmax] for the layer kernel that follows.
struct ScaleSrc {
    float host;
    const float* dev;
    const float* partials;
    int nparts;
    float maxval;
    float* publish;
};

// Eq. (5) decode of one code to fp32 (p = 0 row: zero and subnormals).  Exact.
__device__ __forceinline__ float decode_code(uint32_t code, int e, int m, int b)
{
    uint32_t f = code & ((1u << m) - 1u);
    uint32_t p = (code >> m) & ((1u << e) - 1u);
    float mag = p ? ldexpf(1.0f + (float)f / (float)(1u << m), (int)p - b)
                  : ldexpf((float)f, 1 - b - m);
    return ((code >> (e + m)) & 1u) ? -mag : mag;
}

}  // namespace fpq
