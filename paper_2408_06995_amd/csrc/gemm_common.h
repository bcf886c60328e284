// Device helpers shared by the GEMM / implicit-GEMM kernels of libfpq: LDS tile geometry and the
// code -> bf16 decoders (Eq. (5) of the paper, with the subnormal row of Eq. (9)).
#pragma once
#include "fpq_dev.h"
#include "fpq_host.h"

namespace fpq {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------- activations (codes out)

// x * sigmoid(x) with the hardware exponential and reciprocal: relative error below 1e-6.  For very negative x the
// exponential overflows to +inf and the product is -0: the exact value is below the smallest fp32 number there.
__device__ __forceinline__ float act_silu(float x) { return x * __frcp_rn(1.0f + __expf(-x)); }

// g * Phi(g), Phi the standard normal distribution function = 1 - erfc(g / sqrt 2) / 2, with
// erfc(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2), t = 1 / (1 + p z), z >= 0 (Abramowitz & Stegun
// 7.1.26, absolute error of the formula 1.5e-7); the negative side uses Phi(g) = erfc(|g| / sqrt 2) / 2 directly, so
// nothing cancels.  Absolute error of the result below 4e-7 |g|.
__device__ __forceinline__ float act_gelu(float g)
{
    const float z = fabsf(g) * 0.70710678118654752f;
    const float t = __frcp_rn(fmaf(0.3275911f, z, 1.0f));
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    const float half_erfc = 0.5f * t * p * __expf(-z * z);     // Phi(-|g|)
    return g * (g < 0.0f ? half_erfc : 1.0f - half_erfc);
}

// The same as real function calls, for the rarely taken, fully unrolled element-wise paths (edge tiles, the
// register-staged kernels), where inlining them a few hundred times over makes the kernels spill.
__device__ __attribute__((noinline)) float act_silu_call(float x) { return act_silu(x); }
__device__ __attribute__((noinline)) float act_gelu_call(float g) { return act_gelu(g); }

// The value of the lane 16 away inside each group of 32 lanes (ds_swizzle, bit-mask mode: xor 0x10).
__device__ __forceinline__ float lane_xor16(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
}

// ---------------------------------------------------------------------------------- LDS geometry

// Byte offset of 16-byte chunk c of a tile row.  Rows are ROWB (128 or 64) bytes; the chunk index
// is xor-ed with bits of the row so that the lanes of a half-wave, which read the same chunk of 32
// consecutive rows, spread over all LDS banks.
template <int ROWB>
__device__ __forceinline__ int lds_off(int row, int c)
{
    if (ROWB == 128) return row * 128 + ((c ^ ((row >> 1) & 7)) << 4);
    return row * 64 + ((c ^ ((row >> 2) & 3)) << 4);
}

// ---------------------------------------------------------------------------------- code -> bf16

// Eight codes (two dwords for one-code-per-byte operands, one dword for 4-bit operands) to the
// bf16x8 fragment of one MFMA k-step.  KIND selects the decoder.
struct GenFmt {
    int e, m, b;
};

__device__ __forceinline__ uint32_t generic_pair(uint32_t c0, uint32_t c1, const GenFmt& f)
{
    // fp32 bit pattern with the code's exponent/mantissa fields in place has the value
    // 2^(p-127) (1 + f/2^m) for p >= 1 and the fp32 subnormal f 2^(-126-m) for p = 0; multiplying by
    // 2^(127-b) (as 2^64 * 2^(63-b), both representable for |b| <= 64) yields Eq. (5) and its
    // subnormal row alike.  The result has at most 7 significant bits, so the upper half of the
    // fp32 word is its exact bf16.
    const uint32_t magmask = (1u << (f.e + f.m)) - 1u;
    const float k1 = __uint_as_float((uint32_t)(127 + 64) << 23);        // 2^64
    const float k2 = __uint_as_float((uint32_t)(127 + 63 - f.b) << 23);  // 2^(63-b)
    float v0 = __uint_as_float((c0 & magmask) << (23 - f.m)) * k1 * k2;
    float v1 = __uint_as_float((c1 & magmask) << (23 - f.m)) * k1 * k2;
    uint32_t b0 = (__float_as_uint(v0) >> 16) | (((c0 >> (f.e + f.m)) & 1u) << 15);
    uint32_t b1 = (__float_as_uint(v1) >> 16) | (((c1 >> (f.e + f.m)) & 1u) << 15);
    return b0 | (b1 << 16);
}

template <int KIND>
__device__ __forceinline__ v8bf decode8(uint32_t lo, uint32_t hi, const GenFmt& f)
{
    union {
        v8bf v;
        v2bf p[4];
        uint32_t u[4];
    } o;
    if constexpr (KIND == OPK_FP8) {
        o.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
        o.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
        o.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
        o.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
    } else if constexpr (KIND == OPK_BF8) {
        o.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(lo, 1.0f, false);
        o.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(lo, 1.0f, true);
        o.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(hi, 1.0f, false);
        o.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_bf8(hi, 1.0f, true);
    } else if constexpr (KIND == OPK_FP4) {   // eight 4-bit codes in lo
        o.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(lo, 1.0f, 0);
        o.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(lo, 1.0f, 1);
        o.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(lo, 1.0f, 2);
        o.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(lo, 1.0f, 3);
    } else if constexpr (KIND == OPK_GENERIC8) {
        o.u[0] = generic_pair(lo & 0xffu, (lo >> 8) & 0xffu, f);
        o.u[1] = generic_pair((lo >> 16) & 0xffu, lo >> 24, f);
        o.u[2] = generic_pair(hi & 0xffu, (hi >> 8) & 0xffu, f);
        o.u[3] = generic_pair((hi >> 16) & 0xffu, hi >> 24, f);
    } else {   // OPK_GENERIC4: eight 4-bit codes in lo
        o.u[0] = generic_pair(lo & 0xfu, (lo >> 4) & 0xfu, f);
        o.u[1] = generic_pair((lo >> 8) & 0xfu, (lo >> 12) & 0xfu, f);
        o.u[2] = generic_pair((lo >> 16) & 0xfu, (lo >> 20) & 0xfu, f);
        o.u[3] = generic_pair((lo >> 24) & 0xfu, lo >> 28, f);
    }
    return o.v;
}

constexpr bool kind_is_4bit(int k) { return k == OPK_FP4 || k == OPK_GENERIC4; }
// Format selector of the f8f6f4 MFMA: 0 = E4M3, 1 = E5M2, 4 = E2M1.
constexpr int mfma_fmt(int k) { return k == OPK_FP8 ? 0 : (k == OPK_BF8 ? 1 : 4); }

}  // namespace fpq
