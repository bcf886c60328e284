// Machine-ceiling probes for the benchmark: what this GPU sustains on the matrix instructions the layer kernels use
// (operands in registers, nothing else in the loop) and on a plain device copy.  The roofline fractions of the
// benchmark are quoted against the published peaks; these probes say how much of those a kernel could reach at all.
#include "fpq_host.h"
#include "gemm_common.h"

namespace fpq {

__device__ __forceinline__ uint32_t probe_hash(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// bf16 32x32x16 MFMAs, four independent accumulators per wavefront, eight random fragments per operand that rotate so
// that the operands of consecutive instructions differ (constant operands toggle fewer wires and let the part clock higher).
__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(int iters, float* __restrict__ out)
{
    union F { v8bf v; uint32_t u[4]; };
    F a[8], b[8];
    const uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 64u;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // two bf16 per word: random sign and mantissa, exponent of a value in [0.5, 2)
            a[i].u[j] = (probe_hash(seed + 8 * i + j) & 0x80ff80ffu) | 0x3f003f00u;
            b[i].u[j] = (probe_hash(seed + 8 * i + j + 32) & 0x80ff80ffu) | 0x3f003f00u;
        }
    v16f acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + j) & 7].v, b[(i + 3 * j) & 7].v, acc[j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// The 8-bit form: 32x32x64 f8f6f4 MFMAs on E4M3 operands.
__global__ __launch_bounds__(256) void probe_mfma_fp8_kernel(int iters, float* __restrict__ out)
{
    union F { v8i v; uint32_t u[8]; };
    F a[8], b[8];
    const uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 128u;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            a[i].u[j] = probe_hash(seed + 8 * i + j) & 0xbfbfbfbfu;        // exponent field below 8: magnitudes below 2, no NaN code
            b[i].u[j] = probe_hash(seed + 8 * i + j + 64) & 0xbfbfbfbfu;
        }
    v16f acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[(i + j) & 7].v, b[(i + 3 * j) & 7].v, acc[j], 0, 0, 0,
                                                                       0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// The matrix instruction together with the conversions the fp32-accumulate mode pays for it: one iteration is one
// k-step of 16 of a wave tile of MI x 5 blocks of 32 x 32, (MI + 5) fragments of eight E4M3 codes converted to bf16 in
// registers, then MI * 5 MFMAs.  Codes stay in registers (no LDS, no memory), so this is what the instruction mix of
// the layer kernels could reach at best; MI = 2 is the wave tile of the 256-row kernel, MI = 1 that of the 128-row one.
template <int MI>
__global__ __launch_bounds__(256) void probe_mfma_decode_kernel(int iters, float* __restrict__ out)
{
    uint32_t ca[MI][2], cb[5][2];
    const uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 32u;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) ca[i][j] = probe_hash(seed + 2 * i + j) & 0xbfbfbfbfu;        // no NaN code
#pragma unroll
    for (int i = 0; i < 5; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) cb[i][j] = probe_hash(seed + 8 + 2 * i + j) & 0xbfbfbfbfu;
    v16f acc[MI][5];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    const GenFmt none = {0, 0, 0};
    for (int it = 0; it < iters; ++it) {
        v8bf a[MI], b[5];
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            asm volatile("" : "+v"(ca[i][0]), "+v"(ca[i][1]));     // the codes count as new every k-step: conversions stay in the loop
            a[i] = decode8<OPK_FP8>(ca[i][0], ca[i][1], none);
        }
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            asm volatile("" : "+v"(cb[j][0]), "+v"(cb[j][1]));
            b[j] = decode8<OPK_FP8>(cb[j][0], cb[j][1], none);
        }
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < 5; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// Plain copy and plain fill, one 16-byte element per lane and no loop: many short-lived workgroups that the dispatcher
// hands out in address order measured fastest on this part (6.2 TB/s copy, 6.9 TB/s fill, against 4.8 / 5.8 for blocks
// that loop over a contiguous share), so this is the shape that stands for "what the memory system sustains".
__global__ __launch_bounds__(256) void probe_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_fill_kernel(float4* __restrict__ dst, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) dst[i] = make_float4(1.0f, 2.0f, 3.0f, 4.0f);
}

int launch_probe(int kind, int iters, const void* src, void* dst, size_t bytes, int* grid_out, hipStream_t st)
{
    if (kind == 2 || kind == 5) {
        const size_t n4 = bytes / 16;
        const size_t grid = (n4 + 255) / 256;
        if (grid > 0x7fffffffu) return FPQ_ERR_SHAPE;
        if (grid_out) *grid_out = (int)grid;
        if (kind == 2)
            hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)grid), dim3(256), 0, st, static_cast<const float4*>(src),
                               static_cast<float4*>(dst), n4);
        else
            hipLaunchKernelGGL(probe_fill_kernel, dim3((unsigned)grid), dim3(256), 0, st, static_cast<float4*>(dst), n4);
    } else {
        const int grid = 2048;       // eight workgroups per compute unit: two waves per SIMD resident, four rounds
        if (grid_out) *grid_out = grid;
        if (kind == 0)
            hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3(grid), dim3(256), 0, st, iters, static_cast<float*>(dst));
        else if (kind == 1)
            hipLaunchKernelGGL(probe_mfma_fp8_kernel, dim3(grid), dim3(256), 0, st, iters, static_cast<float*>(dst));
        else if (kind == 3)
            hipLaunchKernelGGL(probe_mfma_decode_kernel<2>, dim3(grid), dim3(256), 0, st, iters, static_cast<float*>(dst));
        else
            hipLaunchKernelGGL(probe_mfma_decode_kernel<1>, dim3(grid), dim3(256), 0, st, iters, static_cast<float*>(dst));
    }
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

}  // namespace fpq
