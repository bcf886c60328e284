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

// Plain copy, 16 bytes per lane, each block a contiguous share with four loads in flight per lane.
__global__ __launch_bounds__(256) void probe_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n4)
{
    const size_t per = (n4 + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * per;
    const size_t e = b0 + per < n4 ? b0 + per : n4;
    for (size_t i = b0 + threadIdx.x; i < e; i += 4 * 256) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < e) v[u] = src[i + u * 256];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < e) dst[i + u * 256] = v[u];
    }
}

int launch_probe(int kind, int iters, const void* src, void* dst, size_t bytes, int* grid_out, hipStream_t st)
{
    if (kind == 0 || kind == 1) {
        const int grid = 2048;       // eight workgroups per compute unit: two waves per SIMD resident, four rounds
        if (grid_out) *grid_out = grid;
        if (kind == 0)
            hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3(grid), dim3(256), 0, st, iters, static_cast<float*>(dst));
        else
            hipLaunchKernelGGL(probe_mfma_fp8_kernel, dim3(grid), dim3(256), 0, st, iters, static_cast<float*>(dst));
    } else {
        const size_t n4 = bytes / 16;
        size_t grid = (n4 + 4095) / 4096;
        grid = grid < 1 ? 1 : (grid > 4096 ? 4096 : grid);
        if (grid_out) *grid_out = (int)grid;
        hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)grid), dim3(256), 0, st, static_cast<const float4*>(src),
                           static_cast<float4*>(dst), n4);
    }
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

}  // namespace fpq
