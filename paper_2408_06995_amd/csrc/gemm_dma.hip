// Large-tile kernel, fp32 results: instantiations, the split-K reductions and the dispatch over operand kinds.
#include "gemm_dma_kernel.h"

namespace fpq {

// y[i] = sum over slices of partial[s][i] (+ what y[i] held when the layer accumulates)
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, size_t n, int splits,
                                                            int accumulate, float* __restrict__ y)
{
    const size_t nthreads = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (((reinterpret_cast<uintptr_t>(partial) | reinterpret_cast<uintptr_t>(y)) & 15) == 0 && (n & 3) == 0) {
        const size_t n4 = n >> 2;
        for (; i < n4; i += nthreads) {
            float4 acc = reinterpret_cast<const float4*>(partial)[i];
            for (int s = 1; s < splits; ++s) {
                const float4 v = reinterpret_cast<const float4*>(partial + (size_t)s * n)[i];
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
            if (accumulate) {
                const float4 v = reinterpret_cast<const float4*>(y)[i];
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
            reinterpret_cast<float4*>(y)[i] = acc;
        }
    } else {
        for (; i < n; i += nthreads) {
            float acc = partial[i];
            for (int s = 1; s < splits; ++s) acc += partial[(size_t)s * n + i];
            if (accumulate) acc += y[i];
            y[i] = acc;
        }
    }
}

// Codes out with split-K: the row-major partial sums [splits][M, N] are added in slice order, quantized and written
// as codes [M, ldq]; a thread takes four consecutive columns of a row (one 32-bit store), columns N .. ldq - 1 get 0.
__global__ __launch_bounds__(256) void splitk_reduce_codes_kernel(const float* __restrict__ partial, int M, int N, int ldq,
                                                                  int splits, int act, QParams qy, float sy,
                                                                  const float* __restrict__ sy_dev,
                                                                  uint8_t* __restrict__ yq)
{
    const float ry = inv_scale(sy, sy_dev);
    const size_t slice = (size_t)M * N;
    const int groups = ldq >> 2;
    const size_t total = (size_t)M * groups;
    // sum over the slices of four consecutive columns of row m starting at column n (n % 4 == 0, inside the row)
    auto sum4 = [&](int m, int n, float (&v)[4]) {
        if ((N & 3) == 0 && n + 3 < N) {   // partial sums are 256-byte aligned: rows of 4 k floats keep 16-byte groups aligned
            const size_t idx = (size_t)m * N + n;
            float4 t = *reinterpret_cast<const float4*>(partial + idx);
            for (int s = 1; s < splits; ++s) {
                const float4 p = *reinterpret_cast<const float4*>(partial + (size_t)s * slice + idx);
                t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
            }
            v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = 0.0f;
                if (n + e < N) {
                    const size_t idx = (size_t)m * N + n + e;
                    v[e] = partial[idx];
                    for (int s = 1; s < splits; ++s) v[e] += partial[(size_t)s * slice + idx];
                }
            }
        }
    };
    for (size_t t = (size_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (size_t)gridDim.x * 256) {
        const int m = (int)(t / groups);
        const int n = (int)(t - (size_t)m * groups) * 4;      // output column
        float v[4];
        int valid = 4;
        if (act == FPQ_ACT_GEGLU) {
            // outputs n .. n + 3 of block n / 16: values at columns 32 (n / 16) + n % 16, gates 16 further on
            const int col = 32 * (n >> 4) + (n & 15);
            float gate[4];
            sum4(m, col, v);
            sum4(m, col + 16, gate);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] *= act_gelu(gate[e]);
        } else {
            sum4(m, n, v);
            valid = N - n < 4 ? (N - n > 0 ? N - n : 0) : 4;
            if (act == FPQ_ACT_SILU) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = act_silu(v[e]);
            }
        }
        uint32_t word = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e < valid) word |= quantize_nearest(v[e], ry, qy) << (8 * e);
        *reinterpret_cast<uint32_t*>(yq + (size_t)m * ldq + n) = word;
    }
}

int launch_splitk_reduce(const GemmArgs& a, hipStream_t st)
{
    if (a.yq) {
        const QParams qy{a.ym, a.yb, a.yem, a.yc};
        size_t grid = ((size_t)a.M * (a.ldq / 4) + 255) / 256;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(splitk_reduce_codes_kernel, dim3((unsigned)grid), dim3(256), 0, st, a.partial, a.M, a.N, a.ldq,
                           a.splits, a.act, qy, a.sy, a.sy_dev, a.yq);
    } else {
        const size_t n = (size_t)a.M * a.N;
        size_t grid = (n / 4 + 255) / 256;
        if (grid < 1) grid = 1;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)grid), dim3(256), 0, st, a.partial, n, a.splits, a.accumulate,
                           a.y);
    }
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

template <int XKIND, int WKIND, int ACC>
static int launch_dma_shape(const GemmArgs& a, hipStream_t st)
{
    if (a.tile == TILE_128x160_S2)
        return a.conv_out ? launch_dma_one<128, 160, 2, XKIND, WKIND, ACC, true, false>(a, st)
                          : launch_dma_one<128, 160, 2, XKIND, WKIND, ACC, false, false>(a, st);
    return a.conv_out ? launch_dma_one<256, 160, 3, XKIND, WKIND, ACC, true, false>(a, st)
                      : launch_dma_one<256, 160, 3, XKIND, WKIND, ACC, false, false>(a, st);
}

// Operand kinds the large-tile kernels are instantiated for.
bool gemm_dma_applicable(const GemmArgs& a)
{
    if (a.tile == TILE_GENERIC || a.kh * a.kw > 31) return false;   // tap-validity masks are 31 bits
    if (a.yq) return a.xkind == OPK_FP8 && (a.wkind == OPK_FP8 || a.wkind == OPK_FP4);   // codes out: see gemm_dma_q.hip
    if (a.acc_mode == FPQ_ACC_FP8_MFMA) return a.xkind == OPK_FP8 && (a.wkind == OPK_FP8 || a.wkind == OPK_FP4);
    return (a.xkind == OPK_FP8 && (a.wkind == OPK_FP8 || a.wkind == OPK_FP4)) ||
           (a.xkind == OPK_GENERIC8 && (a.wkind == OPK_GENERIC8 || a.wkind == OPK_GENERIC4));
}

int launch_gemm_dma(const GemmArgs& a, hipStream_t st)
{
    if (a.yq) return launch_gemm_dma_q(a, st);
    if (a.acc_mode == FPQ_ACC_FP8_MFMA) {
        if (a.xkind == OPK_FP8 && a.wkind == OPK_FP8) return launch_dma_shape<OPK_FP8, OPK_FP8, FPQ_ACC_FP8_MFMA>(a, st);
        if (a.xkind == OPK_FP8 && a.wkind == OPK_FP4) return launch_dma_shape<OPK_FP8, OPK_FP4, FPQ_ACC_FP8_MFMA>(a, st);
        return FPQ_ERR_UNSUPPORTED;
    }
    if (a.xkind == OPK_FP8 && a.wkind == OPK_FP8) return launch_dma_shape<OPK_FP8, OPK_FP8, FPQ_ACC_FP32>(a, st);
    if (a.xkind == OPK_FP8 && a.wkind == OPK_FP4) return launch_dma_shape<OPK_FP8, OPK_FP4, FPQ_ACC_FP32>(a, st);
    if (a.xkind == OPK_GENERIC8 && a.wkind == OPK_GENERIC4) return launch_dma_shape<OPK_GENERIC8, OPK_GENERIC4, FPQ_ACC_FP32>(a, st);
    if (a.xkind == OPK_GENERIC8 && a.wkind == OPK_GENERIC8) return launch_dma_shape<OPK_GENERIC8, OPK_GENERIC8, FPQ_ACC_FP32>(a, st);
    return FPQ_ERR_UNSUPPORTED;
}

}  // namespace fpq
