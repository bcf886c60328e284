// Streaming kernels of libfpq: absmax calibration, the activation quantizer (flat and
// NCHW -> channels-last), dequantize, and the offline weight quantizer / packer.
// All are HBM-bound: 16-byte coalesced loads, the ExMy encode in registers, packed stores.
#include "fpq_dev.h"
#include "fpq_host.h"

namespace fpq {

// ------------------------------------------------------------------------------ absmax

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ float block_max(float v)
{
    __shared__ float part[4];
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    v = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    __syncthreads();
    return v;
}

// r = fl32(1 / scale) for a quantize kernel (all threads of the block call this).
__device__ __forceinline__ float block_inv_scale(const ScaleSrc& s)
{
    if (s.partials == nullptr) return inv_scale(s.host, s.dev);
    float v = 0.0f;
    for (int i = threadIdx.x; i < s.nparts; i += 256) v = fmaxf(v, s.partials[i]);
    v = block_max(v);
    const float sc = (v == 0.0f) ? 1.0f : __fdiv_rn(v, s.maxval);
    if (s.publish && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) {
        s.publish[0] = sc;
        s.publish[1] = v;
    }
    return __fdiv_rn(1.0f, sc);
}

// Tensors from this many elements (64 MB of fp32) on take the contiguous-share / streaming-load kernels.
constexpr size_t kStreamElems = (size_t)16 << 20;

typedef float v4f __attribute__((ext_vector_type(4)));

// Streaming 16-byte load for the last reader of the activations (the quantize kernels): ~10 % more
// bandwidth than a plain load, and the codes just written are not displaced from the caches.  The absmax
// pass uses plain loads, so that what fits the last-level cache is still there for the quantize pass.
__device__ __forceinline__ float4 load_stream(const float4* p)
{
    const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ float max4(float v, const float4& a)
{
    return fmaxf(v, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
}

// Pass 1: each block folds one contiguous share of x into one partial maximum of |x| (contiguous shares
// and eight 16-byte loads in flight per lane measured fastest: ~6.6 TB/s against ~5.3 grid-strided).
__global__ __launch_bounds__(256) void absmax_partial_kernel(const float* __restrict__ x, size_t n,
                                                             float* __restrict__ partial)
{
    float v = 0.0f;
    if ((reinterpret_cast<uintptr_t>(x) & 15) == 0) {
        const float4* x4 = reinterpret_cast<const float4*>(x);
        const size_t n4 = n >> 2;
        const size_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const size_t b0 = (size_t)blockIdx.x * per;
        const size_t e = b0 + per < n4 ? b0 + per : n4;
        // eight loads in flight per lane whatever the length of the share (the last round is predicated)
        for (size_t base = b0 + threadIdx.x; base < e; base += 8 * 256) {
            float4 a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                a[u] = (base + u * 256 < e) ? x4[base + u * 256] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);   // plain loads: the quantize pass that follows re-reads x
#pragma unroll
            for (int u = 0; u < 8; ++u) v = max4(v, a[u]);
        }
        const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x;
        for (size_t j = (n4 << 2) + tid; j < n; j += (size_t)gridDim.x * 256) v = fmaxf(v, fabsf(x[j]));
    } else {
        const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x;
        for (size_t j = tid; j < n; j += (size_t)gridDim.x * 256) v = fmaxf(v, fabsf(x[j]));
    }
    v = block_max(v);
    if (threadIdx.x == 0) partial[blockIdx.x] = v;
}

// Pass 1 for tensors below kStreamElems: each block folds a grid-strided share of x (measured ~1 us
// faster per call than the contiguous-share kernel on the small and cache-resident tensors).
__global__ __launch_bounds__(256) void absmax_partial_strided_kernel(const float* __restrict__ x, size_t n,
                                                             float* __restrict__ partial)
{
    float v = 0.0f;
    const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * 256;
    if ((reinterpret_cast<uintptr_t>(x) & 15) == 0) {
        const float4* x4 = reinterpret_cast<const float4*>(x);
        const size_t n4 = n >> 2;
        size_t i = tid;
        for (; i + 3 * nthreads < n4; i += 4 * nthreads) {
            float4 a = x4[i], b = x4[i + nthreads], c = x4[i + 2 * nthreads], d = x4[i + 3 * nthreads];
            v = fmaxf(v, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
            v = fmaxf(v, fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w))));
            v = fmaxf(v, fmaxf(fmaxf(fabsf(c.x), fabsf(c.y)), fmaxf(fabsf(c.z), fabsf(c.w))));
            v = fmaxf(v, fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w))));
        }
        for (; i < n4; i += nthreads) {
            float4 a = x4[i];
            v = fmaxf(v, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
        }
        for (size_t j = (n4 << 2) + tid; j < n; j += nthreads) v = fmaxf(v, fabsf(x[j]));
    } else {
        for (size_t j = tid; j < n; j += nthreads) v = fmaxf(v, fabsf(x[j]));
    }
    v = block_max(v);
    if (threadIdx.x == 0) partial[blockIdx.x] = v;
}

// Pass 2: one block folds the partials and writes absmax and scale = absmax / maxval.
__global__ __launch_bounds__(256) void absmax_final_kernel(const float* __restrict__ partial, int nparts,
                                                           float maxval, float* __restrict__ absmax_out,
                                                           float* __restrict__ scale_out)
{
    float v = 0.0f;
    for (int i = threadIdx.x; i < nparts; i += 256) v = fmaxf(v, partial[i]);
    v = block_max(v);
    if (threadIdx.x == 0) {
        absmax_out[0] = v;
        if (scale_out) scale_out[0] = (v == 0.0f) ? 1.0f : __fdiv_rn(v, maxval);
    }
}

int launch_absmax_partials(const float* x, size_t n, float* partial, hipStream_t st);

int launch_absmax(const float* x, size_t n, float maxval, float* absmax_out, float* scale_out,
                  float* partial, hipStream_t st)
{
    int nparts = absmax_parts(n);
    launch_absmax_partials(x, n, partial, st);
    hipLaunchKernelGGL(absmax_final_kernel, dim3(1), dim3(256), 0, st, partial, nparts, maxval, absmax_out,
                       scale_out);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// Pass 1 alone, for the dynamic-scale path of the layer entry points (the quantize kernel folds the partials).
int launch_absmax_partials(const float* x, size_t n, float* partial, hipStream_t st)
{
    const int nparts = absmax_parts(n);
    if (nparts > 0) {
        if (n >= kStreamElems)
            hipLaunchKernelGGL(absmax_partial_kernel, dim3(nparts), dim3(256), 0, st, x, n, partial);
        else
            hipLaunchKernelGGL(absmax_partial_strided_kernel, dim3(nparts), dim3(256), 0, st, x, n, partial);
    }
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------ quantize (flat)

// Four elements per lane and step: one 16-byte streaming load, four encodes, one 4-byte (8-bit codes) or
// 2-byte (4-bit codes) store.  Each block walks one contiguous share with four loads in flight per lane.
template <bool FOUR_BIT>
__global__ __launch_bounds__(256) void quantize_vec_kernel(const float4* __restrict__ x4, size_t n4, QParams q,
                                                           ScaleSrc ss, uint8_t* __restrict__ codes)
{
    const float r = block_inv_scale(ss);
    const size_t per = (n4 + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * per;
    const size_t e = b0 + per < n4 ? b0 + per : n4;
    size_t i = b0 + threadIdx.x;
    auto emit = [&](size_t idx, const float4& v) {
        uint32_t c0 = quantize_nearest(v.x, r, q), c1 = quantize_nearest(v.y, r, q);
        uint32_t c2 = quantize_nearest(v.z, r, q), c3 = quantize_nearest(v.w, r, q);
        if (FOUR_BIT)
            reinterpret_cast<uint16_t*>(codes)[idx] = (uint16_t)(c0 | (c1 << 4) | (c2 << 8) | (c3 << 12));
        else
            reinterpret_cast<uint32_t*>(codes)[idx] = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
    };
    for (; i < e; i += 4 * 256) {   // four loads in flight per lane; the last round is predicated
        float4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < e) a[u] = load_stream(x4 + i + u * 256);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < e) emit(i + u * 256, a[u]);
    }
}

// The same for tensors below kStreamElems, grid-strided with plain loads: one 16-byte load, four encodes, one 4-byte (8-bit codes) or
// 2-byte (4-bit codes) store.  Four independent loads are kept in flight per lane.
template <bool FOUR_BIT>
__global__ __launch_bounds__(256) void quantize_vec_strided_kernel(const float4* __restrict__ x4, size_t n4, QParams q,
                                                           ScaleSrc ss, uint8_t* __restrict__ codes)
{
    const float r = block_inv_scale(ss);
    const size_t nthreads = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    auto emit = [&](size_t idx, const float4& v) {
        uint32_t c0 = quantize_nearest(v.x, r, q), c1 = quantize_nearest(v.y, r, q);
        uint32_t c2 = quantize_nearest(v.z, r, q), c3 = quantize_nearest(v.w, r, q);
        if (FOUR_BIT)
            reinterpret_cast<uint16_t*>(codes)[idx] = (uint16_t)(c0 | (c1 << 4) | (c2 << 8) | (c3 << 12));
        else
            reinterpret_cast<uint32_t*>(codes)[idx] = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
    };
    for (; i + 3 * nthreads < n4; i += 4 * nthreads) {
        float4 a = x4[i], b = x4[i + nthreads], c = x4[i + 2 * nthreads], d = x4[i + 3 * nthreads];
        emit(i, a);
        emit(i + nthreads, b);
        emit(i + 2 * nthreads, c);
        emit(i + 3 * nthreads, d);
    }
    for (; i < n4; i += nthreads) emit(i, x4[i]);
}

// One output byte per lane: any alignment, tails.  first = index of the first element handled.
template <bool FOUR_BIT>
__global__ __launch_bounds__(256) void quantize_scalar_kernel(const float* __restrict__ x, size_t first, size_t n,
                                                              QParams q, ScaleSrc ss,
                                                              uint8_t* __restrict__ codes)
{
    const float r = block_inv_scale(ss);
    const size_t per = FOUR_BIT ? 2 : 1;
    size_t j = first / per + (size_t)blockIdx.x * 256 + threadIdx.x;  // output byte
    const size_t nbytes = (n + per - 1) / per;
    const size_t nthreads = (size_t)gridDim.x * 256;
    for (; j < nbytes; j += nthreads) {
        if (FOUR_BIT) {
            uint32_t lo = quantize_nearest(x[2 * j], r, q);
            uint32_t hi = (2 * j + 1 < n) ? quantize_nearest(x[2 * j + 1], r, q) : 0u;
            codes[j] = (uint8_t)(lo | (hi << 4));
        } else {
            codes[j] = (uint8_t)quantize_nearest(x[j], r, q);
        }
    }
}

static int grid_for(size_t work_items, int per_block)
{
    size_t g = (work_items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > 4096) g = 4096;
    return (int)g;
}

int launch_quantize(const float* x, size_t n, const QParams& q, bool four_bit, const ScaleSrc& ss, uint8_t* codes,
                    hipStream_t st)
{
    if (n == 0) return FPQ_OK;
    bool aligned = (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(codes) & 3) == 0;
    size_t n4 = aligned ? (n >> 2) : 0;
    if (n4) {
        int g = grid_for(n4, 256 * 4);
        const float4* x4 = reinterpret_cast<const float4*>(x);
        if (n >= kStreamElems) {
            if (four_bit)
                hipLaunchKernelGGL(quantize_vec_kernel<true>, dim3(g), dim3(256), 0, st, x4, n4, q, ss, codes);
            else
                hipLaunchKernelGGL(quantize_vec_kernel<false>, dim3(g), dim3(256), 0, st, x4, n4, q, ss, codes);
        } else {
            if (four_bit)
                hipLaunchKernelGGL(quantize_vec_strided_kernel<true>, dim3(g), dim3(256), 0, st, x4, n4, q, ss, codes);
            else
                hipLaunchKernelGGL(quantize_vec_strided_kernel<false>, dim3(g), dim3(256), 0, st, x4, n4, q, ss, codes);
        }
    }
    size_t first = n4 << 2;
    if (first < n) {
        int g = grid_for(n - first, 256);
        if (four_bit)
            hipLaunchKernelGGL(quantize_scalar_kernel<true>, dim3(g), dim3(256), 0, st, x, first, n, q, ss, codes);
        else
            hipLaunchKernelGGL(quantize_scalar_kernel<false>, dim3(g), dim3(256), 0, st, x, first, n, q, ss, codes);
    }
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// Dynamic per-tensor scale of a tensor so small that one workgroup holds it in registers (up to 16 Ki elements: the
// time-embedding vectors of the U-Net): all loads in flight at once (sixteen 16-byte loads per lane at most), maximum
// of |x|, scale, and the codes from the registers, in one launch.  Bit-identical to the two-launch form.
__global__ __launch_bounds__(256) void quantize_dynamic_small_kernel(const float4* __restrict__ x4, int n4, QParams q,
                                                                     float maxval, float* __restrict__ publish,
                                                                     uint8_t* __restrict__ codes)
{
    float4 v[16];
    float m = 0.0f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int i = e * 256 + threadIdx.x;
        v[e] = i < n4 ? x4[i] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        m = max4(m, v[e]);
    }
    m = block_max(m);
    const float sc = (m == 0.0f) ? 1.0f : __fdiv_rn(m, maxval);
    if (threadIdx.x == 0) {
        publish[0] = sc;
        publish[1] = m;
    }
    const float r = __fdiv_rn(1.0f, sc);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int i = e * 256 + threadIdx.x;
        if (i < n4) {
            const uint32_t c0 = quantize_nearest(v[e].x, r, q), c1 = quantize_nearest(v[e].y, r, q);
            const uint32_t c2 = quantize_nearest(v[e].z, r, q), c3 = quantize_nearest(v[e].w, r, q);
            reinterpret_cast<uint32_t*>(codes)[i] = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
        }
    }
}

// FPQ_OK when the one-launch form ran, FPQ_ERR_UNSUPPORTED when it does not apply (size, alignment).
int launch_quantize_dynamic_small(const float* x, size_t n, const QParams& q, float maxval, float* publish, uint8_t* codes,
                                  hipStream_t st)
{
    if (n == 0 || n > 16384 || (n & 3) || (reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(codes) & 3))
        return FPQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(quantize_dynamic_small_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<const float4*>(x),
                       (int)(n >> 2), q, maxval, publish, codes);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ------------------------------------------------------------------- grouped dynamic-scale quantizer

// Dynamic per-tensor scales of a group of activation tensors in two launches for the whole group (blockIdx.y picks the
// problem): per-block partial maxima of |x|, then every block of the second kernel folds its problem's partials into
// scale = absmax / maxval (the same arithmetic as the single-tensor form, so the codes are the same bit for bit),
// block 0 of a problem publishes [scale, absmax] where the layer kernel reads its scale, and the elements are encoded.
// Each tensor has a multiple of 16 elements and is 16-byte aligned (rows of K % 16 == 0 codes).
__global__ __launch_bounds__(256) void absmax_grouped_kernel(const GroupedArgs g)
{
    const GroupedProblem& q = g.p[blockIdx.y];
    const float4* x4 = reinterpret_cast<const float4*>(q.x32);
    const int n4 = (q.M * q.K) >> 2;
    float v = 0.0f;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n4; i += kGroupAbsmaxParts * 256) v = max4(v, x4[i]);
    v = block_max(v);
    if (threadIdx.x == 0) q.partials[blockIdx.x] = v;
}

__global__ __launch_bounds__(256) void quantize_grouped_kernel(const GroupedArgs g, QParams qx, float maxval)
{
    const GroupedProblem& q = g.p[blockIdx.y];
    float v = threadIdx.x < kGroupAbsmaxParts ? q.partials[threadIdx.x] : 0.0f;
    v = block_max(v);
    const float sc = (v == 0.0f) ? 1.0f : __fdiv_rn(v, maxval);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        float* pub = const_cast<float*>(q.sx_dev);
        pub[0] = sc;
        pub[1] = v;
    }
    const float r = __fdiv_rn(1.0f, sc);
    const float4* x4 = reinterpret_cast<const float4*>(q.x32);
    uint32_t* codes = reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(q.xcodes));
    const int n4 = (q.M * q.K) >> 2;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n4; i += gridDim.x * 256) {
        const float4 a = x4[i];
        codes[i] = quantize_nearest(a.x, r, qx) | (quantize_nearest(a.y, r, qx) << 8) | (quantize_nearest(a.z, r, qx) << 16) |
                   (quantize_nearest(a.w, r, qx) << 24);
    }
}

int launch_quantize_dynamic_grouped(const GroupedArgs& g, const QParams& qx, float maxval, hipStream_t st)
{
    if (g.count <= 0) return FPQ_OK;
    size_t most = 0;
    for (int i = 0; i < g.count; ++i) {
        const size_t n4 = ((size_t)g.p[i].M * g.p[i].K) >> 2;
        most = n4 > most ? n4 : most;
    }
    hipLaunchKernelGGL(absmax_grouped_kernel, dim3(kGroupAbsmaxParts, (unsigned)g.count), dim3(256), 0, st, g);
    size_t gx = (most + 1023) / 1024;          // four 16-byte loads per lane
    gx = gx < 1 ? 1 : (gx > 256 ? 256 : gx);
    hipLaunchKernelGGL(quantize_grouped_kernel, dim3((unsigned)gx, (unsigned)g.count), dim3(256), 0, st, g, qx, maxval);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ------------------------------------------------------------------- quantize NCHW -> NHWC codes

// One block turns a 64-channel x 64-pixel patch of one image: reads run along pixels (contiguous in
// NCHW), the codes cross an LDS tile, writes run along channels (contiguous in [B,H,W,Cp]).
// Channels C..Cp-1 receive code 0.  Rows of the tile are 68 bytes so that the four-byte column
// groups of neighbouring pixels fall into different LDS banks.
__global__ __launch_bounds__(256) void quantize_nhwc_kernel(const float* __restrict__ x, int B, int C, int Cp, int HW,
                                                            QParams q, ScaleSrc ss, bool stream,
                                                            uint8_t* __restrict__ codes)
{
    constexpr int LDW = 68;
    __shared__ __attribute__((aligned(16))) uint8_t tile[64 * LDW];
    const float r = block_inv_scale(ss);
    // images b = blockIdx.z, blockIdx.z + gridDim.z, ... (the grid's third dimension stops at 65535)
    for (int b = blockIdx.z; b < B; b += gridDim.z) {
    const int c0 = blockIdx.y * 64;
    const int p0 = blockIdx.x * 64;
    const int pq = threadIdx.x & 15;   // pixel quad
    const int cs = threadIdx.x >> 4;   // channel within a pass
    const bool vec_ok = ((HW & 3) == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int cl = pass * 16 + cs;
        const int ch = c0 + cl;
        const int p = p0 + 4 * pq;
        uint32_t cd[4] = {0u, 0u, 0u, 0u};
        if (ch < C) {
            const float* src = x + ((size_t)b * C + ch) * (size_t)HW + p;
            if (vec_ok && p + 3 < HW) {
                const float4 v = stream ? load_stream(reinterpret_cast<const float4*>(src)) : *reinterpret_cast<const float4*>(src);
                cd[0] = quantize_nearest(v.x, r, q);
                cd[1] = quantize_nearest(v.y, r, q);
                cd[2] = quantize_nearest(v.z, r, q);
                cd[3] = quantize_nearest(v.w, r, q);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (p + j < HW) cd[j] = quantize_nearest(src[j], r, q);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) tile[(4 * pq + j) * LDW + cl] = (uint8_t)cd[j];
    }
    __syncthreads();
    const int pl = threadIdx.x >> 2;
    const int part = threadIdx.x & 3;
    const int p = p0 + pl;
    const int ch = c0 + part * 16;
    if (p < HW && ch < Cp) {
        const uint32_t* t4 = reinterpret_cast<const uint32_t*>(tile + pl * LDW + part * 16);
        uint4 v = make_uint4(t4[0], t4[1], t4[2], t4[3]);
        *reinterpret_cast<uint4*>(codes + ((size_t)b * HW + p) * (size_t)Cp + ch) = v;
    }
    __syncthreads();   // the tile is rewritten for the next image
    }
}

int launch_quantize_nhwc(const float* x, int64_t B, int64_t C, int64_t H, int64_t W, const QParams& q,
                         const ScaleSrc& ss, uint8_t* codes, hipStream_t st)
{
    int Cp = (int)padded_channels(C);
    int HW = (int)(H * W);
    dim3 grid((HW + 63) / 64, (Cp + 63) / 64, (unsigned)(B < 65535 ? B : 65535));
    hipLaunchKernelGGL(quantize_nhwc_kernel, grid, dim3(256), 0, st, x, (int)B, (int)C, Cp, HW, q, ss,
                       (size_t)B * C * H * W >= kStreamElems, codes);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------ dequantize

__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t* __restrict__ codes, size_t n, int e, int m,
                                                         int b, float scale, float* __restrict__ out)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * 256;
    for (; i < n; i += nthreads) out[i] = __fmul_rn(decode_code(codes[i], e, m, b), scale);
}

int launch_dequantize(const uint8_t* codes, size_t n, int e, int m, int b, float scale, float* out, hipStream_t st)
{
    if (n == 0) return FPQ_OK;
    hipLaunchKernelGGL(dequantize_kernel, dim3(grid_for(n, 256)), dim3(256), 0, st, codes, n, e, m, b, scale, out);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------ pack weights

// One block per output channel n.  The row's scale is its absmax / c unless given; every element
// is quantized (Eq. (12) with its mask entry, or Eq. (8) without a mask) and written to the packed
// row in (kh, kw, ci) order with ci padded to Cp and the row padded to Kpad, padding = code 0.
// A lane builds one 4-byte word of the packed row: 4 codes, or 8 codes for 4-bit formats.
template <bool FOUR_BIT>
__global__ __launch_bounds__(256) void pack_weights_kernel(const float* __restrict__ w, int Cin, int taps, int Cp,
                                                           int Kpad, QParams q, const float* __restrict__ scale_in,
                                                           const uint8_t* __restrict__ mask,
                                                           uint8_t* __restrict__ packed_rows,
                                                           float* __restrict__ scale_out,
                                                           uint8_t* __restrict__ codes_out)
{
    const int n = blockIdx.x;
    const size_t K = (size_t)Cin * taps;
    const float* row = w + (size_t)n * K;
    const uint8_t* mrow = mask ? mask + (size_t)n * K : nullptr;
    float s;
    if (scale_in) {
        s = scale_in[n];
    } else {
        float v = 0.0f;
        for (size_t i = threadIdx.x; i < K; i += 256) v = fmaxf(v, fabsf(row[i]));
        v = block_max(v);
        s = (v == 0.0f) ? 1.0f : __fdiv_rn(v, q.c);
    }
    if (threadIdx.x == 0) scale_out[n] = s;
    const float r = __fdiv_rn(1.0f, s);
    constexpr int GW = FOUR_BIT ? 8 : 4;
    const size_t row_bytes = FOUR_BIT ? (size_t)Kpad / 2 : (size_t)Kpad;
    uint32_t* dst = reinterpret_cast<uint32_t*>(packed_rows + (size_t)n * row_bytes);
    for (int g = threadIdx.x; g < Kpad / GW; g += 256) {
        const int kp0 = g * GW;
        const int tap = kp0 / Cp;
        const int ci0 = kp0 - tap * Cp;
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < GW; ++j) {
            const int ci = ci0 + j;
            uint32_t code = 0;
            if (tap < taps && ci < Cin) {
                const size_t src = (size_t)ci * taps + tap;   // [Cin, kh, kw] within the row
                code = mrow ? quantize_mask(row[src], r, mrow[src], q) : quantize_nearest(row[src], r, q);
                if (codes_out) codes_out[(size_t)n * K + src] = (uint8_t)code;
            }
            word |= code << (FOUR_BIT ? 4 * j : 8 * j);
        }
        dst[g] = word;
    }
}

int launch_pack_weights(const float* w, int64_t N, int64_t Cin, int taps, const QParams& q, bool four_bit,
                        const float* scale_in, const uint8_t* mask, uint8_t* packed_rows, float* scale_out,
                        uint8_t* codes_out, hipStream_t st)
{
    int Cp = (int)padded_channels(Cin);
    int Kpad = (int)padded_k(Cin, taps);
    if (four_bit)
        hipLaunchKernelGGL(pack_weights_kernel<true>, dim3((unsigned)N), dim3(256), 0, st, w, (int)Cin, taps, Cp, Kpad,
                           q, scale_in, mask, packed_rows, scale_out, codes_out);
    else
        hipLaunchKernelGGL(pack_weights_kernel<false>, dim3((unsigned)N), dim3(256), 0, st, w, (int)Cin, taps, Cp,
                           Kpad, q, scale_in, mask, packed_rows, scale_out, codes_out);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

}  // namespace fpq
