// Gradient-based rounding learning for low-bitwidth weights (Section V-B, Eq. (10)-(14)): one gradient-descent step
// on the per-weight parameters alpha of a linear layer, on calibration activations in full precision.
//
//   y' = clamp(fl32(W * fl32(1 / sw[n])), -c, c),  s = step of Eq. (9) at y',  fl = floor(y' / s)
//   Wq(alpha) = clamp(s (fl + sigmoid(alpha)), -c, c) * sw[n]                                   (Eq. (12), soft)
//   loss = mean((A Wq^T - A W^T)^2) + reg_weight * mean(1 - (2 |sigmoid(alpha) - 0.5|)^20)     (Eq. (11), (13), (14))
//
// The step runs as: D = Wq(alpha) - W (elementwise, with the regulariser's sum);  R = A D^T (the output error
// A Wq^T - A W^T in one product);  mse = mean(R^2);  G = (2 / (M N)) R^T A = d mse / d Wq;
// alpha -= lr (G * dWq/dalpha + reg_weight * dreg/dalpha).  The two products are dense fp32 contractions on the
// fp32 matrix instruction (32x32x2), through one LDS-tiled kernel that takes either operand layout.
#include "fpq_dev.h"
#include "fpq_host.h"

namespace fpq {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float sigmoid_f(float a) { return 1.0f / (1.0f + expf(-a)); }

// The weight on the format's axis: clipped value y', step s of Eq. (9) (a power of two) and floor(y' / s).
struct OnAxis {
    float yc, s, fl;
};
__device__ __forceinline__ OnAxis on_axis(float w, float r, const QParams& q)
{
    OnAxis o;
    o.yc = fminf(fmaxf(__fmul_rn(w, r), -q.c), q.c);
    const uint32_t ab = __float_as_uint(o.yc) & 0x7fffffffu;
    const int P = max((int)(ab >> 23) - 127 + q.b, 1);
    const int es = P - q.b - q.m;
    o.s = __uint_as_float((uint32_t)(127 + es) << 23);
    o.fl = floorf(__fmul_rn(o.yc, __uint_as_float((uint32_t)(127 - es) << 23)));   // exact: |y' / s| < 2^(m+1)
    return o;
}

__device__ __forceinline__ float block_sum(float v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    __shared__ float wsum[4];
    __syncthreads();
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
    __syncthreads();
    return wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// D = Wq(alpha) - W and the per-block sums of the regulariser 1 - (2 |sigmoid - 0.5|)^20.
__global__ __launch_bounds__(256) void rl_soft_kernel(const float* __restrict__ w, const float* __restrict__ sw,
                                                      const float* __restrict__ alpha, size_t n, int K, QParams q,
                                                      float* __restrict__ d, float* __restrict__ reg_partial)
{
    float reg = 0.0f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float s_n = sw[i / K];
        const OnAxis o = on_axis(w[i], __fdiv_rn(1.0f, s_n), q);
        const float sg = sigmoid_f(alpha[i]);
        const float qv = fminf(fmaxf(o.s * (o.fl + sg), -q.c), q.c);
        d[i] = qv * s_n - w[i];
        const float u = 2.0f * fabsf(sg - 0.5f);
        const float u2 = u * u, u4 = u2 * u2, u8 = u4 * u4, u16 = u8 * u8;
        reg += 1.0f - u16 * u4;
    }
    reg = block_sum(reg);
    if (threadIdx.x == 0) reg_partial[blockIdx.x] = reg;
}

// Per-block sums of the squares of r.
__global__ __launch_bounds__(256) void rl_sumsq_kernel(const float* __restrict__ r, size_t n, float* __restrict__ partial)
{
    float s = 0.0f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) s += r[i] * r[i];
    s = block_sum(s);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// loss_out[0] = sum(sq partials) / count_mse, loss_out[1] = sum(reg partials) / count_reg  (double across blocks)
__global__ __launch_bounds__(256) void rl_loss_kernel(const float* __restrict__ sq, int nsq, double count_mse,
                                                      const float* __restrict__ reg, int nreg, double count_reg,
                                                      float* __restrict__ loss_out)
{
    __shared__ double acc[2][256];
    double a = 0.0, b = 0.0;
    for (int i = threadIdx.x; i < nsq; i += 256) a += (double)sq[i];
    for (int i = threadIdx.x; i < nreg; i += 256) b += (double)reg[i];
    acc[0][threadIdx.x] = a;
    acc[1][threadIdx.x] = b;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) {
            acc[0][threadIdx.x] += acc[0][threadIdx.x + off];
            acc[1][threadIdx.x] += acc[1][threadIdx.x + off];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        loss_out[0] = (float)(acc[0][0] / count_mse);
        loss_out[1] = (float)(acc[1][0] / count_reg);
    }
}

// alpha -= lr * (g * dWq/dalpha + reg_weight * dreg/dalpha); the gradient itself goes to grad_out when asked for.
__global__ __launch_bounds__(256) void rl_update_kernel(const float* __restrict__ w, const float* __restrict__ sw,
                                                        float* __restrict__ alpha, const float* __restrict__ g, int gslices,
                                                        size_t n, int K, QParams q, float lr, float reg_scale,
                                                        float* __restrict__ grad_out)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float s_n = sw[i / K];
        const OnAxis o = on_axis(w[i], __fdiv_rn(1.0f, s_n), q);
        const float a = alpha[i];
        const float sg = sigmoid_f(a);
        const float ds = sg * sigmoid_f(-a);                // sigmoid' = sigmoid(a) sigmoid(-a): 1 - sigmoid would cancel for large a
        const float pre = o.s * (o.fl + sg);
        const float dwq = (pre > -q.c && pre < q.c) ? o.s * ds * s_n : 0.0f;     // the outer clamp passes no gradient
        const float dv = sg - 0.5f;
        const float u = 2.0f * fabsf(dv);
        const float u2 = u * u, u4 = u2 * u2, u8 = u4 * u4, u16 = u8 * u8;
        const float dlam = -20.0f * (u16 * u2 * u) * 2.0f * (dv > 0.0f ? 1.0f : (dv < 0.0f ? -1.0f : 0.0f)) * ds;
        float gi = g[i];                                     // d mse / d Wq: the slices of the product, in order
        for (int z = 1; z < gslices; ++z) gi += g[(size_t)z * n + i];
        const float grad = gi * dwq + reg_scale * dlam;
        if (grad_out) grad_out[i] = grad;
        alpha[i] = a - lr * grad;
    }
}

// alpha with sigmoid(alpha) = the weight's fractional position between its grid neighbours, kept inside [eps, 1 - eps].
__global__ __launch_bounds__(256) void rl_init_kernel(const float* __restrict__ w, const float* __restrict__ sw, size_t n,
                                                      int K, QParams q, float eps, float* __restrict__ alpha)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float s_n = sw[i / K];
        const OnAxis o = on_axis(w[i], __fdiv_rn(1.0f, s_n), q);
        const float inv_s = 1.0f / o.s;                                  // exact: a power of two
        const float frac = fminf(fmaxf(o.yc * inv_s - o.fl, eps), 1.0f - eps);   // exact before the clip
        alpha[i] = logf(frac / (1.0f - frac));
    }
}

__global__ __launch_bounds__(256) void rl_mask_kernel(const float* __restrict__ alpha, size_t n, uint8_t* __restrict__ mask)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        mask[i] = alpha[i] >= 0.0f ? 1 : 0;                               // sigmoid(alpha) >= 0.5
}

// A convolution enters rounding learning as the linear layer on its patch matrix: row (b, ho, wo) of a holds the
// receptive field of that output pixel in the order of the flattened weight [Cout, (ci, kh, kw)], zeros where the
// field reaches into the padding.  Lanes run along the row (the kw taps of one (ci, kh) are neighbours in x).
__global__ __launch_bounds__(256) void rl_im2col_kernel(const float* __restrict__ x, int C, int H, int W, int kh, int kw,
                                                        int stride, int pad, int Ho, int Wo, size_t rows,
                                                        float* __restrict__ a)
{
    const int K = C * kh * kw;
    const size_t total = rows * (size_t)K;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t row = i / K;
        const int k = (int)(i - row * K);
        const int ci = k / (kh * kw), t = k - ci * (kh * kw), r = t / kw, c = t - r * kw;
        const int wo = (int)(row % Wo), ho = (int)((row / Wo) % Ho);
        const size_t b = row / ((size_t)Wo * Ho);
        const int h = ho * stride - pad + r, w = wo * stride - pad + c;
        a[i] = (h >= 0 && h < H && w >= 0 && w < W) ? x[((b * C + ci) * H + h) * (size_t)W + w] : 0.0f;
    }
}

// ---------------------------------------------------------------------------------- fp32 contraction
//
// C[i, j] = scale * sum_k P(i, k) Q(j, k), i < I, j < J, k < Kc, with P(i, k) = p[i * pi + k * pk] and the same for Q:
// KCONTIG = true:  pk = 1 (rows of P and Q run along k: C = P Q^T),
// KCONTIG = false: pi = 1 (rows of the stored matrices run along i / j: C = P'^T Q' with P' = [Kc, I], Q' = [Kc, J]).
// A workgroup of four wavefronts owns a T x T tile of C (T = 128 or 64; each wavefront a T/2 x T/2 quarter, as
// (T/64)^2 blocks of the 32x32x2 fp32 matrix instruction) and walks k in steps of 16 through two LDS buffers laid out
// [k][row], so that the lanes of an MFMA operand read consecutive words.  The global loads of step t + 1 (16 bytes
// per lane where alignment allows) are in flight while step t is computed.
template <int T, bool KCONTIG>
__global__ __launch_bounds__(256) void sgemm_kernel(const float* __restrict__ p, long pstride, const float* __restrict__ qm,
                                                    long qstride, int I, int J, int Kc, float scale,
                                                    float* __restrict__ c, long cstride, int vec, int kslice)
{
    constexpr int BK = 16;
    constexpr int LD = T + 4;
    constexpr int NB = T / 64;                     // 32-row blocks per wave and direction
    constexpr int PER4 = T * BK / 4 / 256;         // 16-byte groups of each operand tile per thread and step
    __shared__ __attribute__((aligned(16))) float ps[2][BK * LD];
    __shared__ __attribute__((aligned(16))) float qs[2][BK * LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wi = wave >> 1, wj = wave & 1;
    const int i0 = blockIdx.y * T, j0 = blockIdx.x * T;
    // slice blockIdx.z of the contraction (kslice steps of k each, a multiple of BK) writes its own copy of C
    const int kbeg = blockIdx.z * kslice;
    const int kend = kbeg + kslice < Kc ? kbeg + kslice : Kc;
    c += (size_t)blockIdx.z * (size_t)I * cstride;

    v16f acc[NB][NB];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    // A thread's share of a tile: groups of four elements that are consecutive in memory, group index
    // e * 256 + tid; KCONTIG: row = group / (BK / 4), k = 4 (group % (BK / 4)) .. + 3; otherwise
    // k = group / (T / 4), row = 4 (group % (T / 4)) .. + 3.  `vec` (host-checked: 16-byte aligned bases, strides
    // that are multiples of 4) allows one 16-byte load for a group that lies inside the matrix; anything else is
    // read element by element with zeros outside.
    float4 pr[PER4], qr[PER4];
    auto load_group = [&](const float* base, long stride, int o0, int O, int k0, int group) -> float4 {
        const int row = KCONTIG ? group / (BK / 4) : 4 * (group % (T / 4));
        const int k = KCONTIG ? 4 * (group % (BK / 4)) : group / (T / 4);
        float v[4];
        if (KCONTIG) {
            const float* src = base + (long)(o0 + row) * stride + (k0 + k);
            if (vec && o0 + row < O && k0 + k + 3 < kend) return *reinterpret_cast<const float4*>(src);
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = (o0 + row < O && k0 + k + t < kend) ? src[t] : 0.0f;
        } else {
            const float* src = base + (long)(k0 + k) * stride + (o0 + row);
            if (vec && k0 + k < kend && o0 + row + 3 < O) return *reinterpret_cast<const float4*>(src);
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = (k0 + k < kend && o0 + row + t < O) ? src[t] : 0.0f;
        }
        return make_float4(v[0], v[1], v[2], v[3]);
    };
    auto load = [&](int k0) {
#pragma unroll
        for (int e = 0; e < PER4; ++e) {
            pr[e] = load_group(p, pstride, i0, I, k0, e * 256 + tid);
            qr[e] = load_group(qm, qstride, j0, J, k0, e * 256 + tid);
        }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int e = 0; e < PER4; ++e) {
            const int group = e * 256 + tid;
            if (KCONTIG) {
                const int row = group / (BK / 4), k = 4 * (group % (BK / 4));
                ps[buf][k * LD + row] = pr[e].x; ps[buf][(k + 1) * LD + row] = pr[e].y;
                ps[buf][(k + 2) * LD + row] = pr[e].z; ps[buf][(k + 3) * LD + row] = pr[e].w;
                qs[buf][k * LD + row] = qr[e].x; qs[buf][(k + 1) * LD + row] = qr[e].y;
                qs[buf][(k + 2) * LD + row] = qr[e].z; qs[buf][(k + 3) * LD + row] = qr[e].w;
            } else {
                const int k = group / (T / 4), row = 4 * (group % (T / 4));
                *reinterpret_cast<float4*>(&ps[buf][k * LD + row]) = pr[e];
                *reinterpret_cast<float4*>(&qs[buf][k * LD + row]) = qr[e];
            }
        }
    };

    // two LDS buffers: step t is computed from one while step t + 1 is stored into the other; one barrier per step
    load(kbeg);
    store(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        const bool more = k0 + BK < kend;
        if (more) load(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float pa[NB], qb[NB];
#pragma unroll
            for (int a = 0; a < NB; ++a) pa[a] = ps[buf][(kk + g) * LD + wi * (T / 2) + 32 * a + l32];
#pragma unroll
            for (int b = 0; b < NB; ++b) qb[b] = qs[buf][(kk + g) * LD + wj * (T / 2) + 32 * b + l32];
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[a], qb[b], acc[a][b], 0, 0, 0);
        }
        if (more) store(buf ^ 1);       // nobody reads that buffer: its last readers passed the barrier of the previous step
        __syncthreads();
        buf ^= 1;
    }
    // acc[a][b][r]: row 8 (r / 4) + 4 g + r % 4 of the block (operand P), column l32 (operand Q)
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int j = j0 + wj * (T / 2) + 32 * b + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wi * (T / 2) + 32 * a + 8 * (r >> 2) + 4 * g + (r & 3);
                if (i < I && j < J) c[(long)i * cstride + j] = scale * acc[a][b][r];
            }
        }
}

// slices > 1: the contraction is cut into that many pieces, piece z writes c + z * I * cstride (the caller adds them up)
template <bool KCONTIG>
void launch_sgemm(const float* p, long pstride, const float* q, long qstride, int I, int J, int Kc, float scale, float* c,
                  long cstride, int slices, hipStream_t st)
{
    const int vec = ((reinterpret_cast<uintptr_t>(p) | reinterpret_cast<uintptr_t>(q)) & 15) == 0 && pstride % 4 == 0 &&
                    qstride % 4 == 0;
    const int kslice = ((Kc + slices - 1) / slices + 15) / 16 * 16;
    const long big = (long)((I + 127) / 128) * ((J + 127) / 128) * slices;
    if (big >= 256)
        hipLaunchKernelGGL((sgemm_kernel<128, KCONTIG>), dim3((J + 127) / 128, (I + 127) / 128, slices), dim3(256), 0, st, p,
                           pstride, q, qstride, I, J, Kc, scale, c, cstride, vec, kslice);
    else
        hipLaunchKernelGGL((sgemm_kernel<64, KCONTIG>), dim3((J + 63) / 64, (I + 63) / 64, slices), dim3(256), 0, st, p,
                           pstride, q, qstride, I, J, Kc, scale, c, cstride, vec, kslice);
}

// Slices of the gradient product (its contraction runs over the M calibration rows, its output is only [N, K]): enough
// to give the 128-row tile a few hundred workgroups, each slice at least 512 rows deep, at most 8.
int rl_slices(int64_t M, int64_t N, int64_t K)
{
    const int64_t tiles = ((N + 127) / 128) * ((K + 127) / 128);
    int64_t s = (384 + tiles - 1) / tiles;
    if (s > M / 512) s = M / 512;
    if (s > 8) s = 8;
    return s < 1 ? 1 : (int)s;
}

int blocks_for(size_t n)
{
    const size_t b = (n + 1023) / 1024;
    return b < 1 ? 1 : (b > 1024 ? 1024 : (int)b);
}

}  // namespace

size_t rl_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    // D [N, K], R [M, N], 2 x 1024 partial sums, G [slices][N, K]
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    return up((size_t)N * K * 4) + up((size_t)M * N * 4) + 2 * 4096 + up((size_t)rl_slices(M, N, K) * N * K * 4);
}

int launch_rl_im2col(const float* x, int64_t B, int64_t C, int64_t H, int64_t W, int kh, int kw, int stride, int pad,
                     float* a, hipStream_t st)
{
    const int Ho = (int)((H + 2 * pad - kh) / stride + 1), Wo = (int)((W + 2 * pad - kw) / stride + 1);
    const size_t rows = (size_t)B * Ho * Wo;
    const size_t total = rows * (size_t)(C * kh * kw);
    size_t grid = (total + 1023) / 1024;
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(rl_im2col_kernel, dim3((unsigned)grid), dim3(256), 0, st, x, (int)C, (int)H, (int)W, kh, kw, stride, pad,
                       Ho, Wo, rows, a);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

int launch_rl_init(const float* w, const float* sw, int64_t N, int64_t K, const QParams& q, float* alpha, hipStream_t st)
{
    const size_t n = (size_t)N * K;
    hipLaunchKernelGGL(rl_init_kernel, dim3(blocks_for(n)), dim3(256), 0, st, w, sw, n, (int)K, q, 1e-3f, alpha);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

int launch_rl_mask(const float* alpha, size_t n, uint8_t* mask, hipStream_t st)
{
    hipLaunchKernelGGL(rl_mask_kernel, dim3(blocks_for(n)), dim3(256), 0, st, alpha, n, mask);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

int launch_rl_step(const float* w, const float* sw, int64_t N, int64_t K, const QParams& q, float* alpha, const float* a,
                   int64_t M, float lr, float reg_weight, float* loss_out, float* grad_out, void* workspace, hipStream_t st)
{
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    float* d = reinterpret_cast<float*>(ws);
    float* r = reinterpret_cast<float*>(ws + up((size_t)N * K * 4));
    float* regp = reinterpret_cast<float*>(ws + up((size_t)N * K * 4) + up((size_t)M * N * 4));
    float* sqp = regp + 1024;
    float* g = sqp + 1024;
    const int slices = rl_slices(M, N, K);
    const size_t nw = (size_t)N * K, nr = (size_t)M * N;
    const int bw = blocks_for(nw), br = blocks_for(nr);
    hipLaunchKernelGGL(rl_soft_kernel, dim3(bw), dim3(256), 0, st, w, sw, alpha, nw, (int)K, q, d, regp);
    // R[m, n] = sum_k A[m, k] D[n, k]
    launch_sgemm<true>(a, K, d, K, (int)M, (int)N, (int)K, 1.0f, r, N, 1, st);
    hipLaunchKernelGGL(rl_sumsq_kernel, dim3(br), dim3(256), 0, st, r, nr, sqp);
    hipLaunchKernelGGL(rl_loss_kernel, dim3(1), dim3(256), 0, st, sqp, br, (double)nr, regp, bw, (double)nw, loss_out);
    // G[n, k] = (2 / (M N)) sum_m R[m, n] A[m, k]
    launch_sgemm<false>(r, N, a, K, (int)N, (int)K, (int)M, (float)(2.0 / (double)nr), g, K, slices, st);
    hipLaunchKernelGGL(rl_update_kernel, dim3(bw), dim3(256), 0, st, w, sw, alpha, g, slices, nw, (int)K, q, lr,
                       (float)((double)reg_weight / (double)nw), grad_out);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

}  // namespace fpq
