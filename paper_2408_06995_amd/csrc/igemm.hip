// The same-bitwidth integer baseline the paper compares against (Section IV-A, Eq. (4)): uniform quantizer with scale
// s = (max - min) / (2^b - 1) and zero point z = -round(min / s), and a linear layer on its codes with the 8-bit integer
// matrix instruction of gfx950 (v_mfma_i32_32x32x32_i8, exact 32-bit sums).
//
// The matrix instruction multiplies signed bytes, the codes are unsigned (0 .. 2^b - 1) with a zero point, so the
// operands are offset: activations enter as a' = q - 128, 8-bit weights as b' = q - 128 (stored that way when packed),
// 4-bit weights as b' = q (0 .. 15 fits a signed byte).  With za = zx - 128 and zb = zw - 128 (or zw):
//   sum_k (qx - zx)(qw - zw) = sum_k a' b'  -  zb * sum_k a'  -  za * sum_k b'  +  K * za * zb,
// all in 32-bit integers (K <= 32768 keeps the result below 2^31; intermediate wrap-around cancels).  The row sums of b'
// are computed when the weights are packed, those of a' by a small kernel before the layer.
#include "fpq_dev.h"
#include "fpq_host.h"
#include "gemm_common.h"

namespace fpq {

typedef int v4i32 __attribute__((ext_vector_type(4)));
typedef int v16i32 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------- min / max -> (s, z)

__device__ __forceinline__ void block_minmax(float& lo, float& hi)
{
    __shared__ float plo[4], phi[4];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, 64));
        hi = fmaxf(hi, __shfl_xor(hi, off, 64));
    }
    if ((threadIdx.x & 63) == 0) { plo[threadIdx.x >> 6] = lo; phi[threadIdx.x >> 6] = hi; }
    __syncthreads();
    lo = fminf(fminf(plo[0], plo[1]), fminf(plo[2], plo[3]));
    hi = fmaxf(fmaxf(phi[0], phi[1]), fmaxf(phi[2], phi[3]));
    __syncthreads();
}

// Eq. (4): s = fl32(fl32(max - min) / (2^b - 1)) (1 for a constant tensor), z = -round(fl32(min * fl32(1 / s))).
__device__ __forceinline__ void int_params_of(float lo, float hi, int levels, float& s, int& z)
{
    const float rng = __fsub_rn(hi, lo);
    s = (rng == 0.0f) ? 1.0f : __fdiv_rn(rng, (float)levels);
    const float r = __fdiv_rn(1.0f, s);
    z = -(int)rintf(__fmul_rn(lo, r));
}

__global__ __launch_bounds__(256) void int_minmax_partial_kernel(const float* __restrict__ x, size_t n, float* __restrict__ partial)
{
    float lo = INFINITY, hi = -INFINITY;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float v = x[i];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    block_minmax(lo, hi);
    if (threadIdx.x == 0) { partial[2 * blockIdx.x] = lo; partial[2 * blockIdx.x + 1] = hi; }
}

__global__ __launch_bounds__(256) void int_minmax_final_kernel(const float* __restrict__ partial, int nparts, int levels, int empty,
                                                               fpq_int_params* __restrict__ out)
{
    float lo = INFINITY, hi = -INFINITY;
    for (int i = threadIdx.x; i < nparts; i += 256) { lo = fminf(lo, partial[2 * i]); hi = fmaxf(hi, partial[2 * i + 1]); }
    block_minmax(lo, hi);
    if (threadIdx.x == 0) {
        if (empty) lo = hi = 0.0f;
        float s; int z;
        int_params_of(lo, hi, levels, s, z);
        out->scale = s;
        out->zero_point = z;
        out->min = lo;
        out->max = hi;
    }
}

static int int_minmax_parts(size_t n)
{
    size_t g = (n + 4095) / 4096;
    return (int)(g < 1 ? 1 : (g > 1024 ? 1024 : g));
}

int launch_int_params(const float* x, size_t n, int bits, fpq_int_params* out, float* partial, hipStream_t st)
{
    const int parts = int_minmax_parts(n);
    hipLaunchKernelGGL(int_minmax_partial_kernel, dim3(parts), dim3(256), 0, st, x, n, partial);
    hipLaunchKernelGGL(int_minmax_final_kernel, dim3(1), dim3(256), 0, st, partial, parts, (1 << bits) - 1, n == 0 ? 1 : 0, out);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------- quantize

// q = clamp(round(fl32(x * r)) + z; 0, 2^b - 1), ties to even; NaN gives code 0.
__device__ __forceinline__ uint32_t int_code(float x, float r, int z, int qmax)
{
    const float y = rintf(__fmul_rn(x, r));
    // |y| can exceed the int range: clamp in float first (z is small against 2^30)
    const float yc = fminf(fmaxf(y, -1073741824.0f), 1073741824.0f);
    const long long q = (long long)(int)yc + (long long)z;
    return (uint32_t)(q < 0 ? 0 : (q > qmax ? qmax : q));
}

__global__ __launch_bounds__(256) void int_quantize_kernel(const float* __restrict__ x, size_t n, int qmax, float scale, int zp,
                                                           const fpq_int_params* __restrict__ params_dev,
                                                           uint8_t* __restrict__ codes)
{
    const float s = params_dev ? params_dev->scale : scale;
    const int z = params_dev ? params_dev->zero_point : zp;
    const float r = __fdiv_rn(1.0f, s);
    const size_t nthreads = (size_t)gridDim.x * 256;
    const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (((reinterpret_cast<uintptr_t>(x) & 15) | (reinterpret_cast<uintptr_t>(codes) & 3)) == 0) {
        const size_t n4 = n >> 2;
        for (size_t i = tid; i < n4; i += nthreads) {
            const float4 v = reinterpret_cast<const float4*>(x)[i];
            reinterpret_cast<uint32_t*>(codes)[i] = int_code(v.x, r, z, qmax) | (int_code(v.y, r, z, qmax) << 8) |
                                                   (int_code(v.z, r, z, qmax) << 16) | (int_code(v.w, r, z, qmax) << 24);
        }
        for (size_t j = (n4 << 2) + tid; j < n; j += nthreads) codes[j] = (uint8_t)int_code(x[j], r, z, qmax);
    } else {
        for (size_t j = tid; j < n; j += nthreads) codes[j] = (uint8_t)int_code(x[j], r, z, qmax);
    }
}

int launch_int_quantize(const float* x, size_t n, int bits, float scale, int zp, const fpq_int_params* params_dev, uint8_t* codes,
                        hipStream_t st)
{
    if (n == 0) return FPQ_OK;
    size_t g = (n / 4 + 1023) / 1024;
    g = g < 1 ? 1 : (g > 2048 ? 2048 : g);
    hipLaunchKernelGGL(int_quantize_kernel, dim3((unsigned)g), dim3(256), 0, st, x, n, (1 << bits) - 1, scale, zp, params_dev, codes);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------- weights: per-channel (s, z), codes, row sums

// One block per output channel.  Packed row: Kpad bytes of b' = q - 128 (8-bit), or Kpad / 2 bytes holding b' = q as
// nibbles (4-bit), where byte j of every 4-byte word carries k = 8 w + j in its low and k = 8 w + 4 + j in its high nibble
// (w = the word's index), so that masking the low and the high nibbles of a word yields two words of four consecutive k.
// Padding (k >= K) is b' = 0: it adds nothing to the products nor to the row sum.
template <bool FOUR_BIT>
__global__ __launch_bounds__(256) void int_pack_weights_kernel(const float* __restrict__ w, int K, int Kpad, int bits,
                                                               uint8_t* __restrict__ rows, float* __restrict__ scale_out,
                                                               int32_t* __restrict__ zp_out, int32_t* __restrict__ rowsum_out,
                                                               uint8_t* __restrict__ codes_out)
{
    const int n = blockIdx.x;
    const float* row = w + (size_t)n * K;
    float lo = INFINITY, hi = -INFINITY;
    for (int i = threadIdx.x; i < K; i += 256) { lo = fminf(lo, row[i]); hi = fmaxf(hi, row[i]); }
    block_minmax(lo, hi);
    float s; int z;
    const int qmax = (1 << bits) - 1;
    int_params_of(lo, hi, qmax, s, z);
    if (threadIdx.x == 0) { scale_out[n] = s; zp_out[n] = z; }
    const float r = __fdiv_rn(1.0f, s);
    int sum = 0;
    if (FOUR_BIT) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(rows + (size_t)n * (Kpad / 2));
        for (int wd = threadIdx.x; wd < Kpad / 8; wd += 256) {
            uint32_t word = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int k = 8 * wd + j;
                uint32_t q = 0;
                if (k < K) {
                    q = int_code(row[k], r, z, qmax);
                    if (codes_out) codes_out[(size_t)n * K + k] = (uint8_t)q;
                    sum += (int)q;
                }
                word |= q << (j < 4 ? 8 * j : 8 * (j - 4) + 4);
            }
            dst[wd] = word;
        }
    } else {
        uint32_t* dst = reinterpret_cast<uint32_t*>(rows + (size_t)n * Kpad);
        for (int wd = threadIdx.x; wd < Kpad / 4; wd += 256) {
            uint32_t word = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = 4 * wd + j;
                if (k < K) {
                    const uint32_t q = int_code(row[k], r, z, qmax);
                    if (codes_out) codes_out[(size_t)n * K + k] = (uint8_t)q;
                    sum += (int)q - 128;
                    word |= (q ^ 0x80u) << (8 * j);
                }
            }
            dst[wd] = word;
        }
    }
    __shared__ int part[4];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) rowsum_out[n] = part[0] + part[1] + part[2] + part[3];
}

int launch_int_pack_weights(const float* w, int64_t N, int64_t K, int bits, uint8_t* rows, float* scale_out, int32_t* zp_out,
                            int32_t* rowsum_out, uint8_t* codes_out, hipStream_t st)
{
    const int Kpad = (int)padded_k(K, 1);
    if (bits == 4)
        hipLaunchKernelGGL(int_pack_weights_kernel<true>, dim3((unsigned)N), dim3(256), 0, st, w, (int)K, Kpad, bits, rows, scale_out,
                           zp_out, rowsum_out, codes_out);
    else
        hipLaunchKernelGGL(int_pack_weights_kernel<false>, dim3((unsigned)N), dim3(256), 0, st, w, (int)K, Kpad, bits, rows, scale_out,
                           zp_out, rowsum_out, codes_out);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------- row sums of the activation codes

// rowsum[m] = sum_k (q[m, k] - 128): one wavefront per row, 16 bytes per lane and step.
__global__ __launch_bounds__(256) void int_rowsum_kernel(const uint8_t* __restrict__ codes, int M, int K, int32_t* __restrict__ rowsum)
{
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const uint8_t* row = codes + (size_t)m * K;
    int sum = 0;
    for (int k = lane * 16; k < K; k += 64 * 16) {            // K % 16 == 0
        const uint4 v = *reinterpret_cast<const uint4*>(row + k);
        const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            sum += (int)(wds[i] & 0xff) + (int)((wds[i] >> 8) & 0xff) + (int)((wds[i] >> 16) & 0xff) + (int)(wds[i] >> 24) - 512;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) rowsum[m] = sum;
}

// ---------------------------------------------------------------------------------- the layer

struct IGemmArgs {
    const uint8_t* x;        // activation codes [M, K], K % 16 == 0
    const uint8_t* wrows;    // packed weight rows
    const int32_t* wsum;     // [N] row sums of b'
    const float* sw;         // [N]
    const int32_t* zw;       // [N]
    const float* bias;       // [N] or null
    const int32_t* xsum;     // [M] row sums of a'
    const fpq_int_params* px_dev;   // activation scale / zero point on the device, or null
    float sx;
    int zx;
    float* y;
    int M, N, K, Kpad;
};

// A workgroup of four wavefronts (2 x 2) owns a BX x BW tile; K in steps of 128 codes through two LDS stages,
// register-staged loads, four 32-code integer MFMA steps per K step.  Activations are the row operand (accumulator
// registers run along m), weights the lane operand, so a half-wave stores 128 consecutive bytes of an output row.
template <int BX, int BW, bool W4>
__global__ __launch_bounds__(256) void igemm_kernel(const IGemmArgs a)
{
    constexpr int XROWB = 128, WROWB = W4 ? 64 : 128;
    constexpr int XTILE = BX * XROWB, WTILE = BW * WROWB, STAGE = XTILE + WTILE;
    constexpr int XLD = BX / 32;
    constexpr int WCPR = WROWB / 16, WROWS_PER_PASS = 256 / WCPR, WLD = (BW + WROWS_PER_PASS - 1) / WROWS_PER_PASS;
    constexpr int TP = BX / 2, TQ = BW / 2, MI = TP / 32, NI = TQ / 32;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int tiles_w = (a.N + BW - 1) / BW;
    const int tx = blockIdx.x / tiles_w, tw = blockIdx.x - tx * tiles_w;
    const int m0 = tx * BX, n0 = tw * BW;
    const int xc = tid & 7, xr0 = tid >> 3;
    const int wc = tid % WCPR, wr0 = tid / WCPR;
    const size_t wrow_bytes = W4 ? (size_t)a.Kpad / 2 : (size_t)a.Kpad;
    uint4 xreg[XLD], wreg[WLD];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < XLD; ++i) {
            const int m = m0 + xr0 + 32 * i;
            const int k = kt * 128 + xc * 16;
            // rows and k beyond the tensor read as a' = 0, i.e. the byte 0x80 before the sign flip below
            xreg[i] = (m < a.M && k < a.K) ? *reinterpret_cast<const uint4*>(a.x + (size_t)m * a.K + k)
                                           : make_uint4(0x80808080u, 0x80808080u, 0x80808080u, 0x80808080u);
        }
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const int row = wr0 + WROWS_PER_PASS * i;
            wreg[i] = (row < BW && n0 + row < a.N)
                          ? *reinterpret_cast<const uint4*>(a.wrows + (size_t)(n0 + row) * wrow_bytes + (size_t)kt * WROWB + wc * 16)
                          : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int stage) {
        uint8_t* xs = smem + stage * STAGE;
        uint8_t* ws = xs + XTILE;
#pragma unroll
        for (int i = 0; i < XLD; ++i) {
            uint4 v = xreg[i];                     // unsigned code -> signed a' = q - 128: flip the top bit of every byte
            v.x ^= 0x80808080u; v.y ^= 0x80808080u; v.z ^= 0x80808080u; v.w ^= 0x80808080u;
            *reinterpret_cast<uint4*>(xs + lds_off<XROWB>(xr0 + 32 * i, xc)) = v;
        }
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const int row = wr0 + WROWS_PER_PASS * i;
            if (row < BW) *reinterpret_cast<uint4*>(ws + lds_off<WROWB>(row, wc)) = wreg[i];
        }
    };
    v16i32 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    const int wp = wave >> 1, wq = wave & 1;
    const int prow0 = wp * TP + l32, qrow0 = wq * TQ + l32;
    auto compute = [&](int stage) {
        const uint8_t* xs = smem + stage * STAGE;
        const uint8_t* ws = xs + XTILE;
#pragma unroll
        for (int c = 0; c < 4; ++c) {               // four chunks of 32 codes; lane half g takes codes 16 g .. 16 g + 15 of a chunk
            v4i32 af[MI], bf_[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const uint4 v = *reinterpret_cast<const uint4*>(xs + lds_off<XROWB>(prow0 + 32 * i, 2 * c + g));
                af[i] = v4i32{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int row = qrow0 + 32 * j;
                if (W4) {
                    // 16 codes = 8 bytes = words 2 h, 2 h + 1 of the row's step (h = 2 c + g): low nibbles, then high nibbles
                    const uint2 v = *reinterpret_cast<const uint2*>(ws + lds_off<WROWB>(row, c) + g * 8);
                    bf_[j] = v4i32{(int)(v.x & 0x0f0f0f0fu), (int)((v.x >> 4) & 0x0f0f0f0fu), (int)(v.y & 0x0f0f0f0fu),
                                   (int)((v.y >> 4) & 0x0f0f0f0fu)};
                } else {
                    const uint4 v = *reinterpret_cast<const uint4*>(ws + lds_off<WROWB>(row, 2 * c + g));
                    bf_[j] = v4i32{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
                }
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf_[j], acc[i][j], 0, 0, 0);
        }
    };
    const int nk = a.Kpad / 128;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_global(kt + 1);
        compute(cur);
        if (kt + 1 < nk) store_lds(cur ^ 1);
        __syncthreads();
    }
    // ---- epilogue: fold the zero points out with the row sums, scale, store
    const float sx = a.px_dev ? a.px_dev->scale : a.sx;
    const int za = (a.px_dev ? a.px_dev->zero_point : a.zx) - 128;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int n = n0 + wq * TQ + 32 * j + l32;
        if (n >= a.N) continue;
        const int zb = a.zw[n] - (W4 ? 0 : 128);
        const int colterm = (int)((uint32_t)a.K * (uint32_t)za * (uint32_t)zb - (uint32_t)za * (uint32_t)a.wsum[n]);
        const float sc = sx * a.sw[n];
        const float bv = a.bias ? a.bias[n] : 0.0f;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wp * TP + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                if (m < a.M) {
                    // unsigned arithmetic: intermediate values may wrap, the result fits (K <= 32768)
                    const int total = (int)((uint32_t)acc[i][j][r] - (uint32_t)zb * (uint32_t)a.xsum[m] + (uint32_t)colterm);
                    a.y[(size_t)m * a.N + n] = (float)total * sc + bv;
                }
            }
    }
}

template <int BX, int BW, bool W4>
static int launch_igemm_one(const IGemmArgs& a, hipStream_t st)
{
    constexpr int smem = 2 * (BX * 128 + BW * (W4 ? 64 : 128));
    const int tiles = ((a.M + BX - 1) / BX) * ((a.N + BW - 1) / BW);
    auto kern = igemm_kernel<BX, BW, W4>;
    if (smem > 64 * 1024) {
        static std::atomic<uint64_t> allowed{0};
        if (!allow_dynamic_lds(reinterpret_cast<const void*>(kern), smem, allowed)) return FPQ_ERR_LAUNCH;
    }
    hipLaunchKernelGGL(kern, dim3(tiles), dim3(256), smem, st, a);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

int launch_int_gemm(const uint8_t* x, float sx, int zx, const fpq_int_params* px_dev, const uint8_t* wrows, const int32_t* wsum,
                    int wbits, const float* sw, const int32_t* zw, const float* bias, float* y, int64_t M, int64_t N, int64_t K,
                    int32_t* xsum, hipStream_t st)
{
    if (M <= 0 || N <= 0) return FPQ_OK;
    hipLaunchKernelGGL(int_rowsum_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, x, (int)M, (int)K, xsum);
    IGemmArgs a{x, wrows, wsum, sw, zw, bias, xsum, px_dev, sx, zx, y, (int)M, (int)N, (int)K, (int)padded_k(K, 1)};
    const long big = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (wbits == 4) return big >= 256 ? launch_igemm_one<128, 128, true>(a, st) : launch_igemm_one<64, 64, true>(a, st);
    return big >= 256 ? launch_igemm_one<128, 128, false>(a, st) : launch_igemm_one<64, 64, false>(a, st);
}

}  // namespace fpq
