// Encoding and bias search of Section V-A (Algorithm 1) as one pass over the tensor.
//
// A candidate is an encoding (e, m) with the max value c_j = absmax * (j + 1) / J; its real-valued
// bias (Eq. (7) solved for b) is carried as the integer bias b0 = 2^(e-1) plus the scale
// c_j / c0, c0 = Eq. (7) at b0, so a candidate is exactly what fpq_quantize computes for the format
// (e, m, b0) and that scale.  Every lane holds eight elements in registers and walks all
// n_enc x J candidates over them: quantize (the same magic-add rounding as the encoder, kept as a
// value instead of a code), dequantize, squared error.  The kernel is bound by vector ALU work
// (about 11 instructions per element and candidate), the tensor is read once.
#include "fpq_dev.h"
#include "fpq_host.h"

namespace fpq {

constexpr int kSearchElems = 8;   // elements per lane and round

// Per-block partial sums of squared errors: partial[block][candidate].
__global__ __launch_bounds__(256) void search_partial_kernel(const float* __restrict__ x, size_t n,
                                                             const float* __restrict__ absmax_dev, SearchArgs a,
                                                             float* __restrict__ partial)
{
    __shared__ float tab_r[kSearchMaxCandidates], tab_s[kSearchMaxCandidates];
    __shared__ float wacc[4][kSearchMaxCandidates];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int NC = a.n_enc * a.J;
    float am = absmax_dev[0];
    if (!(am > 0.0f)) am = 1.0f;
    for (int c = tid; c < NC; c += 256) {
        const int i = c / a.J, j = c - i * a.J;
        const float cj = (float)((double)am * (double)(j + 1) / (double)a.J);
        const float sc = (float)((double)cj / (double)a.enc[i].c0);
        tab_s[c] = sc;
        tab_r[c] = __fdiv_rn(1.0f, sc);
        wacc[0][c] = wacc[1][c] = wacc[2][c] = wacc[3][c] = 0.0f;
    }
    __syncthreads();
    const size_t chunk = (size_t)256 * kSearchElems;
    const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15) == 0;
    for (size_t base = (size_t)blockIdx.x * chunk; base < n; base += (size_t)gridDim.x * chunk) {
        const size_t i0 = base + (size_t)tid * kSearchElems;
        float ax[kSearchElems];
        if (aligned && i0 + kSearchElems <= n) {
            const float4 v0 = *reinterpret_cast<const float4*>(x + i0);
            const float4 v1 = *reinterpret_cast<const float4*>(x + i0 + 4);
            ax[0] = fabsf(v0.x); ax[1] = fabsf(v0.y); ax[2] = fabsf(v0.z); ax[3] = fabsf(v0.w);
            ax[4] = fabsf(v1.x); ax[5] = fabsf(v1.y); ax[6] = fabsf(v1.z); ax[7] = fabsf(v1.w);
        } else {
#pragma unroll
            for (int k = 0; k < kSearchElems; ++k) ax[k] = (i0 + k < n) ? fabsf(x[i0 + k]) : 0.0f;   // 0 adds no error
        }
        for (int i = 0; i < a.n_enc; ++i) {
            const int m = a.enc[i].m, b0 = a.enc[i].b0;
            const float c0 = a.enc[i].c0;
            const int cbase = i * a.J;
            for (int j = 0; j < a.J; ++j) {
                const float r = tab_r[cbase + j], sc = tab_s[cbase + j];
                float sum = 0.0f;
#pragma unroll
                for (int k = 0; k < kSearchElems; ++k) {
                    const float aa = fminf(__fmul_rn(ax[k], r), c0);                        // Eq. (6)
                    const int P = max((int)(__float_as_uint(aa) >> 23) - 127 + b0, 1);    // Eq. (9): s = 2^(P-b-m)
                    const float C = __uint_as_float((uint32_t)(P - b0 - m + 150) << 23);  // 2^23 s
                    const float q = __fsub_rn(__fadd_rn(aa, C), C);                       // Eq. (8): rne(aa / s) s
                    const float d = __fmaf_rn(-q, sc, ax[k]);
                    sum = __fmaf_rn(d, d, sum);
                }
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
                if (lane == 0) wacc[wave][cbase + j] += sum;
            }
        }
    }
    __syncthreads();
    for (int c = tid; c < NC; c += 256)
        partial[(size_t)blockIdx.x * NC + c] = (wacc[0][c] + wacc[1][c]) + (wacc[2][c] + wacc[3][c]);
}

// Sums the partials in double, writes every candidate's mean squared error and scans them in the
// order of Algorithm 1 (encodings outer, biases inner, strict comparison: the first minimum wins).
__global__ __launch_bounds__(256) void search_final_kernel(const float* __restrict__ partial, int nblocks, size_t n,
                                                           const float* __restrict__ absmax_dev, SearchArgs a,
                                                           float* __restrict__ mse_out,
                                                           fpq_search_result* __restrict__ result)
{
    __shared__ double mse[kSearchMaxCandidates];
    const int NC = a.n_enc * a.J;
    for (int c = threadIdx.x; c < NC; c += 256) {
        double s = 0.0;
        for (int b = 0; b < nblocks; ++b) s += (double)partial[(size_t)b * NC + c];
        s = n ? s / (double)n : 0.0;
        mse[c] = s;
        if (mse_out) mse_out[c] = (float)s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int best = 0;
        double prev = mse[0];
        for (int c = 1; c < NC; ++c)
            if (prev > mse[c]) {
                prev = mse[c];
                best = c;
            }
        float am = absmax_dev[0];
        if (!(am > 0.0f)) am = 1.0f;
        const int i = best / a.J, j = best - i * a.J;
        const float cj = (float)((double)am * (double)(j + 1) / (double)a.J);
        const int e = a.enc[i].e, m = a.enc[i].m;
        result->encoding = i;
        result->bias_index = j;
        result->ebits = e;
        result->mbits = m;
        result->int_bias = a.enc[i].b0;
        result->maxval = cj;
        result->scale = (float)((double)cj / (double)a.enc[i].c0);
        result->mse = (float)prev;
        // Eq. (7) solved for the bias: c = (2 - 2^-m) 2^(2^e - b - 1)
        result->real_bias = (float)((double)((1 << e) - 1) - log2((double)cj / (2.0 - exp2((double)-m))));
    }
}

int launch_search(const float* x, size_t n, const SearchArgs& a, const float* absmax_dev, float* partial,
                  float* mse_out, fpq_search_result* result, hipStream_t st)
{
    const int nblocks = search_blocks(n);
    if (nblocks > 0)
        hipLaunchKernelGGL(search_partial_kernel, dim3(nblocks), dim3(256), 0, st, x, n, absmax_dev, a, partial);
    hipLaunchKernelGGL(search_final_kernel, dim3(1), dim3(256), 0, st, partial, nblocks, n, absmax_dev, a, mse_out,
                       result);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

}  // namespace fpq
