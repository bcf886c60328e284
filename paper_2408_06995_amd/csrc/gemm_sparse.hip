// Structured-sparse weight operand (Section VI, "Sparsity"; the paper's future work: use the zeros that quantization
// produces).  Two parts:
//   pack_weights_sparse_kernel  quantizes a weight tensor as fpq_pack_weights does, then keeps in every group of four
//                               consecutive input channels (per output channel and kernel tap) the two codes of largest
//                               magnitude (equal magnitudes: the lower channel) and stores only those, with a 2-bit position
//                               each: half the weight bytes.  A group with at most two non-zero codes loses nothing.
//   gemm_sparse_kernel          the layer on that operand with the sparse matrix instruction of gfx950
//                               (v_smfmac_f32_32x32x32_bf16): codes are expanded to bf16 in registers as in the dense
//                               fp32-accumulate path, every kept product is exact and summed in fp32.
//
// What the instruction pairs with what (measured with one-hot operands): the dense operand's lane (column j, half h)
// holds 16 consecutive k, k = 16 h + t; the sparse operand's lane (row i, half g) holds eight kept values, value v
// belonging to the group of four k that starts at 16 (v / 4) + 8 g + 4 ((v % 4) / 2), at the position given by bits
// 2v + 1 : 2v of the lane's index word; positions are free (any two of the four, in any order).  The result has the
// layout of the dense 32 x 32 instructions: register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32.
//
// Packed layout (after the 256-byte header): N rows of kept codes (Kpad / 2 bytes; Kpad / 4 for formats of at most 4
// bits), then, 256-byte aligned, N rows of position words (Kpad / 8 bytes).  K runs in (kh, kw, ci) order with ci
// padded to 16 and K to 128 as in the dense layout.  Each chunk of 32 k has 16 kept codes, stored in the order in
// which the lanes take them (the eight of lane half 0, then the eight of lane half 1), and one 32-bit position word
// in the same order.
#include <type_traits>

#include "gemm_common.h"

namespace fpq {

typedef __bf16 v16bf __attribute__((ext_vector_type(16)));

// Position of group G (0..7) of a 32-k chunk in the stored order: lane half and pair index within the half.
__host__ __device__ __forceinline__ int sparse_slot_of_group(int G)
{
    const int g = (G >> 1) & 1;
    const int pair = (G & 1) | ((G >> 2) << 1);
    return 8 * g + 2 * pair;          // index of the group's first kept code among the chunk's 16
}

// ---------------------------------------------------------------------------------- prune + pack

__device__ __forceinline__ float block_max4(float v)
{
    __shared__ float part[4];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    v = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    __syncthreads();
    return v;
}

// One block per output channel; a thread builds whole 32-k chunks (16 kept codes + one position word).
template <bool FOUR_BIT>
__global__ __launch_bounds__(256) void pack_weights_sparse_kernel(const float* __restrict__ w, int Cin, int taps, int Cp, int Kpad,
                                                                  QParams q, const float* __restrict__ scale_in,
                                                                  const uint8_t* __restrict__ mask,
                                                                  uint8_t* __restrict__ code_rows, uint32_t* __restrict__ pos_rows,
                                                                  float* __restrict__ scale_out, uint8_t* __restrict__ codes_out,
                                                                  unsigned long long* __restrict__ altered)
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
        v = block_max4(v);
        s = (v == 0.0f) ? 1.0f : __fdiv_rn(v, q.c);
    }
    if (threadIdx.x == 0) scale_out[n] = s;
    const float r = __fdiv_rn(1.0f, s);
    const uint32_t magmask = (1u << q.em) - 1u;
    const size_t code_row_bytes = FOUR_BIT ? (size_t)Kpad / 4 : (size_t)Kpad / 2;
    uint8_t* crow = code_rows + (size_t)n * code_row_bytes;
    uint32_t* prow = pos_rows + (size_t)n * (Kpad / 32);
    unsigned lost = 0;
    for (int ch = threadIdx.x; ch < Kpad / 32; ch += 256) {
        uint32_t kept[16];
        uint32_t pos = 0;
#pragma unroll
        for (int G = 0; G < 8; ++G) {
            const int kp0 = ch * 32 + G * 4;          // packed k of the group's first element; Cp % 4 == 0: one tap
            const int tap = kp0 / Cp;
            const int ci0 = kp0 - tap * Cp;
            uint32_t code[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ci = ci0 + e;
                code[e] = 0;
                if (tap < taps && ci < Cin) {
                    const size_t src = (size_t)ci * taps + tap;
                    code[e] = mrow ? quantize_mask(row[src], r, mrow[src], q) : quantize_nearest(row[src], r, q);
                }
            }
            // the two largest magnitudes (a code without its sign bit grows with its magnitude); equal: lower index
            int i0 = 0;
#pragma unroll
            for (int e = 1; e < 4; ++e)
                if ((code[e] & magmask) > (code[i0] & magmask)) i0 = e;
            int i1 = i0 == 0 ? 1 : 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e != i0 && e != i1 && (code[e] & magmask) > (code[i1] & magmask)) i1 = e;
            // ties between i1 and a lower index that is not i0: the scan above keeps the lower index, as the strict
            // comparison only moves to a later element when it is larger
            const int lo = i0 < i1 ? i0 : i1, hi = i0 < i1 ? i1 : i0;
            bool dropped_nonzero = false;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (e != lo && e != hi) {
                    dropped_nonzero = dropped_nonzero || (code[e] & magmask) != 0;
                    code[e] = 0;
                }
            }
            lost += dropped_nonzero ? 1u : 0u;
            const int u = sparse_slot_of_group(G);
            kept[u] = code[lo];
            kept[u + 1] = code[hi];
            pos |= (uint32_t)lo << (2 * u);
            pos |= (uint32_t)hi << (2 * u + 2);
            if (codes_out) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ci = ci0 + e;
                    if (tap < taps && ci < Cin) codes_out[(size_t)n * K + (size_t)ci * taps + tap] = (uint8_t)code[e];
                }
            }
        }
        if (FOUR_BIT) {
            uint32_t w0 = 0, w1 = 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                w0 |= kept[u] << (4 * u);
                w1 |= kept[8 + u] << (4 * u);
            }
            reinterpret_cast<uint32_t*>(crow)[2 * ch] = w0;
            reinterpret_cast<uint32_t*>(crow)[2 * ch + 1] = w1;
        } else {
            uint32_t wd[4] = {0, 0, 0, 0};
#pragma unroll
            for (int u = 0; u < 16; ++u) wd[u >> 2] |= kept[u] << (8 * (u & 3));
            reinterpret_cast<uint4*>(crow)[ch] = make_uint4(wd[0], wd[1], wd[2], wd[3]);
        }
        prow[ch] = pos;
    }
    if (lost) atomicAdd(altered, (unsigned long long)lost);
}

__global__ void zero_u64_kernel(unsigned long long* p) { *p = 0ull; }

int launch_pack_weights_sparse(const float* w, int64_t N, int64_t Cin, int taps, const QParams& q, bool four_bit,
                               const float* scale_in, const uint8_t* mask, uint8_t* code_rows, uint32_t* pos_rows,
                               float* scale_out, uint8_t* codes_out, unsigned long long* altered, hipStream_t st)
{
    const int Cp = (int)padded_channels(Cin);
    const int Kpad = (int)padded_k(Cin, taps);
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, st, altered);
    if (four_bit)
        hipLaunchKernelGGL(pack_weights_sparse_kernel<true>, dim3((unsigned)N), dim3(256), 0, st, w, (int)Cin, taps, Cp, Kpad, q,
                           scale_in, mask, code_rows, pos_rows, scale_out, codes_out, altered);
    else
        hipLaunchKernelGGL(pack_weights_sparse_kernel<false>, dim3((unsigned)N), dim3(256), 0, st, w, (int)Cin, taps, Cp, Kpad, q,
                           scale_in, mask, code_rows, pos_rows, scale_out, codes_out, altered);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------- the layer

// A workgroup of four wavefronts (2 x 2) owns BW weight rows x BX activation rows and walks K in steps of 128 k:
// global --16-byte loads--> registers --> LDS (two stages) --> fragments --> 4 sparse MFMA steps of 32 k.
// The weights are the sparse (row) operand, so the lanes of the result run along the activation rows / output pixels:
// NCHW results are written along the pixel index (coalesced), row-major results 16 bytes per lane.
// Activations: hardware E4M3 codes; weights: hardware E4M3 or E2M1 codes (WKIND).
template <int BX, int BW, int WKIND, bool CONV>
__global__ __launch_bounds__(256) void gemm_sparse_kernel(const GemmArgs a, const uint32_t* __restrict__ pos_rows)
{
    constexpr bool W4 = kind_is_4bit(WKIND);
    constexpr int XROWB = 128;
    constexpr int WROWB = W4 ? 32 : 64;        // kept codes of one weight row per K step
    constexpr int PROWB = 20;                  // four position words per row and K step, rows 20 bytes apart (bank spread)
    constexpr int XTILE = BX * XROWB, WTILE = BW * WROWB, PTILE = BW * PROWB;
    constexpr int STAGE = XTILE + WTILE + ((PTILE + 15) / 16 * 16);
    constexpr int XLD = BX / 32;
    constexpr int WCPR = WROWB / 16;
    constexpr int WROWS_PER_PASS = 256 / WCPR;
    constexpr int WLD = (BW + WROWS_PER_PASS - 1) / WROWS_PER_PASS;
    constexpr int TP = BW / 2, TQ = BX / 2;    // per-wave tile: weight rows x activation rows
    constexpr int MI = TP / 32, NI = TQ / 32;
    static_assert(TP % 32 == 0 && TQ % 32 == 0 && BW <= 256, "tile shape");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;

    const int tiles_w = (a.N + BW - 1) / BW;
    const int tiles_x = (a.M + BX - 1) / BX;
    const int tx = blockIdx.x / tiles_w, tw = blockIdx.x - tx * tiles_w;
    if (tx >= tiles_x) return;
    const int m0 = tx * BX, n0 = tw * BW;

    // ---- activation loads (as in the dense register-staged kernel)
    const int xc = tid & 7, xr0 = tid >> 3;
    int xbase[XLD], xhw[XLD];
#pragma unroll
    for (int i = 0; i < XLD; ++i) {
        const int m = m0 + xr0 + 32 * i;
        if (m < a.M) {
            if (CONV) {
                const int hw = a.Ho * a.Wo;
                const int bi = m / hw;
                const int rem = m - bi * hw;
                const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
                const int hi0 = ho * a.stride - a.pad, wi0 = wo * a.stride - a.pad;
                xbase[i] = ((bi * a.H + hi0) * a.W + wi0) * a.Cp;
                xhw[i] = ((hi0 + 0x4000) << 16) | (wi0 + 0x4000);
            } else {
                xbase[i] = m * a.Cp;
                xhw[i] = 0;
            }
        } else {
            xbase[i] = 0;
            xhw[i] = -1;
        }
    }
    int x_ci = xc * 16, x_kh = 0, x_kw = 0, x_k = xc * 16;
    if (CONV) {
        while (x_ci >= a.Cp) {
            x_ci -= a.Cp;
            if (++x_kw == a.kw) { x_kw = 0; ++x_kh; }
        }
    }
    const int wc = tid % WCPR, wr0 = tid / WCPR;
    const size_t wrow_bytes = W4 ? (size_t)a.Kpad / 4 : (size_t)a.Kpad / 2;
    const size_t prow_words = (size_t)a.Kpad / 32;

    uint4 xreg[XLD], wreg[WLD], preg;
    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < XLD; ++i) {
            bool ok = (xhw[i] != -1) && (x_k < a.Kreal);
            int off;
            if (CONV) {
                const int hi = (xhw[i] >> 16) - 0x4000 + x_kh, wi = (xhw[i] & 0xffff) - 0x4000 + x_kw;
                ok = ok && ((unsigned)hi < (unsigned)a.H) && ((unsigned)wi < (unsigned)a.W);
                off = xbase[i] + (x_kh * a.W + x_kw) * a.Cp + x_ci;
            } else {
                off = xbase[i] + x_k;
            }
            xreg[i] = ok ? *reinterpret_cast<const uint4*>(a.x + off) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const int row = wr0 + WROWS_PER_PASS * i;
            const bool ok = (row < BW) && (n0 + row < a.N);
            wreg[i] = ok ? *reinterpret_cast<const uint4*>(a.wrows + (size_t)(n0 + row) * wrow_bytes + (size_t)kt * WROWB + wc * 16)
                         : make_uint4(0, 0, 0, 0);
        }
        preg = (tid < BW && n0 + tid < a.N) ? *reinterpret_cast<const uint4*>(pos_rows + (size_t)(n0 + tid) * prow_words + (size_t)kt * 4)
                                            : make_uint4(0, 0, 0, 0);
        x_k += 128;
        if (CONV) {
            x_ci += 128;
            while (x_ci >= a.Cp) {
                x_ci -= a.Cp;
                if (++x_kw == a.kw) { x_kw = 0; ++x_kh; }
            }
        }
    };
    auto w_off = [&](int row, int c) -> int { return W4 ? row * 32 + c * 16 : lds_off<64>(row, c); };
    auto store_lds = [&](int stage) {
        uint8_t* xs = smem + stage * STAGE;
        uint8_t* ws = xs + XTILE;
        uint32_t* ps = reinterpret_cast<uint32_t*>(ws + WTILE);
#pragma unroll
        for (int i = 0; i < XLD; ++i) *reinterpret_cast<uint4*>(xs + lds_off<XROWB>(xr0 + 32 * i, xc)) = xreg[i];
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const int row = wr0 + WROWS_PER_PASS * i;
            if (row < BW) *reinterpret_cast<uint4*>(ws + w_off(row, wc)) = wreg[i];
        }
        if (tid < BW) {
            ps[tid * 5 + 0] = preg.x; ps[tid * 5 + 1] = preg.y; ps[tid * 5 + 2] = preg.z; ps[tid * 5 + 3] = preg.w;
        }
    };

    v16f acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int wp = wave & 1, wq = wave >> 1;      // wave coordinates along the weight rows / the activation rows
    const int prow0 = wp * TP + l32, qrow0 = wq * TQ + l32;
    const GenFmt nofmt{0, 0, 0};

    auto compute = [&](int stage) {
        const uint8_t* xs = smem + stage * STAGE;
        const uint8_t* ws = xs + XTILE;
        const uint32_t* ps = reinterpret_cast<const uint32_t*>(ws + WTILE);
#pragma unroll
        for (int c = 0; c < 4; ++c) {                  // four chunks of 32 k
            v8bf af[MI];
            int pidx[MI];
            v16bf bfr[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int row = prow0 + 32 * i;
                if (W4) {
                    const uint32_t v = *reinterpret_cast<const uint32_t*>(ws + row * 32 + c * 8 + g * 4);
                    af[i] = decode8<WKIND>(v, 0u, nofmt);
                } else {
                    const uint2 v = *reinterpret_cast<const uint2*>(ws + lds_off<64>(row, c) + g * 8);
                    af[i] = decode8<WKIND>(v.x, v.y, nofmt);
                }
                pidx[i] = (int)((ps[row * 5 + c] >> (16 * g)) & 0xffffu);
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const uint4 v = *reinterpret_cast<const uint4*>(xs + lds_off<XROWB>(qrow0 + 32 * j, 2 * c + g));
                union { v16bf v; v8bf h[2]; } u;
                u.h[0] = decode8<OPK_FP8>(v.x, v.y, nofmt);
                u.h[1] = decode8<OPK_FP8>(v.z, v.w, nofmt);
                bfr[j] = u.v;
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(af[i], bfr[j], acc[i][j], pidx[i], 0, 0);
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

    // ---- epilogue: register r of a lane is weight row n = 8 (r / 4) + 4 g + r % 4 of block i, the lane is activation row m
    const float sxa = (a.sx_dev ? a.sx_dev[0] : a.sx) * a.alpha;
    if constexpr (CONV) {
        // NCHW: the lanes run along the pixel index, which is contiguous in y
        const int hw = a.Ho * a.Wo;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int m = m0 + wq * TQ + 32 * j + l32;
            if (m >= a.M) continue;
            const int bi = m / hw;
            float* ybase = a.y + (size_t)bi * a.N * hw + (m - bi * hw);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int n = n0 + wp * TP + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (n < a.N) ybase[(size_t)n * hw] = acc[i][j][r] * (sxa * a.sw[n]) + (a.bias ? a.bias[n] : 0.0f);
                }
        }
    } else {
        // row-major [M, N]: the lanes hold rows, so each 32 x 32 block crosses a wavefront-private LDS tile (the K loop
        // ended with a barrier; the ring is free) and leaves with 32 lanes on 128 consecutive bytes of a row
        float* tile = reinterpret_cast<float*>(smem) + wave * (32 * 33);
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int nb = n0 + wp * TP + 32 * i;            // first column of the block
            const int n = nb + l32;
            const float sc = n < a.N ? sxa * a.sw[n] : 0.0f;
            const float bv = (n < a.N && a.bias) ? a.bias[n] : 0.0f;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int mb = m0 + wq * TQ + 32 * j;         // first row of the block
#pragma unroll
                for (int r = 0; r < 16; ++r) tile[l32 * 33 + 8 * (r >> 2) + 4 * g + (r & 3)] = acc[i][j][r];
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) {
                    const int ml = 2 * rr + g;
                    const float v = tile[ml * 33 + l32];
                    if (mb + ml < a.M && n < a.N) a.y[(size_t)(mb + ml) * a.N + n] = v * sc + bv;
                }
            }
        }
    }
}

template <int BX, int BW, int WKIND, bool CONV>
static int launch_sparse_one(const GemmArgs& a, const uint32_t* pos_rows, hipStream_t st)
{
    constexpr int WROWB = kind_is_4bit(WKIND) ? 32 : 64;
    constexpr int smem = 2 * (BX * 128 + BW * WROWB + (BW * 20 + 15) / 16 * 16);
    const int tiles = ((a.M + BX - 1) / BX) * ((a.N + BW - 1) / BW);
    hipLaunchKernelGGL((gemm_sparse_kernel<BX, BW, WKIND, CONV>), dim3(tiles), dim3(256), smem, st, a, pos_rows);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

template <int WKIND, bool CONV>
static int launch_sparse_tiles(const GemmArgs& a, const uint32_t* pos_rows, hipStream_t st)
{
    const long big = (long)((a.M + 127) / 128) * ((a.N + 127) / 128);
    if (big >= 256) return launch_sparse_one<128, 128, WKIND, CONV>(a, pos_rows, st);
    return launch_sparse_one<64, 64, WKIND, CONV>(a, pos_rows, st);
}

// a.wrows: the kept-code rows; pos_rows: the position words.  Hardware E4M3 activations, E4M3 or E2M1 weights.
int launch_gemm_sparse(const GemmArgs& a, const uint32_t* pos_rows, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0) return FPQ_OK;
    if (a.xkind != OPK_FP8 || (a.wkind != OPK_FP8 && a.wkind != OPK_FP4) || a.acc_mode != FPQ_ACC_FP32 || a.yq || a.accumulate)
        return FPQ_ERR_UNSUPPORTED;
    if (a.wkind == OPK_FP8)
        return a.conv_out ? launch_sparse_tiles<OPK_FP8, true>(a, pos_rows, st) : launch_sparse_tiles<OPK_FP8, false>(a, pos_rows, st);
    return a.conv_out ? launch_sparse_tiles<OPK_FP4, true>(a, pos_rows, st) : launch_sparse_tiles<OPK_FP4, false>(a, pos_rows, st);
}

}  // namespace fpq
