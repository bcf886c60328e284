// Quantized linear / convolution layer on ExMy codes for gfx950 (Section V-B: Y^q = W^q A).
//
// One kernel template serves linear layers and convolutions (implicit GEMM with M = B*Ho*Wo,
// K = kh*kw*Cp, N = Cout).  A workgroup of four wavefronts owns a BX x BW tile of the output
// (BX activation rows, BW weight rows) and walks K in steps of 128 codes:
//   global memory --16-byte loads--> registers --> LDS (xor-swizzled 16-byte chunks, two stages)
//   LDS --16-byte reads--> registers --> MFMA 32x32 blocks, fp32 accumulators
//   epilogue: acc * (sx * alpha * sw[n]) + bias[n], stored so that the 32 lanes of a half-wave
//   write consecutive addresses (along n for linear output, along the pixel index for NCHW output,
//   which is why a convolution feeds the weights as the MFMA row operand).
// Codes stay codes (1 byte, or 4 bits for FP4 weights) all the way into registers.  Two arithmetic
// back ends consume them:
//   ACC_FP32      codes are expanded to bf16 in registers (hardware scaled converts for E4M3 /
//                 E2M1 bit patterns, shifts and one multiply for any other ExMy) and multiplied by
//                 the bf16 MFMA, whose fp32 accumulation keeps every product bit;
//   ACC_FP8_MFMA  codes are fed to the 8-bit / 4-bit MFMA (32x32x64) directly.
// K ordering inside a 128-code step is private to this file: any order is valid as long as both
// operands use the same one, and each back end picks the order its register layout wants.
#include <type_traits>

#include "gemm_common.h"

namespace fpq {

// ---------------------------------------------------------------------------------- the kernel

// The work of one workgroup: output tile number `block` of problem a (smem: the workgroup's dynamic LDS).
template <int BX, int BW, int WGX, int WGW, int XKIND, int WKIND, int ACC, bool CONV>
__device__ __forceinline__ void gemm_tile(const GemmArgs& a, int block, uint8_t* smem)
{
    constexpr bool W4 = kind_is_4bit(WKIND);
    constexpr int XROWB = 128;                 // bytes of one activation tile row per K step
    constexpr int WROWB = W4 ? 64 : 128;
    constexpr int XTILE = BX * XROWB;
    constexpr int WTILE = BW * WROWB;
    constexpr int STAGE = XTILE + WTILE;
    constexpr int XLD = BX / 32;               // 16-byte chunks per lane and stage, activations
    constexpr int WCPR = WROWB / 16;           // chunks per weight row
    constexpr int WROWS_PER_PASS = 256 / WCPR;
    constexpr int WLD = (BW + WROWS_PER_PASS - 1) / WROWS_PER_PASS;
    // MFMA row operand P and lane operand Q: linear output wants lanes along n (P = activations),
    // NCHW output wants lanes along the pixel index (P = weights).
    constexpr int BP = CONV ? BW : BX, BQ = CONV ? BX : BW;
    constexpr int WGP = CONV ? WGW : WGX, WGQ = CONV ? WGX : WGW;
    constexpr int TP = BP / WGP, TQ = BQ / WGQ;
    constexpr int MI = TP / 32, NI = TQ / 32;
    static_assert(WGX * WGW == 4 && TP % 32 == 0 && TQ % 32 == 0, "tile shape");
    constexpr int PKIND = CONV ? WKIND : XKIND, QKIND = CONV ? XKIND : WKIND;
    constexpr int PROWB = CONV ? WROWB : XROWB, QROWB = CONV ? XROWB : WROWB;
    constexpr bool P4 = kind_is_4bit(PKIND), Q4 = kind_is_4bit(QKIND);
    constexpr int PFMT = mfma_fmt(PKIND), QFMT = mfma_fmt(QKIND);   // immediates of the MFMA

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int g = lane >> 5;

    // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8 XCDs; regroup them so
    // that each XCD (one L2) works on a contiguous run of tiles that share activation rows.
    const int tiles_w = (a.N + BW - 1) / BW;
    const int tiles_x = (a.M + BX - 1) / BX;
    const int ntiles = tiles_w * tiles_x;
    int bid = block;
    {
        const int per = ntiles >> 3;
        if (bid < (per << 3)) bid = (bid & 7) * per + (bid >> 3);
    }
    const int tx = bid / tiles_w, tw = bid - tx * tiles_w;
    const int m0 = tx * BX, n0 = tw * BW;

    // ---- per-lane load bookkeeping
    const int xc = tid & 7;                    // chunk column of this lane in the activation tile
    const int xr0 = tid >> 3;                  // first row; further rows are +32
    int xbase[XLD];                            // code offset of (pixel, channel 0), tap (0,0)
    int xhw[XLD];                              // (hi0 + 0x4000) << 16 | (wi0 + 0x4000), or -1 if row >= M
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
    int x_ci = xc * 16, x_kh = 0, x_kw = 0, x_k = xc * 16;   // K position of this lane's chunk
    if (CONV) {
        while (x_ci >= a.Cp) {
            x_ci -= a.Cp;
            if (++x_kw == a.kw) { x_kw = 0; ++x_kh; }
        }
    }
    const int wc = tid % WCPR;
    const int wr0 = tid / WCPR;
    const size_t wrow_bytes = W4 ? (size_t)a.Kpad / 2 : (size_t)a.Kpad;

    uint4 xreg[XLD], wreg[WLD];

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
            const int n = n0 + row;
            const bool ok = (row < BW) && (n < a.N);
            wreg[i] = ok ? *reinterpret_cast<const uint4*>(a.wrows + (size_t)n * wrow_bytes +
                                                          (size_t)kt * WROWB + wc * 16)
                         : make_uint4(0, 0, 0, 0);
        }
        // advance this lane's K position by one step
        x_k += 128;
        if (CONV) {
            x_ci += 128;
            while (x_ci >= a.Cp) {
                x_ci -= a.Cp;
                if (++x_kw == a.kw) { x_kw = 0; ++x_kh; }
            }
        }
    };
    auto store_lds = [&](int stage) {
        uint8_t* xs = smem + stage * STAGE;
        uint8_t* ws = xs + XTILE;
#pragma unroll
        for (int i = 0; i < XLD; ++i)
            *reinterpret_cast<uint4*>(xs + lds_off<XROWB>(xr0 + 32 * i, xc)) = xreg[i];
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const int row = wr0 + WROWS_PER_PASS * i;
            if (row < BW) *reinterpret_cast<uint4*>(ws + lds_off<WROWB>(row, wc)) = wreg[i];
        }
    };

    // ---- accumulators
    v16f acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int wp = CONV ? (wave % WGW) : (wave / WGW);   // wave coordinate along P
    const int wq = CONV ? (wave / WGW) : (wave % WGW);   // wave coordinate along Q
    const int prow0 = wp * TP + l32;
    const int qrow0 = wq * TQ + l32;
    const GenFmt pf = CONV ? GenFmt{a.we, a.wm, a.wb} : GenFmt{a.xe, a.xm, a.xb};
    const GenFmt qf = CONV ? GenFmt{a.xe, a.xm, a.xb} : GenFmt{a.we, a.wm, a.wb};

    auto compute = [&](int stage) {
        const uint8_t* xs = smem + stage * STAGE;
        const uint8_t* ws = xs + XTILE;
        const uint8_t* ps = CONV ? ws : xs;
        const uint8_t* qs = CONV ? xs : ws;
        if constexpr (ACC == FPQ_ACC_FP32) {
            // 128 codes = 4 rounds; in round j lane half g holds codes (2j+g)*16 .. +15 of the row and
            // feeds them to two bf16 k-steps of 8 codes each.
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint4 praw[MI], qraw[NI];
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int row = prow0 + 32 * i;
                    if (P4) {
                        uint2 v = *reinterpret_cast<const uint2*>(ps + lds_off<PROWB>(row, j) + g * 8);
                        praw[i] = make_uint4(v.x, v.y, 0, 0);
                    } else {
                        praw[i] = *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 2 * j + g));
                    }
                }
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const int row = qrow0 + 32 * i;
                    if (Q4) {
                        uint2 v = *reinterpret_cast<const uint2*>(qs + lds_off<QROWB>(row, j) + g * 8);
                        qraw[i] = make_uint4(v.x, v.y, 0, 0);
                    } else {
                        qraw[i] = *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 2 * j + g));
                    }
                }
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    v8bf pfr[MI], qfr[NI];
#pragma unroll
                    for (int i = 0; i < MI; ++i)
                        pfr[i] = P4 ? decode8<PKIND>(t ? praw[i].y : praw[i].x, 0u, pf)
                                    : decode8<PKIND>(t ? praw[i].z : praw[i].x, t ? praw[i].w : praw[i].y, pf);
#pragma unroll
                    for (int i = 0; i < NI; ++i)
                        qfr[i] = Q4 ? decode8<QKIND>(t ? qraw[i].y : qraw[i].x, 0u, qf)
                                    : decode8<QKIND>(t ? qraw[i].z : qraw[i].x, t ? qraw[i].w : qraw[i].y, qf);
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int jj = 0; jj < NI; ++jj)
                            acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pfr[i], qfr[jj], acc[i][jj], 0, 0, 0);
                }
            }
        } else {
            // 128 codes = two 64-code MFMA steps.  Within a step the instruction pairs byte i < 16 of an
            // 8-bit operand (lane half g) with K index 16g + i and byte 16 + i with 32 + 16g + i, and nibble
            // i of a 4-bit operand with K index 32g + i; the chunk choices below follow from that.
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                v8i pfr[MI], qfr[NI];
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int row = prow0 + 32 * i;
                    union { v8i v; uint4 q[2]; } u;
                    if (P4) {
                        u.q[0] = *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 2 * kk + g));
                        u.q[1] = make_uint4(0, 0, 0, 0);
                    } else {
                        u.q[0] = *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 4 * kk + g));
                        u.q[1] = *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 4 * kk + 2 + g));
                    }
                    pfr[i] = u.v;
                }
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const int row = qrow0 + 32 * i;
                    union { v8i v; uint4 q[2]; } u;
                    if (Q4) {
                        u.q[0] = *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 2 * kk + g));
                        u.q[1] = make_uint4(0, 0, 0, 0);
                    } else {
                        u.q[0] = *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 4 * kk + g));
                        u.q[1] = *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 4 * kk + 2 + g));
                    }
                    qfr[i] = u.v;
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int jj = 0; jj < NI; ++jj)
                        acc[i][jj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            pfr[i], qfr[jj], acc[i][jj], PFMT, QFMT, 0, 0, 0, 0);
            }
        }
    };

    // ---- main loop: two LDS stages, next step's global loads in flight during the MFMAs
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

    // ---- epilogue
    const float sxa = (a.sx_dev ? a.sx_dev[0] : a.sx) * a.alpha;
    // two copies of the stores, chosen once (with the choice per element the compiler loads y ahead of every
    // store, also when nothing is added)
    auto store_all = [&](auto add_to_y) {
        auto put = [&](float* yp, float v) {
            if constexpr (decltype(add_to_y)::value)
                *yp = v + *yp;
            else
                *yp = v;
        };
        if (!CONV) {
            // P = activations: acc[i][j][r] is (m, n) = (row block i, r -> 8(r/4) + 4g + r%4 ; lane -> n)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int n = n0 + wq * TQ + 32 * j + l32;
                if (n >= a.N) continue;
                const float sc = sxa * a.sw[n];
                const float bv = a.bias ? a.bias[n] : 0.0f;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = m0 + wp * TP + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (m < a.M) put(a.y + (size_t)m * a.N + n, acc[i][j][r] * sc + bv);
                    }
            }
        } else {
            // P = weights: rows are n, lanes are pixels m
            const int hw = a.Ho * a.Wo;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int m = m0 + wq * TQ + 32 * j + l32;
                if (m >= a.M) continue;
                const int bi = m / hw;
                const int pix = m - bi * hw;
                float* ybase = a.y + (size_t)bi * a.N * hw + pix;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int n = n0 + wp * TP + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (n < a.N) {
                            const float sc = sxa * a.sw[n];
                            const float bv = a.bias ? a.bias[n] : 0.0f;
                            put(ybase + (size_t)n * hw, acc[i][j][r] * sc + bv);
                        }
                    }
            }
        }
    };
    if (a.yq) {
        // codes out (row-major [M, ldq], one byte per output; columns N .. ldq - 1 get code 0)
        const QParams qy{a.ym, a.yb, a.yem, a.yc};
        const float ry = inv_scale(a.sy, a.sy_dev);
        if (!CONV) {
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int n = n0 + wq * TQ + 32 * j + l32;    // tiles start at multiples of 32: a block of 32 columns is one j
                const float sc = n < a.N ? sxa * a.sw[n] : 0.0f;
                const float bv = (n < a.N && a.bias) ? a.bias[n] : 0.0f;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = m0 + wp * TP + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                        float v = acc[i][j][r] * sc + bv;
                        if (a.act == FPQ_ACT_GEGLU) {
                            // lanes 0-15 of each 32: values, lanes 16-31: the gates of the same outputs (all lanes exchange)
                            v *= act_gelu_call(lane_xor16(v));
                            if (m < a.M && l32 < 16 && n < a.N)
                                a.yq[(size_t)m * a.ldq + ((n - l32) >> 1) + l32] = (uint8_t)quantize_nearest(v, ry, qy);
                        } else {
                            if (a.act == FPQ_ACT_SILU) v = act_silu_call(v);
                            if (m < a.M && n < a.ldq)
                                a.yq[(size_t)m * a.ldq + n] = n < a.N ? (uint8_t)quantize_nearest(v, ry, qy) : (uint8_t)0;
                        }
                    }
            }
        } else {
            // P = weights: a lane is a pixel m, its registers run over channels n (4 consecutive ones per r / 4)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int m = m0 + wq * TQ + 32 * j + l32;
                if (m >= a.M) continue;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int n = n0 + wp * TP + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (n < a.N) {
                            const float sc = sxa * a.sw[n];
                            const float bv = a.bias ? a.bias[n] : 0.0f;
                            float v = acc[i][j][r] * sc + bv;
                            if (a.act == FPQ_ACT_SILU) v = act_silu_call(v);
                            a.yq[(size_t)m * a.ldq + n] = (uint8_t)quantize_nearest(v, ry, qy);
                        } else if (n < a.ldq) {
                            a.yq[(size_t)m * a.ldq + n] = 0;
                        }
                    }
            }
        }
        return;
    }
    if (a.accumulate)
        store_all(std::true_type{});
    else
        store_all(std::false_type{});
}

template <int BX, int BW, int WGX, int WGW, int XKIND, int WKIND, int ACC, bool CONV>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    gemm_tile<BX, BW, WGX, WGW, XKIND, WKIND, ACC, CONV>(a, blockIdx.x, smem);
}

// Grouped linear layers: blockIdx.y picks the problem, blockIdx.x the output tile within it (the grid is as wide as
// the problem with the most tiles; workgroups beyond a problem's own tile count leave at once).
__device__ __forceinline__ GemmArgs grouped_problem_args(const GroupedArgs& g, int pi)
{
    GemmArgs a = g.common;
    const GroupedProblem& q = g.p[pi];
    a.x = q.xcodes;
    a.wrows = q.wrows;
    a.sw = q.sw;
    a.bias = q.bias;
    a.sx_dev = q.sx_dev;
    a.y = q.y;
    a.M = q.M; a.N = q.N; a.Kpad = q.Kpad; a.Kreal = q.K;
    a.B = q.M; a.H = 1; a.W = 1; a.Cp = q.K; a.Ho = 1; a.Wo = 1;
    return a;
}

template <int XKIND, int WKIND, int ACC>
__global__ __launch_bounds__(256) void gemm_grouped_kernel(const GroupedArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const GemmArgs a = grouped_problem_args(g, blockIdx.y);
    const int tiles = ((a.M + 63) / 64) * ((a.N + 63) / 64);
    if ((int)blockIdx.x >= tiles) return;
    gemm_tile<64, 64, 2, 2, XKIND, WKIND, ACC, false>(a, blockIdx.x, smem);
}

// ---------------------------------------------------------------------------------- dispatch

template <int BX, int BW, int WGX, int WGW, int XKIND, int WKIND, int ACC, bool CONV>
static int launch_one(const GemmArgs& a, hipStream_t st)
{
    constexpr int WROWB = kind_is_4bit(WKIND) ? 64 : 128;
    constexpr int smem = 2 * (BX * 128 + BW * WROWB);
    const int tiles = ((a.M + BX - 1) / BX) * ((a.N + BW - 1) / BW);
    auto kern = gemm_kernel<BX, BW, WGX, WGW, XKIND, WKIND, ACC, CONV>;
    if (smem > 64 * 1024) {
        static std::atomic<uint64_t> allowed{0};   // per instantiation
        if (!allow_dynamic_lds(reinterpret_cast<const void*>(kern), smem, allowed)) return FPQ_ERR_LAUNCH;
    }
    hipLaunchKernelGGL(kern, dim3(tiles), dim3(256), smem, st, a);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

template <int XKIND, int WKIND, int ACC, bool CONV>
static int launch_tiles(const GemmArgs& a, hipStream_t st)
{
    // Tile choice: the large tile when it still yields at least two waves of workgroups over the 256
    // compute units, otherwise the small one.
    const long big = (long)((a.M + 127) / 128) * ((a.N + 127) / 128);
    if (big >= 512) return launch_one<128, 128, 2, 2, XKIND, WKIND, ACC, CONV>(a, st);
    return launch_one<64, 64, 2, 2, XKIND, WKIND, ACC, CONV>(a, st);
}

template <int XKIND, int WKIND, int ACC>
static int launch_conv_or_linear(const GemmArgs& a, hipStream_t st)
{
    return a.conv_out ? launch_tiles<XKIND, WKIND, ACC, true>(a, st) : launch_tiles<XKIND, WKIND, ACC, false>(a, st);
}

// ---------------------------------------------------------------------------------- M <= 16
//
// Linear layers with at most 16 rows (the time-embedding projections of the U-Net: M = batch).  The work is a few
// MFLOP; what counts is the length of the dependent chain.  A workgroup owns 16 output columns; its four wavefronts
// split K in steps of 64 codes (two 16x16x32 bf16 MFMAs per step: A = the rows of x, padded to 16 with zeros, B = 16
// weight rows), keep up to five steps of loads in flight each, and add their partial blocks through LDS.
// Hardware E4M3 activations with E4M3 or E2M1 weights, fp32 accumulate, fp32 result.
typedef float v4f_t __attribute__((ext_vector_type(4)));

template <int WKIND>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const GemmArgs a)
{
    constexpr bool W4 = kind_is_4bit(WKIND);
    constexpr int U = 5;    // K = 1280, the width of the embedding layers, is one round of loads per wave
    __shared__ float red[3][64][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, kq = lane >> 4;        // row of x / weight row within the block; the lane's quarter of a step
    const int n0 = blockIdx.x * 16;
    const int K = a.Kreal;                            // codes per row of x (a multiple of 16)
    const int nsteps = (K + 63) / 64;                 // a step = 64 codes = two MFMAs
    const bool has_m = r16 < a.M, has_n = n0 + r16 < a.N;
    const uint8_t* xrow = a.x + (size_t)(has_m ? r16 : 0) * K;
    const uint8_t* wrow = a.wrows + (size_t)(has_n ? n0 + r16 : 0) * (W4 ? a.Kpad / 2 : a.Kpad);
    const GenFmt nofmt{0, 0, 0};
    v4f_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
    // Which k a lane feeds to which MFMA is free as long as both operands agree: the lane takes the 16 consecutive
    // codes 64 s + 16 kq .. + 15 of its row in one load (the four lanes of a row read 64 contiguous bytes), the
    // first eight go to the step's first MFMA, the other eight to its second.
    for (int s0 = wave; s0 < nsteps; s0 += 4 * U) {
        uint4 xv[U], wv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = 64 * (s0 + 4 * u) + 16 * kq;         // K % 16 == 0: the 16 codes lie inside the row or outside
            const bool in = s0 + 4 * u < nsteps && k < K;
            xv[u] = (in && has_m) ? *reinterpret_cast<const uint4*>(xrow + k) : make_uint4(0u, 0u, 0u, 0u);
            if (W4) {
                const uint2 t = (in && has_n) ? *reinterpret_cast<const uint2*>(wrow + k / 2) : make_uint2(0u, 0u);
                wv[u] = make_uint4(t.x, 0u, t.y, 0u);
            } else {
                wv[u] = (in && has_n) ? *reinterpret_cast<const uint4*>(wrow + k) : make_uint4(0u, 0u, 0u, 0u);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(decode8<OPK_FP8>(xv[u].x, xv[u].y, nofmt),
                                                          decode8<WKIND>(wv[u].x, wv[u].y, nofmt), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(decode8<OPK_FP8>(xv[u].z, xv[u].w, nofmt),
                                                          decode8<WKIND>(wv[u].z, wv[u].w, nofmt), acc, 0, 0, 0);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave - 1][lane][r] = acc[r];
    }
    __syncthreads();
    if (wave == 0) {
        // acc[r]: row 4 (lane / 16) + r of x, column lane % 16 of the block
        const int n = n0 + r16;
        if (n < a.N) {
            const float sc = (a.sx_dev ? a.sx_dev[0] : a.sx) * a.alpha * a.sw[n];
            const float bv = a.bias ? a.bias[n] : 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = 4 * kq + r;
                if (m < a.M) a.y[(size_t)m * a.N + n] = (acc[r] + red[0][lane][r] + red[1][lane][r] + red[2][lane][r]) * sc + bv;
            }
        }
    }
}

// The same layer straight from the fp32 activations with a dynamic per-tensor scale (x of at most 16 Ki elements,
// rows of K % 16 == 0 values): every workgroup finds max |x| itself (the tensor is a few tens of KB, read from L2),
// quantizes it into LDS and runs the MFMA steps of gemm_skinny_kernel on those codes: one launch instead of the
// quantizer's and the layer's.  The weight loads of the first round go out before the activations are touched.
// Codes, scale, K split and summation order are those of the two-launch form, so the result is bit-identical.
template <int WKIND>
__device__ __forceinline__ void gemm_skinny_dynamic_block(const GemmArgs& a, int block, const float4* __restrict__ x4, int n4,
                                                          const QParams& qx, float maxval, uint32_t* __restrict__ codes_out,
                                                          float* __restrict__ publish)
{
    constexpr bool W4 = kind_is_4bit(WKIND);
    constexpr int U = 5;
    __shared__ float red[3][64][4];
    __shared__ float part[4];
    __shared__ __attribute__((aligned(16))) uint8_t xcodes[16384];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const int n0 = block * 16;
    const int K = a.Kreal;
    const int nsteps = (K + 63) / 64;
    const bool has_m = r16 < a.M, has_n = n0 + r16 < a.N;
    const uint8_t* wrow = a.wrows + (size_t)(has_n ? n0 + r16 : 0) * (W4 ? a.Kpad / 2 : a.Kpad);
    const GenFmt nofmt{0, 0, 0};
    auto load_w = [&](int s) -> uint4 {
        const int k = 64 * s + 16 * kq;
        const bool in = s < nsteps && k < K && has_n;
        if (W4) {
            const uint2 t = in ? *reinterpret_cast<const uint2*>(wrow + k / 2) : make_uint2(0u, 0u);
            return make_uint4(t.x, 0u, t.y, 0u);
        }
        return in ? *reinterpret_cast<const uint4*>(wrow + k) : make_uint4(0u, 0u, 0u, 0u);
    };
    uint4 wv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) wv[u] = load_w(wave + 4 * u);
    // ---- max |x|, scale, codes into LDS (element order of x: row-major [M, K])
    float4 v[16];
    float m = 0.0f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int i = e * 256 + threadIdx.x;
        v[e] = i < n4 ? x4[i] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v[e].x), fabsf(v[e].y)), fmaxf(fabsf(v[e].z), fabsf(v[e].w))));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) part[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    const float sx = (m == 0.0f) ? 1.0f : __fdiv_rn(m, maxval);
    const float rx = __fdiv_rn(1.0f, sx);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int i = e * 256 + threadIdx.x;
        if (i < n4) {
            const uint32_t c0 = quantize_nearest(v[e].x, rx, qx), c1 = quantize_nearest(v[e].y, rx, qx);
            const uint32_t c2 = quantize_nearest(v[e].z, rx, qx), c3 = quantize_nearest(v[e].w, rx, qx);
            const uint32_t word = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
            reinterpret_cast<uint32_t*>(xcodes)[i] = word;
            if (block == 0) codes_out[i] = word;      // the first workgroup leaves codes and scale where the
        }                                                  // two-launch form does, for inspection
    }
    if (block == 0 && threadIdx.x == 0) {
        publish[0] = sx;
        publish[1] = m;
    }
    __syncthreads();
    // ---- the MFMA steps of gemm_skinny_kernel, activations from LDS
    const uint8_t* xrow = xcodes + (size_t)(has_m ? r16 : 0) * K;
    v4f_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s0 = wave; s0 < nsteps; s0 += 4 * U) {
        if (s0 != wave) {
#pragma unroll
            for (int u = 0; u < U; ++u) wv[u] = load_w(s0 + 4 * u);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = 64 * (s0 + 4 * u) + 16 * kq;
            const bool in = s0 + 4 * u < nsteps && k < K && has_m;
            const uint4 xv = in ? *reinterpret_cast<const uint4*>(xrow + k) : make_uint4(0u, 0u, 0u, 0u);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(decode8<OPK_FP8>(xv.x, xv.y, nofmt),
                                                          decode8<WKIND>(wv[u].x, wv[u].y, nofmt), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(decode8<OPK_FP8>(xv.z, xv.w, nofmt),
                                                          decode8<WKIND>(wv[u].z, wv[u].w, nofmt), acc, 0, 0, 0);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave - 1][lane][r] = acc[r];
    }
    __syncthreads();
    if (wave == 0) {
        const int n = n0 + r16;
        if (n < a.N) {
            const float sc = sx * a.alpha * a.sw[n];
            const float bv = a.bias ? a.bias[n] : 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int mrow = 4 * kq + r;
                if (mrow < a.M)
                    a.y[(size_t)mrow * a.N + n] = (acc[r] + red[0][lane][r] + red[1][lane][r] + red[2][lane][r]) * sc + bv;
            }
        }
    }
}

template <int WKIND>
__global__ __launch_bounds__(256) void gemm_skinny_dynamic_kernel(const GemmArgs a, const float4* __restrict__ x4, int n4,
                                                                  QParams qx, float maxval, uint32_t* __restrict__ codes_out,
                                                                  float* __restrict__ publish)
{
    gemm_skinny_dynamic_block<WKIND>(a, blockIdx.x, x4, n4, qx, maxval, codes_out, publish);
}

// The same for a group of such layers in one launch: blockIdx.y picks the problem.
template <int WKIND>
__global__ __launch_bounds__(256) void gemm_skinny_dynamic_grouped_kernel(const GroupedArgs g, QParams qx, float maxval)
{
    const GemmArgs a = grouped_problem_args(g, blockIdx.y);
    if ((int)blockIdx.x * 16 >= a.N) return;
    const GroupedProblem& q = g.p[blockIdx.y];
    gemm_skinny_dynamic_block<WKIND>(a, blockIdx.x, reinterpret_cast<const float4*>(q.x32), (a.M * a.Kreal) >> 2, qx, maxval,
                                     reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(q.xcodes)), const_cast<float*>(q.sx_dev));
}

static bool skinny_applicable(const GemmArgs& a)
{
    return !a.conv_out && a.M <= 16 && a.acc_mode == FPQ_ACC_FP32 && a.xkind == OPK_FP8 &&
           (a.wkind == OPK_FP8 || a.wkind == OPK_FP4) && !a.yq && !a.accumulate && a.splits == 1;
}

// FPQ_OK when the one-launch form of a dynamically scaled linear layer with at most 16 rows ran,
// FPQ_ERR_UNSUPPORTED when it does not apply (shape, formats, alignment): the caller then quantizes and calls launch_gemm.
int launch_gemm_skinny_dynamic(const GemmArgs& a, const float* x, const QParams& qx, float maxval, uint8_t* codes,
                               float* publish, hipStream_t st)
{
    const size_t n = (size_t)a.M * a.Kreal;
    if (!skinny_applicable(a) || a.M < 1 || a.N < 1 || n > 16384 || (a.Kreal & 15) || (reinterpret_cast<uintptr_t>(x) & 15))
        return FPQ_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)((a.N + 15) / 16));
    if (a.wkind == OPK_FP8)
        hipLaunchKernelGGL(gemm_skinny_dynamic_kernel<OPK_FP8>, grid, dim3(256), 0, st, a, reinterpret_cast<const float4*>(x),
                           (int)(n >> 2), qx, maxval, reinterpret_cast<uint32_t*>(codes), publish);
    else
        hipLaunchKernelGGL(gemm_skinny_dynamic_kernel<OPK_FP4>, grid, dim3(256), 0, st, a, reinterpret_cast<const float4*>(x),
                           (int)(n >> 2), qx, maxval, reinterpret_cast<uint32_t*>(codes), publish);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------------- grouped linear layers

bool skinny_grouped_applicable(const GroupedArgs& g)
{
    const GemmArgs& c = g.common;
    if (c.acc_mode != FPQ_ACC_FP32 || c.xkind != OPK_FP8 || (c.wkind != OPK_FP8 && c.wkind != OPK_FP4)) return false;
    for (int i = 0; i < g.count; ++i) {
        const GroupedProblem& q = g.p[i];
        if (q.M > 16 || !q.x32 || (size_t)q.M * q.K > 16384 || (q.K & 15) || (reinterpret_cast<uintptr_t>(q.x32) & 15))
            return false;
    }
    return true;
}

int launch_gemm_skinny_dynamic_grouped(const GroupedArgs& g, const QParams& qx, float maxval, hipStream_t st)
{
    int maxn = 0;
    for (int i = 0; i < g.count; ++i) maxn = g.p[i].N > maxn ? g.p[i].N : maxn;
    const dim3 grid((unsigned)((maxn + 15) / 16), (unsigned)g.count);
    if (g.common.wkind == OPK_FP8)
        hipLaunchKernelGGL(gemm_skinny_dynamic_grouped_kernel<OPK_FP8>, grid, dim3(256), 0, st, g, qx, maxval);
    else
        hipLaunchKernelGGL(gemm_skinny_dynamic_grouped_kernel<OPK_FP4>, grid, dim3(256), 0, st, g, qx, maxval);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

template <int XKIND, int WKIND, int ACC>
static int launch_grouped_one(const GroupedArgs& g, hipStream_t st)
{
    constexpr int WROWB = kind_is_4bit(WKIND) ? 64 : 128;
    constexpr int smem = 2 * (64 * 128 + 64 * WROWB);
    int maxt = 0;
    for (int i = 0; i < g.count; ++i) {
        const int t = ((g.p[i].M + 63) / 64) * ((g.p[i].N + 63) / 64);
        maxt = t > maxt ? t : maxt;
    }
    hipLaunchKernelGGL((gemm_grouped_kernel<XKIND, WKIND, ACC>), dim3((unsigned)maxt, (unsigned)g.count), dim3(256), smem, st, g);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

int launch_gemm_grouped(const GroupedArgs& g, hipStream_t st)
{
    const GemmArgs& a = g.common;
    if (g.count <= 0) return FPQ_OK;
    if (a.acc_mode == FPQ_ACC_FP8_MFMA) {
        if (a.xkind == OPK_FP8 && a.wkind == OPK_FP8) return launch_grouped_one<OPK_FP8, OPK_FP8, FPQ_ACC_FP8_MFMA>(g, st);
        if (a.xkind == OPK_FP8 && a.wkind == OPK_FP4) return launch_grouped_one<OPK_FP8, OPK_FP4, FPQ_ACC_FP8_MFMA>(g, st);
        return FPQ_ERR_UNSUPPORTED;
    }
    if (a.xkind == OPK_FP8 && a.wkind == OPK_FP8) return launch_grouped_one<OPK_FP8, OPK_FP8, FPQ_ACC_FP32>(g, st);
    if (a.xkind == OPK_FP8 && a.wkind == OPK_FP4) return launch_grouped_one<OPK_FP8, OPK_FP4, FPQ_ACC_FP32>(g, st);
    if (kind_is_4bit(a.wkind)) return launch_grouped_one<OPK_GENERIC8, OPK_GENERIC4, FPQ_ACC_FP32>(g, st);
    return launch_grouped_one<OPK_GENERIC8, OPK_GENERIC8, FPQ_ACC_FP32>(g, st);
}

int launch_gemm(const GemmArgs& a, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0) return FPQ_OK;
    if (skinny_applicable(a)) {
        const dim3 grid((unsigned)((a.N + 15) / 16));
        if (a.wkind == OPK_FP8)
            hipLaunchKernelGGL(gemm_skinny_kernel<OPK_FP8>, grid, dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL(gemm_skinny_kernel<OPK_FP4>, grid, dim3(256), 0, st, a);
        return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
    }
    if (gemm_dma_applicable(a)) return launch_gemm_dma(a, st);
    if (a.splits > 1) return FPQ_ERR_UNSUPPORTED;   // plan_gemm only splits for the large-tile kernels
    if (a.acc_mode == FPQ_ACC_FP8_MFMA) {
        if (a.xkind == OPK_FP8 && a.wkind == OPK_FP8) return launch_conv_or_linear<OPK_FP8, OPK_FP8, FPQ_ACC_FP8_MFMA>(a, st);
        if (a.xkind == OPK_FP8 && a.wkind == OPK_FP4) return launch_conv_or_linear<OPK_FP8, OPK_FP4, FPQ_ACC_FP8_MFMA>(a, st);
        if (a.xkind == OPK_FP8 && a.wkind == OPK_BF8) return launch_conv_or_linear<OPK_FP8, OPK_BF8, FPQ_ACC_FP8_MFMA>(a, st);
        if (a.xkind == OPK_BF8 && a.wkind == OPK_FP8) return launch_conv_or_linear<OPK_BF8, OPK_FP8, FPQ_ACC_FP8_MFMA>(a, st);
        if (a.xkind == OPK_BF8 && a.wkind == OPK_BF8) return launch_conv_or_linear<OPK_BF8, OPK_BF8, FPQ_ACC_FP8_MFMA>(a, st);
        if (a.xkind == OPK_BF8 && a.wkind == OPK_FP4) return launch_conv_or_linear<OPK_BF8, OPK_FP4, FPQ_ACC_FP8_MFMA>(a, st);
        return FPQ_ERR_UNSUPPORTED;
    }
    if (a.xkind == OPK_FP8 && a.wkind == OPK_FP8) return launch_conv_or_linear<OPK_FP8, OPK_FP8, FPQ_ACC_FP32>(a, st);
    if (a.xkind == OPK_FP8 && a.wkind == OPK_FP4) return launch_conv_or_linear<OPK_FP8, OPK_FP4, FPQ_ACC_FP32>(a, st);
    // every other pairing: arithmetic decode of both operands
    if (kind_is_4bit(a.wkind)) return launch_conv_or_linear<OPK_GENERIC8, OPK_GENERIC4, FPQ_ACC_FP32>(a, st);
    return launch_conv_or_linear<OPK_GENERIC8, OPK_GENERIC8, FPQ_ACC_FP32>(a, st);
}

}  // namespace fpq
