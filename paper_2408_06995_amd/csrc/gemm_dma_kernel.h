// Quantized linear / convolution layer on ExMy codes for gfx950: the large-tile kernel (template and its launcher;
// gemm_dma.hip instantiates it for fp32 results, gemm_dma_q.hip for results that leave as codes).
//
// A workgroup of four wavefronts owns a BX x BW tile (BX activation rows, BW weight rows; the
// wavefronts split the activation rows) and walks its K range in steps of 128 codes through an LDS
// ring of two or three stages.  Codes travel global memory -> LDS without touching registers:
// buffer_load_dwordx4 ... lds writes 64 lanes x 16 bytes to consecutive LDS addresses, and a lane
// whose element does not exist (row beyond M or N, padding pixel of the convolution, K beyond the
// real length) gives an offset outside the buffer, for which the hardware delivers zeros = code 0.
// The xor swizzle of the LDS tile (see lds_off) is applied on the global side, by choosing which
// 16-byte chunk a lane fetches.  Loads for step k + NSTAGE - 1 are issued while step k is computed;
// one s_waitcnt vmcnt + s_barrier per step, placed three quarters into the step, makes the next ring
// slot valid, and the rest of the step already reads and converts that slot's first fragments, so
// the MFMA stream never stops at a step boundary (the counts are spelled out at tail_sync).
//
// The kernel is persistent: the grid has at most one (256-row tile) or two (128-row tile) workgroups
// per compute unit and each workgroup walks a strided list of work items (output tile, K slice); the
// loads of the next item are in flight while the current item's results are scaled and stored, and
// the waits that follow an epilogue count its stores instead of draining them.
//
// Split-K: the K steps of an output tile can be cut into slices; slice s writes its scaled partial
// sums to partial[s] and a second kernel adds the slices into y.
//
// Codes out (QOUT): when the layer's result feeds another quantized layer, the epilogue quantizes it (Eq. (6)-(9),
// the next layer's format and per-tensor scale) and writes one byte per output instead of four.
#pragma once
#include <type_traits>

#include "gemm_common.h"

namespace fpq {

typedef int v4i __attribute__((ext_vector_type(4)));

// One wave-wide 16-byte-per-lane load from a buffer straight into LDS: lane i's bytes land at
// lds_addr + 16 i; a lane whose voff is not below the buffer's size gets zeros.  Written as inline
// assembly so that the compiler's wait-count insertion does not see an LDS write here (it would
// drain every outstanding load before each following LDS read); the waits are placed by hand in
// the main loop.  m0 carries the LDS base; nothing else in these kernels uses m0.
__device__ __forceinline__ void dma16(v4i rsrc, unsigned voff, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(rsrc)   // uniform, but may live in a VGPR
                 : "memory");
}

// Raw buffer descriptor: base address, no stride, size in bytes, 32-bit untyped data.
__device__ __forceinline__ v4i make_rsrc(const void* base, unsigned bytes)
{
    const unsigned long long b = reinterpret_cast<unsigned long long>(base);
    v4i r;
    r.x = (int)(unsigned)b;
    r.y = (int)((unsigned)(b >> 32) & 0xffffu);
    r.z = (int)bytes;
    r.w = 0x00020000;
    return r;
}

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

typedef float v4f __attribute__((ext_vector_type(4)));
// Results leave with streaming (non-temporal) stores: an output is far larger than the L2 and would
// otherwise push out the operand tiles that other workgroups are about to re-read.
__device__ __forceinline__ void store_out(float* p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void store_out4(float* p, float x, float y, float z, float w)
{
    const v4f v = {x, y, z, w};
    __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
}

// Four fp32 results -> four codes in one word (byte e = value e) with the activation quantizer of Eq. (6)-(9): multiply
// by r = fl32(1 / scale), clip to +-c, round to nearest even on the format's grid.  For the two formats the hardware
// converts (ykind 1: (4, 3, 7), 2: (5, 2, 15), any max value c of their grids up to the hardware's own) the rounding is
// one conversion instruction per pair of values, which after the clip is the same round-to-nearest-even on the same
// grid, subnormals and the sign of a zero result included; every other format takes the arithmetic encoder.
template <int YKIND>
__device__ __forceinline__ uint32_t codes_of4(float v0, float v1, float v2, float v3, float r, const QParams& q)
{
    if (YKIND != 0) {
        const float y0 = __builtin_amdgcn_fmed3f(__fmul_rn(v0, r), -q.c, q.c);
        const float y1 = __builtin_amdgcn_fmed3f(__fmul_rn(v1, r), -q.c, q.c);
        const float y2 = __builtin_amdgcn_fmed3f(__fmul_rn(v2, r), -q.c, q.c);
        const float y3 = __builtin_amdgcn_fmed3f(__fmul_rn(v3, r), -q.c, q.c);
        int w;
        if (YKIND == 1) {
            w = __builtin_amdgcn_cvt_pk_fp8_f32(y0, y1, 0, false);
            w = __builtin_amdgcn_cvt_pk_fp8_f32(y2, y3, w, true);
        } else {
            w = __builtin_amdgcn_cvt_pk_bf8_f32(y0, y1, 0, false);
            w = __builtin_amdgcn_cvt_pk_bf8_f32(y2, y3, w, true);
        }
        return (uint32_t)w;
    }
    return quantize_nearest(v0, r, q) | (quantize_nearest(v1, r, q) << 8) | (quantize_nearest(v2, r, q) << 16) |
           (quantize_nearest(v3, r, q) << 24);
}

// 4 x 4 byte transpose inside each quad of lanes: byte k of the word of quad lane b becomes byte b of the word of
// quad lane k.  Two exchange steps (with the lane one away, then two away), each one DPP move and one byte permute;
// sel1 / sel2 are the lane's permute selectors from transpose_selectors().
__device__ __forceinline__ uint32_t quad_transpose_bytes(uint32_t d, uint32_t sel1, uint32_t sel2)
{
    const uint32_t x = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)d, 0xB1, 0xF, 0xF, true);
    const uint32_t t = __builtin_amdgcn_perm(x, d, sel1);
    const uint32_t u = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, 0x4E, 0xF, 0xF, true);
    return __builtin_amdgcn_perm(u, t, sel2);
}
// Permute selectors (byte values 0-3: own word, 4-7: the partner's): step 1 keeps the own bytes of even rows in an
// even lane (of odd rows in an odd lane) and takes the partner's bytes of the same rows beside them; step 2 keeps
// one half and takes the partner's same half.
__device__ __forceinline__ void transpose_selectors(int quad_pos, uint32_t& sel1, uint32_t& sel2)
{
    sel1 = (quad_pos & 1) ? 0x03070105u : 0x06020400u;
    sel2 = (quad_pos & 2) ? 0x03020706u : 0x05040100u;
}

// Exchange helpers for the epilogue's 4 x 4 transpose: the value of the lane whose number differs in bit 0
// (or bit 1) within the same quad of lanes.
__device__ __forceinline__ float quad_xor1(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_xor2(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
}
// v[i] of quad lane b becomes what v[b] of quad lane i was (b0, b1 = bits of the lane's position in its quad).
__device__ __forceinline__ void quad_transpose(float (&v)[4], bool b0, bool b1)
{
#pragma unroll
    for (int p = 0; p < 4; p += 2) {
        const float lo = v[p], hi = v[p + 1];
        const float xhi = quad_xor1(hi), xlo = quad_xor1(lo);
        v[p] = b0 ? xhi : lo;
        v[p + 1] = b0 ? hi : xlo;
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const float lo = v[p], hi = v[p + 2];
        const float xhi = quad_xor2(hi), xlo = quad_xor2(lo);
        v[p] = b1 ? xhi : lo;
        v[p + 2] = b1 ? hi : xlo;
    }
}

template <int BX, int BW, int NSTAGE, int XKIND, int WKIND, int ACC, bool CONV, bool QOUT>
__global__ __launch_bounds__(256, ((BX <= 128 && NSTAGE <= 2) ? 2 : 1)) void gemm_dma_kernel(const GemmArgs a)
{
    constexpr bool W4 = kind_is_4bit(WKIND);
    constexpr int XROWB = 128;
    constexpr int WROWB = W4 ? 64 : 128;
    constexpr int XTILE = BX * XROWB;
    constexpr int WTILE = (BW * WROWB + 4095) / 4096 * 4096;   // whole 1-KB loads for each of 4 waves
    constexpr int STAGE = XTILE + WTILE;
    constexpr int XLD = XTILE / 4096;          // loads per wave and stage, activations
    constexpr int WLD = WTILE / 4096;          // loads per wave and stage, weights
    constexpr int LOADS = XLD + WLD;
    constexpr int XRPL = 8;                    // tile rows covered by one wave-wide load (128-byte rows)
    constexpr int WRPL = 1024 / WROWB;
    static_assert(XTILE % 4096 == 0, "activation tile must split evenly over the waves");
    // P = operand indexed by the accumulator registers, Q = operand indexed by the lane.
    // P = activations, Q = weights (see the epilogue for what that means for the stores).
    constexpr bool P_IS_W = false;
    constexpr int TX = BX / 4;                 // activation rows per wave
    constexpr int TP = P_IS_W ? BW : TX, TQ = P_IS_W ? TX : BW;
    constexpr int MI = TP / 32, NI = TQ / 32;
    static_assert(BW % 32 == 0 && TX % 32 == 0, "tile shape");
    constexpr int PKIND = P_IS_W ? WKIND : XKIND, QKIND = P_IS_W ? XKIND : WKIND;
    constexpr int PROWB = P_IS_W ? WROWB : XROWB, QROWB = P_IS_W ? XROWB : WROWB;
    constexpr bool P4 = kind_is_4bit(PKIND), Q4 = kind_is_4bit(QKIND);
    constexpr int PFMT = mfma_fmt(PKIND), QFMT = mfma_fmt(QKIND);

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int l32 = lane & 31;
    const int g = lane >> 5;

    // Work items = (output tile, K slice), tile-major.  Workgroup ids go round-robin over the 8 XCDs;
    // regroup them so that each XCD (one L2) holds a contiguous run of logical ids, hence of items,
    // which share activation rows.  Logical workgroup q takes items q, q + G, q + 2G, ...
    const int tiles_w = (a.N + BW - 1) / BW;
    const int tiles_x = (a.M + BX - 1) / BX;
    const int nitems = tiles_w * tiles_x * a.splits;
    const int G = gridDim.x;
    int q = blockIdx.x;
    {
        const int per = G >> 3;
        if (q < (per << 3)) q = (q & 7) * per + (q >> 3);
    }
    const int nk_all = a.Kpad / 128;

    // ---- load bookkeeping
    const v4i xrsrc = make_rsrc(a.x, a.x_bytes);
    const v4i wrsrc = make_rsrc(a.wrows, a.w_bytes);
    const unsigned lds0 = (unsigned)(size_t)((__attribute__((address_space(3))) void*)smem);
    constexpr unsigned OOB = 0x80000000u;

    // Activations: load i of this wave covers tile rows (4 i + wave) * 8 .. + 8; lane p holds row p / 8 of
    // them and LDS chunk p % 8, i.e. logical chunk (p % 8) ^ swizzle(row).  The swizzle term is the same
    // for all i, so a lane fetches the same K offset within every row it serves.
    const int xrl = lane >> 3;
    const int xc = (lane & 7) ^ ((wave * 4 + (lane >> 4)) & 7);
    unsigned xbase[XLD];                       // byte offset of the row's tap (0,0), channel 0 (wraps below zero for halo rows)
    unsigned xmask[XLD];                       // bit t: tap t of this row exists (inside the image, row < M); linear: bit 0
    int x_k = 0, x_ci = 0, x_kh = 0, x_kw = 0, x_tap = 0;   // K position of this lane's chunk
    int x_sel = 31;                            // x_tap, or 31 (a bit that is never set) once past the end of K
    unsigned x_delta = 0;                      // byte offset of (tap, channel) relative to xbase
    // Weights: same scheme on rows of WROWB bytes.
    const int wrl = W4 ? (lane >> 2) : (lane >> 3);
    const int wc = W4 ? ((lane & 3) ^ ((lane >> 4) & 3)) : ((lane & 7) ^ ((wave * 4 + (lane >> 4)) & 7));
    const unsigned wrow_bytes = W4 ? (unsigned)a.Kpad / 2 : (unsigned)a.Kpad;
    unsigned wbase[WLD];

    bool ihas = true;                          // false once this workgroup has no more loads to issue
    auto x_refresh = [&]() {
        x_sel = (ihas && x_k < a.Kreal) ? x_tap : 31;
        x_delta = CONV ? (unsigned)((x_kh * a.W + x_kw) * a.Cp + x_ci) : (unsigned)x_k;
    };

    int i_item = q;                            // item whose loads are being issued
    int i_rem = 0;                             // K steps of it not yet issued
    auto issue_setup = [&]() {
        const int tile = i_item / a.splits, sl = i_item - tile * a.splits;
        const int tx = tile / tiles_w, tw = tile - tx * tiles_w;
        const int m0 = tx * BX, n0 = tw * BW;
        const int kt0 = (int)((long)nk_all * sl / a.splits);
        i_rem = (int)((long)nk_all * (sl + 1) / a.splits) - kt0;
        int hi0[XLD], wi0[XLD];
#pragma unroll
        for (int i = 0; i < XLD; ++i) {
            const int m = m0 + (4 * i + wave) * XRPL + xrl;
            const bool rowok = m < a.M;
            hi0[i] = wi0[i] = 0;
            if (CONV) {
                const int hw = a.Ho * a.Wo;
                const int bi = m / hw;
                const int rem = m - bi * hw;
                const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
                hi0[i] = ho * a.stride - a.pad;
                wi0[i] = wo * a.stride - a.pad;
                xbase[i] = (unsigned)(((bi * a.H + hi0[i]) * a.W + wi0[i]) * a.Cp);
                xmask[i] = rowok ? 0u : 0x80000000u;   // bit 31 marks a row to skip while the taps are collected
            } else {
                xbase[i] = (unsigned)m * (unsigned)a.Cp;
                xmask[i] = rowok ? 1u : 0u;
            }
        }
        if (CONV) {
            int r = 0, c = 0;
            const int ntaps = a.kh * a.kw;
            for (int t = 0; t < ntaps; ++t) {
#pragma unroll
                for (int i = 0; i < XLD; ++i) {
                    const bool ok = ((unsigned)(hi0[i] + r) < (unsigned)a.H) & ((unsigned)(wi0[i] + c) < (unsigned)a.W);
                    xmask[i] |= ok ? (1u << t) : 0u;
                }
                if (++c == a.kw) { c = 0; ++r; }
            }
#pragma unroll
            for (int i = 0; i < XLD; ++i) xmask[i] = (xmask[i] & 0x80000000u) ? 0u : xmask[i];
        }
        x_k = kt0 * 128 + xc * 16;
        x_ci = x_k;
        x_kh = x_kw = x_tap = 0;
        if (CONV) {
            x_tap = x_k / a.Cp;
            x_ci = x_k - x_tap * a.Cp;
            x_kh = x_tap / a.kw;
            x_kw = x_tap - x_kh * a.kw;
        }
        x_refresh();
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const int row = (4 * i + wave) * WRPL + wrl;
            const int n = n0 + row;
            wbase[i] = (row < BW && n < a.N) ? (unsigned)n * wrow_bytes + (unsigned)kt0 * WROWB + wc * 16 : OOB;
        }
    };

    // Load number idx of a step (0 .. LOADS-1) into ring slot `stage`: four VALU instructions and the load.
    auto issue_one = [&](int idx, int stage) {
        const unsigned xs = lds0 + stage * STAGE;
        if (idx < XLD) {
            const unsigned off = ((xmask[idx] >> x_sel) & 1u) ? xbase[idx] + x_delta : OOB;
            dma16(xrsrc, off, xs + (4 * idx + wave) * 1024);
        } else {
            dma16(wrsrc, wbase[idx - XLD], xs + XTILE + (4 * (idx - XLD) + wave) * 1024);
        }
    };
    // After the LOADS loads of a step: move this lane's K position on by 128 codes.
    auto issue_advance = [&]() {
#pragma unroll
        for (int i = 0; i < WLD; ++i)
            if (wbase[i] != OOB) wbase[i] += WROWB;
        x_k += 128;
        if (CONV) {
            x_ci += 128;
            while (x_ci >= a.Cp) {
                x_ci -= a.Cp;
                ++x_tap;
                if (++x_kw == a.kw) { x_kw = 0; ++x_kh; }
            }
        }
        x_refresh();
    };

    // ---- accumulators
    v16f acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int xrow0 = wave * TX + l32;         // this lane's first activation row in the tile
    const int prow0 = P_IS_W ? l32 : xrow0;
    const int qrow0 = P_IS_W ? xrow0 : l32;
    const GenFmt wfm{a.we, a.wm, a.wb}, xfm{a.xe, a.xm, a.xb};
    const GenFmt pf = P_IS_W ? wfm : xfm, qf = P_IS_W ? xfm : wfm;

    // ---- FPQ_ACC_FP32: one K step = 128 codes = 4 rounds of LDS reads x 2 bf16 MFMA steps of 8 codes per
    // lane half.  In round j lane half g reads codes (2j+g)*16 .. +15 of each of its rows (both operands use
    // the same K order, so any order is valid).  The loop is software-pipelined by hand, one slot per MFMA:
    // after MFMA k of step st come the LDS read of fragment k for the next round and the converts of
    // fragment k for step st + 1.  A wavefront issues in order and is alone on its SIMD (or one of two), so
    // the matrix unit only stays busy if those reads and converts sit between the MFMAs; sched_barrier
    // keeps the slots apart.  The pipeline runs across K steps and work items: the last two MFMA steps of
    // a K step read and convert the first fragments of the next ring slot, after the wait + barrier that
    // make that slot valid (tail_sync), so raw[0] / frag[0] are live on entry to every K step.
    constexpr int NF = MI + NI, NM = MI * NI;
    uint4 raw[2][NF];
    v8bf frag[2][NF];
    auto lds_read = [&](int stage, int jr, int f) -> uint4 {
        const uint8_t* xs = smem + stage * STAGE;
        const uint8_t* ws = xs + XTILE;
        const uint8_t* ps = P_IS_W ? ws : xs;
        const uint8_t* qs = P_IS_W ? xs : ws;
        if (f < MI) {
            const int row = prow0 + 32 * f;
            if (P4) {
                const uint2 v = *reinterpret_cast<const uint2*>(ps + lds_off<PROWB>(row, jr) + g * 8);
                return make_uint4(v.x, v.y, 0, 0);
            }
            return *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 2 * jr + g));
        }
        const int row = qrow0 + 32 * (f - MI);
        if (Q4) {
            const uint2 v = *reinterpret_cast<const uint2*>(qs + lds_off<QROWB>(row, jr) + g * 8);
            return make_uint4(v.x, v.y, 0, 0);
        }
        return *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 2 * jr + g));
    };
    auto dec = [&](int st, int f) -> v8bf {
        const uint4 r = raw[(st >> 1) & 1][f];
        const int t = st & 1;
        if (f < MI)
            return P4 ? decode8<PKIND>(t ? r.y : r.x, 0u, pf) : decode8<PKIND>(t ? r.z : r.x, t ? r.w : r.y, pf);
        return Q4 ? decode8<QKIND>(t ? r.y : r.x, 0u, qf) : decode8<QKIND>(t ? r.z : r.x, t ? r.w : r.y, qf);
    };
    auto first_fragments = [&](int stage) {
#pragma unroll
        for (int f = 0; f < NF; ++f) raw[0][f] = lds_read(stage, 0, f);
#pragma unroll
        for (int f = 0; f < NF; ++f) frag[0][f] = dec(0, f);
    };

    // Wait until the loads of the next K step have landed, then meet the other waves: after the barrier
    // every wave's share of that ring slot is valid, and every wave has finished reading the ring slot
    // of the current step (its last LDS read was consumed an MFMA step ago), which the loads issued
    // from the next step on overwrite.  Buffer loads and stores of a wave retire in issue order, so
    // "vmcnt <= n" means that all but the n youngest operations are complete.  Younger than the wanted
    // group are the NSTAGE - 2 groups issued after it; and, while the wanted group still dates from
    // before the last epilogue (the first NSTAGE - 2 steps after it), also that epilogue's stores and the
    // two scale / bias loads of the item (the counter saturates at 63, hence the min).  With two stages
    // the wanted loads are themselves the youngest, so the wait is for zero.
    enum { W_NORMAL = 0, W_FIRST = 1, W_AFTER_STORES = 2, W_DRAIN = 3, W_AFTER_CODES = 4 };
    constexpr int SFULL = CONV ? MI * 4 * NI : MI * 16 * NI;   // store instructions of the epilogue of a whole tile
    constexpr int SCODES = MI * 4 * NI;                        // the same when the tile leaves as codes
    constexpr int AHEAD = (NSTAGE - 2) * LOADS;                // loads younger than the wanted group
    auto tail_sync = [&](int mode) {
        if (mode == W_DRAIN)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        else if (mode == W_NORMAL)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(AHEAD));
        else if (mode == W_FIRST)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(AHEAD + 2 < 63 ? AHEAD + 2 : 63));
        else if (!QOUT || mode == W_AFTER_STORES)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(AHEAD + 2 + SFULL < 63 ? AHEAD + 2 + SFULL : 63));
        else
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(AHEAD + 2 + SCODES < 63 ? AHEAD + 2 + SCODES : 63));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    auto compute = [&](int stage, int next_stage, int to_stage, int mode) {
#pragma unroll
        for (int st = 0; st < 8; ++st) {
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                const int i = k / NI, jj = k - i * NI;
                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[st & 1][i], frag[st & 1][MI + jj], acc[i][jj],
                                                                    0, 0, 0);
                if (st == 6 && k == 0) tail_sync(mode);
#pragma unroll
                for (int f = k; f < NF; f += NM) {
                    if ((st & 1) == 0) {
                        if (st < 6)
                            raw[((st >> 1) + 1) & 1][f] = lds_read(stage, (st >> 1) + 1, f);
                        else
                            raw[0][f] = lds_read(next_stage, 0, f);
                    }
                    frag[(st + 1) & 1][f] = dec((st + 1) & 7, f);
                }
                // the loads of the step NSTAGE - 1 ahead: one every third slot
                if ((st * NM + k) % 3 == 2 && (st * NM + k) / 3 < LOADS) issue_one((st * NM + k) / 3, to_stage);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        static_assert(3 * LOADS <= 6 * NM, "the loads of a step must be issued before its tail_sync");
    };

    // ---- FPQ_ACC_FP8_MFMA: codes feed the 8-bit / 4-bit MFMA directly, two 64-code MFMA steps per K step.  The
    // instruction pairs byte i < 16 of an 8-bit operand (lane half g) with K index 16g + i and byte 16 + i
    // with 32 + 16g + i, and nibble i of a 4-bit operand with K index 32g + i; the chunk choices follow.
    // Same pipeline as above with register fragments double-buffered per MFMA step: while the MFMAs of one
    // 64-code step run, the fragments of the next step are read from LDS (those of the next ring slot after
    // the tail_sync that opens the second step); the loads of the K step NSTAGE - 1 ahead go out two per slot
    // during the first step, so all of them precede the tail_sync.
    v8i frag8[2][NF];
    auto lds_read8 = [&](int stage, int kk, int f) -> v8i {
        const uint8_t* xs = smem + stage * STAGE;
        const uint8_t* ws = xs + XTILE;
        const uint8_t* ps = P_IS_W ? ws : xs;
        const uint8_t* qs = P_IS_W ? xs : ws;
        union { v8i v; uint4 q[2]; } u;
        if (f < MI) {
            const int row = prow0 + 32 * f;
            if (P4) {
                u.q[0] = *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 2 * kk + g));
                u.q[1] = make_uint4(0, 0, 0, 0);
            } else {
                u.q[0] = *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 4 * kk + g));
                u.q[1] = *reinterpret_cast<const uint4*>(ps + lds_off<PROWB>(row, 4 * kk + 2 + g));
            }
        } else {
            const int row = qrow0 + 32 * (f - MI);
            if (Q4) {
                u.q[0] = *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 2 * kk + g));
                u.q[1] = make_uint4(0, 0, 0, 0);
            } else {
                u.q[0] = *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 4 * kk + g));
                u.q[1] = *reinterpret_cast<const uint4*>(qs + lds_off<QROWB>(row, 4 * kk + 2 + g));
            }
        }
        return u.v;
    };
    auto first_fragments8 = [&](int stage) {
#pragma unroll
        for (int f = 0; f < NF; ++f) frag8[0][f] = lds_read8(stage, 0, f);
    };
    auto compute8 = [&](int stage, int next_stage, int to_stage, int mode) {
#pragma unroll
        for (int st = 0; st < 2; ++st) {
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                const int i = k / NI, jj = k - i * NI;
                acc[i][jj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag8[st][i], frag8[st][MI + jj], acc[i][jj],
                                                                           PFMT, QFMT, 0, 0, 0, 0);
                if (st == 1 && k == 0) tail_sync(mode);
#pragma unroll
                for (int f = k; f < NF; f += NM)
                    frag8[st ^ 1][f] = st == 0 ? lds_read8(stage, 1, f) : lds_read8(next_stage, 0, f);
                if (st == 0) {
                    if (2 * k < LOADS) issue_one(2 * k, to_stage);
                    if (2 * k + 1 < LOADS) issue_one(2 * k + 1, to_stage);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        static_assert(LOADS <= 2 * NM, "the loads of a step must be issued before its tail_sync");
    };

    // ---- epilogue of one work item: acc * (sx * alpha * sw[n]) + bias[n].
    // P = activations (accumulator registers run along m), Q = weights (lanes run along n), so the scale
    // and bias of a lane depend only on the column block j.  The BW scales and biases of a work item are
    // fetched into LDS (behind the ring, two alternating slots) by two loads of the same kind as the tile
    // loads, issued by every wave when the item starts: they retire in order with the tile loads, so no
    // wait of their own is needed before the K loop, and a missing bias (or a K slice other than the first)
    // is an out-of-range offset, which reads as zero.
    const float sxa = (a.sx_dev ? a.sx_dev[0] : a.sx) * a.alpha;
    constexpr int RING = NSTAGE * STAGE;
    const v4i swrsrc = make_rsrc(a.sw, (unsigned)a.N * 4u);
    const v4i brsrc = make_rsrc(a.bias, a.bias ? (unsigned)a.N * 4u : 0u);
    auto issue_scales = [&](int n0, int sl, int par) {
        const unsigned off = lane < BW / 4 ? (unsigned)(n0 * 4 + lane * 16) : OOB;
        dma16(swrsrc, off, lds0 + RING + par * 2048);
        dma16(brsrc, sl == 0 ? off : OOB, lds0 + RING + par * 2048 + 1024);
    };
    // Whole tiles take the fast path: a 4 x 4 transpose inside each quad of lanes (two DPP exchange steps)
    // turns "lane = output channel, 4 registers = 4 consecutive rows / pixels" into a layout in which
    // eight neighbouring lanes together hold 128 consecutive output bytes, so that every store
    // instruction writes whole cache lines, 16 bytes per lane:
    //   row-major [M, N]: the four registers r % 4 (rows) swap with the lane's position b in its quad
    //     (columns): afterwards lane (a, b) holds row 8 q + 4 g + b, columns 4 a .. 4 a + 3;
    //   NCHW: the four register groups q (pixels 8 q + 4 g .. + 3) swap with b (channels): afterwards
    //     lane (a, b) holds, in group q, channel 4 a + q and pixels 8 b + 4 g .. + 3.
    // Either way the scale and bias of the lane's values are the four entries 4 a .. 4 a + 3 of the
    // column block.  Returns the wait mode that the stores issued call for (see tail_sync).
    const QParams qy{a.ym, a.yb, a.yem, a.yc};
    const float ry = QOUT ? inv_scale(a.sy, a.sy_dev) : 0.0f;
    auto epilogue = [&](int m0, int n0, int sl, int par) -> int {
        const float* stab = reinterpret_cast<const float*>(smem + RING + par * 2048);
        const bool full = (m0 + BX <= a.M) && (n0 + BW <= a.N);   // whole tile inside the output
        const int mw = m0 + wave * TX;                           // first row of this wave
        const int qa = l32 >> 2, qb = l32 & 3;
        const bool b0 = qb & 1, b1 = qb & 2;
        if (QOUT && a.splits == 1) {
            // ---- codes out: quantize acc * scale + bias for the next layer, one byte per output, row-major
            // [M, ldq].  Whole tiles: a lane turns the four consecutive rows of each register group into four
            // codes of its column (one word), then a 4 x 4 byte transpose inside each quad of lanes leaves lane
            // (a, b) with row 8 q + 4 g + b, columns 4 a .. 4 a + 3 of the column block: one 32-bit store, and
            // eight lanes cover 32 consecutive bytes of a row.
            if (full && (a.ykind != 0 || a.act == 0)) {
                uint32_t sel1, sel2;
                transpose_selectors(qb, sel1, sel2);
                float sc[NI], bv[NI];
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    sc[j] = sxa * stab[32 * j + l32];
                    bv[j] = stab[256 + 32 * j + l32];
                }
                // the column blocks innermost: the five 32-byte pieces of a row's 160 bytes leave back to back.
                // One copy of the loops per conversion kind, chosen once per tile.
                auto codes_tile = [&](auto kind, auto activation) {
                    constexpr int YK = decltype(kind)::value;
                    constexpr int ACT = decltype(activation)::value;
                    // GEGLU halves the row: block j's 16 outputs sit at columns (n0 + 32 j) / 2 .. + 15
                    uint8_t* rowp = ACT == FPQ_ACT_GEGLU ? a.yq + (size_t)(mw + 4 * g + qb) * a.ldq + (n0 >> 1) + 4 * qa
                                                         : a.yq + (size_t)(mw + 4 * g + qb) * a.ldq + n0 + 4 * qa;
                    const size_t step = (size_t)8 * a.ldq;
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
#pragma unroll
                            for (int j = 0; j < NI; ++j) {
                                float v[4];
#pragma unroll
                                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q4 + e] * sc[j] + bv[j];
                                if (ACT == FPQ_ACT_SILU) {
#pragma unroll
                                    for (int e = 0; e < 4; ++e) v[e] = act_silu(v[e]);
                                }
                                if (ACT == FPQ_ACT_GEGLU) {
                                    // lanes 0-15 of each 32 hold the values, lanes 16-31 the gates of the same outputs.
                                    // One gelu serves two rows: the value lanes take the partner's gate of row e, the
                                    // gate lanes keep their own gate of row e + 1 and send the result back afterwards.
#pragma unroll
                                    for (int e = 0; e < 4; e += 2) {
                                        const float partner = lane_xor16(v[e]);      // every lane takes part
                                        const float ge = act_gelu(l32 < 16 ? partner : v[e + 1]);
                                        const float back = lane_xor16(ge);
                                        v[e] *= ge;            // meaningful in the value lanes only
                                        v[e + 1] *= back;
                                    }
                                }
                                const uint32_t row = quad_transpose_bytes(codes_of4<YK>(v[0], v[1], v[2], v[3], ry, qy), sel1, sel2);
                                if (ACT == FPQ_ACT_GEGLU) {
                                    if (l32 < 16) __builtin_nontemporal_store(row, reinterpret_cast<uint32_t*>(rowp + 16 * j));
                                } else {
                                    __builtin_nontemporal_store(row, reinterpret_cast<uint32_t*>(rowp + 32 * j));
                                }
                            }
                            rowp += step;
                        }
                };
                // the hardware formats get a copy per activation; the arithmetic encoder (rare as an output format,
                // and large) only the plain one, its activations go through the element-wise path below
                if (a.ykind == 1) {
                    if (a.act == FPQ_ACT_GEGLU)
                        codes_tile(std::integral_constant<int, 1>{}, std::integral_constant<int, FPQ_ACT_GEGLU>{});
                    else if (a.act == FPQ_ACT_SILU)
                        codes_tile(std::integral_constant<int, 1>{}, std::integral_constant<int, FPQ_ACT_SILU>{});
                    else
                        codes_tile(std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{});
                } else if (a.ykind == 2) {
                    if (a.act == FPQ_ACT_GEGLU)
                        codes_tile(std::integral_constant<int, 2>{}, std::integral_constant<int, FPQ_ACT_GEGLU>{});
                    else if (a.act == FPQ_ACT_SILU)
                        codes_tile(std::integral_constant<int, 2>{}, std::integral_constant<int, FPQ_ACT_SILU>{});
                    else
                        codes_tile(std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{});
                } else {
                    codes_tile(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
                }
                return W_AFTER_CODES;
            }
            // tiles that cross the edge of the output: byte stores; the padding columns N .. ldq - 1 get code 0
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int n = n0 + 32 * j + l32;
                const float sc1 = sxa * stab[32 * j + l32];
                const float bv1 = stab[256 + 32 * j + l32];
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = mw + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                        float v = acc[i][j][r] * sc1 + bv1;
                        if (a.act == FPQ_ACT_GEGLU) {
                            v *= act_gelu_call(lane_xor16(v));      // every lane takes part in the exchange
                            const int no = ((n0 + 32 * j) >> 1) + l32;
                            if (m < a.M && l32 < 16 && n < a.N) a.yq[(size_t)m * a.ldq + no] = (uint8_t)quantize_nearest(v, ry, qy);
                        } else {
                            if (a.act == FPQ_ACT_SILU) v = act_silu_call(v);
                            if (m < a.M && n < a.ldq)
                                a.yq[(size_t)m * a.ldq + n] = n < a.N ? (uint8_t)quantize_nearest(v, ry, qy) : (uint8_t)0;
                        }
                    }
            }
            return W_DRAIN;
        }
        // split-K: slice s writes its scaled partial sums to partial[s]; a second kernel adds the slices.  With
        // codes out the partial sums are kept row-major for convolutions too (the codes are channels-last).
        float* const yout = a.splits > 1 ? a.partial + (size_t)sl * ((size_t)a.M * a.N) : a.y;
        constexpr bool rowmajor = !CONV || QOUT;
        const int hw = rowmajor ? 4 : a.Ho * a.Wo;
        // adding to y (not to split-K partials, which the reduction adds to y) takes the element-wise path
        const bool accum = a.accumulate && a.splits == 1;
        const bool vec = full && !accum && ((hw & 3) == 0) && ((reinterpret_cast<uintptr_t>(yout) & 15) == 0);
        if (vec) {
            float4 sc4[NI], bv4[NI];
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const float4 s4 = *reinterpret_cast<const float4*>(stab + 32 * j + 4 * qa);
                sc4[j] = make_float4(s4.x * sxa, s4.y * sxa, s4.z * sxa, s4.w * sxa);
                bv4[j] = *reinterpret_cast<const float4*>(stab + 256 + 32 * j + 4 * qa);
            }
            if constexpr (!CONV || QOUT) {
                // row-major output keeps the plain layout: 32 lanes store 128 consecutive bytes of one row
                // (measured faster than 16-byte stores spread over eight rows)
                const unsigned lane_off = (unsigned)(4 * g * a.N + l32);
                float sc[NI], bv[NI];
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    sc[j] = sxa * stab[32 * j + l32];
                    bv[j] = stab[256 + 32 * j + l32];
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float* rowp = yout + (size_t)(mw + 32 * i + 8 * (r >> 2) + (r & 3)) * a.N + n0;   // uniform
#pragma unroll
                        for (int j = 0; j < NI; ++j) store_out(rowp + lane_off + 32 * j, acc[i][j][r] * sc[j] + bv[j]);
                    }
                return CONV ? W_DRAIN : W_AFTER_STORES;   // a convolution's wait counts are those of its NCHW stores
            } else {
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int m = mw + 32 * i + 8 * qb + 4 * g;   // hw % 4 == 0: the four pixels lie in one image
                    const int bi = m / hw;
                    const int pix = m - bi * hw;
                    float* mp = yout + ((size_t)bi * a.N + n0 + 4 * qa) * hw + pix;
#pragma unroll
                    for (int j = 0; j < NI; ++j) {
                        float v[4][4];   // [pixel e][group q]
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
#pragma unroll
                            for (int q4 = 0; q4 < 4; ++q4) v[e][q4] = acc[i][j][4 * q4 + e];
                            quad_transpose(v[e], b0, b1);
                        }
                        const float scq[4] = {sc4[j].x, sc4[j].y, sc4[j].z, sc4[j].w};
                        const float bvq[4] = {bv4[j].x, bv4[j].y, bv4[j].z, bv4[j].w};
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4)
                            store_out4(mp + (size_t)(32 * j + q4) * hw, v[0][q4] * scq[q4] + bvq[q4],
                                       v[1][q4] * scq[q4] + bvq[q4], v[2][q4] * scq[q4] + bvq[q4],
                                       v[3][q4] * scq[q4] + bvq[q4]);
                    }
                }
                return W_AFTER_STORES;
            }
        }
        // tiles that cross the edge of the output, or an output that does not allow 16-byte stores
        float sc[NI], bv[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            sc[j] = sxa * stab[32 * j + l32];
            bv[j] = stab[256 + 32 * j + l32];
        }
        // two copies of the loop, chosen once: with the choice inside, the compiler loads y ahead of every store
        // (the store makes the address known to be valid), which serialises the plain case as well
        auto element_wise = [&](auto add_to_y) {
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = mw + 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (m >= a.M) continue;
                    size_t base;
                    size_t nstride;
                    if (!rowmajor) {
                        const int bi = m / hw;
                        base = (size_t)bi * a.N * hw + (m - bi * hw);
                        nstride = (size_t)hw;
                    } else {
                        base = (size_t)m * a.N;
                        nstride = 1;
                    }
#pragma unroll
                    for (int j = 0; j < NI; ++j) {
                        const int n = n0 + 32 * j + l32;
                        if (n < a.N) {
                            float* yp = yout + base + (size_t)n * nstride;
                            const float v = acc[i][j][r] * sc[j] + bv[j];
                            if constexpr (decltype(add_to_y)::value)
                                *yp = v + *yp;
                            else
                                *yp = v;
                        }
                    }
                }
        };
        if (accum)
            element_wise(std::true_type{});
        else
            element_wise(std::false_type{});
        return W_DRAIN;
    };

    // ---- main loop over the K steps of all work items of this workgroup.  Each wave issues LOADS buffer
    // loads per step and they complete in order.  The loads run NSTAGE - 1 steps ahead of the MFMAs,
    // across item boundaries.  Every step issues one group of LOADS loads; once the work items run out
    // the group is a dummy (every offset out of range: zeros into a free ring slot, no memory traffic),
    // which keeps the control flow and the vmcnt arithmetic uniform.
    int istage = 0;
    ihas = i_item < nitems;
    if (ihas) issue_setup();
    auto issued = [&]() {
        issue_advance();
        istage = (istage + 1 == NSTAGE) ? 0 : istage + 1;
        if (ihas && --i_rem == 0) {
            i_item += G;
            ihas = i_item < nitems;
            if (ihas) {
                issue_setup();
            } else {
                x_sel = 31;
#pragma unroll
                for (int i = 0; i < WLD; ++i) wbase[i] = OOB;
            }
        }
    };
    if (!ihas) {
        x_sel = 31;
#pragma unroll
        for (int i = 0; i < WLD; ++i) wbase[i] = OOB;
    }
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) {
#pragma unroll
        for (int idx = 0; idx < LOADS; ++idx) issue_one(idx, istage);
        issued();
    }

    int cstage = 0;
    int par = 0;
    auto clear_acc = [&]() {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    };
    {
        // the first ring slot: its group is the oldest of the NSTAGE - 1 outstanding ones
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(LOADS * (NSTAGE - 2)));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if constexpr (ACC == FPQ_ACC_FP32)
            first_fragments(0);
        else
            first_fragments8(0);
        int after = W_FIRST;   // what precedes the current item: nothing, counted stores, or uncounted stores
        int since = 0;         // K steps since then
        for (int c_item = q; c_item < nitems; c_item += G) {
            const int tile = c_item / a.splits, sl = c_item - tile * a.splits;
            const int tx = tile / tiles_w, tw = tile - tx * tiles_w;
            const int nk = (int)((long)nk_all * (sl + 1) / a.splits) - (int)((long)nk_all * sl / a.splits);
            issue_scales(tw * BW, sl, par);
            for (int kt = 0; kt < nk; ++kt) {
                const int nstage = (cstage + 1 == NSTAGE) ? 0 : cstage + 1;
                const int mode = since < NSTAGE - 2 ? after : (int)W_NORMAL;
                if constexpr (ACC == FPQ_ACC_FP32)
                    compute(cstage, nstage, istage, mode);
                else
                    compute8(cstage, nstage, istage, mode);
                ++since;
                issued();
                cstage = nstage;
            }
            // the scale loads are older than the loads issued during the item's K steps (at least one group)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(LOADS));
            asm volatile("" ::: "memory");
            after = epilogue(tx * BX, tw * BW, sl, par);
            since = 0;
            par ^= 1;
            clear_acc();
        }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // no load may land in LDS after the workgroup has gone
}

// Adds up the K slices in the workspace (gemm_dma.hip): into y, or quantized into the code matrix.
int launch_splitk_reduce(const GemmArgs& a, hipStream_t st);

template <int BX, int BW, int NSTAGE, int XKIND, int WKIND, int ACC, bool CONV, bool QOUT>
static int launch_dma_one(const GemmArgs& a, hipStream_t st)
{
    constexpr int WROWB = kind_is_4bit(WKIND) ? 64 : 128;
    constexpr int smem = NSTAGE * (BX * 128 + (BW * WROWB + 4095) / 4096 * 4096) + 4096;   // ring + scale / bias slots
    const int tiles = ((a.M + BX - 1) / BX) * ((a.N + BW - 1) / BW);
    auto kern = gemm_dma_kernel<BX, BW, NSTAGE, XKIND, WKIND, ACC, CONV, QOUT>;
    static std::atomic<uint64_t> allowed{0};   // per instantiation
    if (!allow_dynamic_lds(reinterpret_cast<const void*>(kern), smem, allowed)) return FPQ_ERR_LAUNCH;
    const int nitems = tiles * a.splits;
    constexpr int max_wgs = (smem <= 80 * 1024) ? 512 : 256;   // resident workgroups: two per compute unit when the LDS allows
    hipLaunchKernelGGL(kern, dim3(nitems < max_wgs ? nitems : max_wgs), dim3(256), smem, st, a);
    if (a.splits > 1) return launch_splitk_reduce(a, st);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}


}  // namespace fpq
