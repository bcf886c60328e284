// Host-side declarations shared by the libfpq translation units: buffer geometry, the packed
// weight header, and the kernel launchers that api.hip calls after validating arguments.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/fpq.h"

namespace fpq {

struct QParams;
struct ScaleSrc;

// Channels of a channels-last code buffer: C rounded up to a whole 16-byte chunk.
static inline int64_t padded_channels(int64_t C) { return (C + 15) / 16 * 16; }

// A kernel that uses more than 64 KB of dynamic LDS must be told so once per device; `done` is the launcher's
// bit mask of the devices that have been (one static per kernel instantiation; setting it twice is harmless).
static inline bool allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const uint64_t bit = dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (done.load(std::memory_order_relaxed) & bit)) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    done.fetch_or(bit, std::memory_order_relaxed);
    return true;
}

// Length of a packed weight row: taps * Cp rounded up to the 128-code K step of the kernels.
static inline int64_t padded_k(int64_t Cin, int64_t taps) { return (taps * padded_channels(Cin) + 127) / 128 * 128; }

// Blocks of the first absmax pass (each folds >= 4096 elements; at most 1024 partials).
static inline int absmax_parts(size_t n)
{
    size_t g = (n + 4095) / 4096;
    return (int)(g > 1024 ? 1024 : g);
}

// Header in front of the packed rows.  The rows start kPackedRowsOffset bytes into the buffer so that, for a
// 256-byte aligned buffer, every 128-byte K chunk of a row is one whole cache line (a chunk that straddles two
// lines halves the rate of the LDS loads).
struct PackedHeader {
    uint32_t magic;      // 'FPQW'
    uint32_t layout;     // 1
    int32_t ebits, mbits, bias;
    float maxval;
    int64_t N, Cin;
    int32_t kh, kw;
    int32_t Cp, Kpad;
    uint32_t reserved[2];
};
static_assert(sizeof(PackedHeader) == 64, "header is 64 bytes");
constexpr size_t kPackedRowsOffset = 256;
constexpr uint32_t kPackedMagic = 0x57515046u;

// How an operand's codes reach the matrix unit.
enum OperandKind : int {
    OPK_FP8 = 0,      // (4, 3, b): hardware E4M3 bit pattern, value * 2^(7 - b)
    OPK_BF8 = 1,      // (5, 2, b): hardware E5M2 bit pattern, value * 2^(15 - b)
    OPK_FP4 = 2,      // (2, 1, b): hardware E2M1 bit pattern, value * 2^(1 - b), two codes per byte
    OPK_GENERIC8 = 3, // any other format, one code per byte, decoded arithmetically
    OPK_GENERIC4 = 4  // any other format of <= 4 bits, two codes per byte, decoded arithmetically
};

struct GemmArgs {
    const uint8_t* x;       // activation codes, channels-last [B, H, W, Cp] (linear: [M, K])
    const uint8_t* wrows;   // packed weight rows (after the header)
    const float* sw;        // [N]
    const float* bias;      // [N] or null
    const float* sx_dev;    // device scale or null
    float sx;               // host scale (used when sx_dev is null)
    float alpha;            // power of two that maps hardware-decoded values to format values
    float* y;
    int M, N;               // GEMM sizes (M = B * Ho * Wo)
    int Kpad;               // packed row length in codes
    int Kreal;              // taps * Cp: codes of x that exist
    int B, H, W, Cp;        // activation geometry (linear: B = M, H = W = 1)
    int Ho, Wo;
    int kh, kw, stride, pad;
    int conv_out;           // 1: y is NCHW [B, N, Ho, Wo]; 0: y is [M, N]
    int xkind, wkind;       // OperandKind
    int xe, xm, xb;         // activation format (for the generic decode)
    int we, wm, wb;         // weight format
    int acc_mode;
    uint32_t x_bytes;       // size of the activation code buffer (bound of the buffer loads)
    uint32_t w_bytes;       // size of the packed weight rows
    float* partial;         // split-K: splits x [M*N] partial results (null: no split)
    int splits;             // number of K slices (>= 1)
    int tile;               // GemmTile chosen by plan_gemm
    int accumulate;         // 1: add the result to y instead of storing it
    // Output as codes for the next quantized layer (not null): the fp32 result is quantized with Eq. (6)-(9)
    // (format below, per-tensor scale sy / sy_dev) and written one code per byte, row-major [M, ldq]
    // (a convolution's rows are its output pixels, i.e. channels-last); y is not written.
    uint8_t* yq;
    int ldq;                // codes per row: N rounded up to 16; columns N .. ldq - 1 receive code 0
    int ym, yb, yem;        // output format: mantissa bits, bias, e + m
    float yc;               // its max value
    int ykind;              // 1 / 2: the format is the hardware's E4M3 / E5M2 (conversion instruction); 0: any other
    float sy;               // host scale (used when sy_dev is null)
    const float* sy_dev;
    int act;                // 0, FPQ_ACT_SILU or FPQ_ACT_GEGLU: applied to the fp32 result before it is quantized
};

// Grouped linear layers (fpq_gemm_grouped): up to kGroupMax independent problems per launch, each launch taking the
// problems' pointers and sizes as a kernel argument (no copy to the device, so the call can be captured into a graph).
constexpr int kGroupMax = 32;
constexpr int kGroupAbsmaxParts = 32;   // partial maxima per problem in the dynamic-scale form
struct GroupedProblem {
    const float* x32;       // fp32 activations [M, K] (dynamic-scale form) or null
    const uint8_t* xcodes;  // activation codes [M, K]: the caller's, or where the grouped quantizer writes them
    const uint8_t* wrows;   // packed weight rows (after the header)
    const float* sw;        // [N]
    const float* bias;      // [N] or null
    const float* sx_dev;    // device scale of the codes; dynamic-scale form: where [scale, absmax] are published
    float* y;               // [M, N]
    float* partials;        // dynamic-scale form: kGroupAbsmaxParts partial maxima
    int M, N, K, Kpad;      // K = codes per row of x (a multiple of 16), Kpad = packed row length in codes
};
struct GroupedArgs {
    GroupedProblem p[kGroupMax];
    int count;
    GemmArgs common;        // formats, operand kinds, alpha, accumulate mode; the per-problem fields are filled in the kernel
};
static_assert(sizeof(GroupedArgs) <= 4096, "kernel arguments are limited to 4 KB");

// Kernel family / tile for a problem, and how many K slices share an output tile.
enum GemmTile : int {
    TILE_GENERIC = 0,    // register-staged 128x128 / 64x64 kernels: any shape
    TILE_256x160_S3 = 1, // LDS-DMA kernel, three stages: deep K
    TILE_128x160_S2 = 2  // LDS-DMA kernel, two stages, two workgroups per compute unit
};
struct GemmPlan {
    int tile;
    int splits;
};

// The large-tile kernels need N to be a multiple of 160 (every U-Net width, a multiple of 320, is) and pay off
// from a few hundred thousand outputs on.
// Deep K with enough 256-row tiles to fill the compute units takes the 256 x 160 tile with three
// stages (one workgroup per compute unit); everything else takes the 128 x 160 tile with two stages,
// of which two workgroups fit on a compute unit.  When the tile grid alone would leave compute units
// idle and K is deep, K is cut into slices (each split costs a reduction launch and a round trip of
// the partial sums, which only a deep K pays back): 2 to 4 slices of the 256-row tile when that gives
// about one work item per compute unit with at least 32 K steps each, otherwise one work item per compute
// unit of the 128-row tile (two when each keeps 20 K steps), with at least 8 K steps each.  Problems of a few tiles and a
// short K are bound by the length of their serial K loop and are sliced as well.  At most 256 MB of
// partial sums.
static inline GemmPlan plan_gemm(int64_t M, int64_t N, int64_t Kpad)
{
    GemmPlan p{TILE_GENERIC, 1};
    if (N % 160 != 0 || M < 1) return p;
    if (M <= 16) return p;   // at most 16 rows: the register-staged kernels (linear layers: one that splits K over its waves)
    const int64_t nk = Kpad / 128;
    // Small outputs with a short K: the register-staged kernel with its 64 x 64 tiles spreads them over more
    // workgroups and has a shorter serial K loop (M = 616, K = 768: 6.5 us against 12 us).
    if (M * N <= ((int64_t)2 << 20) && nk <= 20) return p;
    const int64_t tiles256 = ((M + 255) / 256) * (N / 160);
    const int64_t tiles = ((M + 127) / 128) * (N / 160);
    int64_t s = 1;
    if (nk >= 16 && tiles256 >= 192) {
        p.tile = TILE_256x160_S3;
        return p;
    }
    p.tile = TILE_128x160_S2;
    if (tiles256 < 192 && tiles256 >= 48 && nk >= 32 * ((256 + tiles256 / 2) / tiles256)) {
        p.tile = TILE_256x160_S3;
        s = (256 + tiles256 / 2) / tiles256;
    } else if (tiles < 192 && nk >= 16) {
        s = (256 + tiles - 1) / tiles;              // one work item per compute unit ...
        if (nk / (2 * s) >= 20) s *= 2;             // ... two when each still has 20 K steps
        if (s > nk / 8) s = nk / 8;
        if (s > 32) s = 32;
    } else if (tiles <= 16 && nk >= 4) {
        s = nk / 2 < 8 ? nk / 2 : 8;
    }
    while (s > 1 && s * M * N * 4 > ((int64_t)256 << 20)) --s;
    if (s < 1) s = 1;
    p.splits = (int)s;
    return p;
}
static inline size_t split_workspace_bytes(const GemmPlan& p, int64_t M, int64_t N)
{
    return p.splits > 1 ? (size_t)p.splits * (size_t)M * (size_t)N * sizeof(float) : 0;
}

// Encoding / bias search (Section V-A): at most 8 encodings x 128 bias candidates.
constexpr int kSearchMaxEncodings = 8;
constexpr int kSearchMaxCandidates = 1024;
struct SearchEnc {
    int32_t e, m, b0;   // b0 = 2^(e-1)
    float c0;           // Eq. (7) at b0
};
struct SearchArgs {
    int32_t n_enc, J;
    SearchEnc enc[kSearchMaxEncodings];
};
// Blocks of the search pass: 2048 elements per block and round, at most 1024 blocks.
static inline int search_blocks(size_t n)
{
    size_t g = (n + 2047) / 2048;
    return (int)(g > 1024 ? 1024 : g);
}
int launch_search(const float* x, size_t n, const SearchArgs& a, const float* absmax_dev, float* partial,
                  float* mse_out, fpq_search_result* result, hipStream_t st);

// Rounding learning (Section V-B): launchers of rounding.hip.
size_t rl_workspace_bytes(int64_t M, int64_t N, int64_t K);
int launch_rl_init(const float* w, const float* sw, int64_t N, int64_t K, const QParams& q, float* alpha, hipStream_t st);
int launch_rl_mask(const float* alpha, size_t n, uint8_t* mask, hipStream_t st);
int launch_rl_im2col(const float* x, int64_t B, int64_t C, int64_t H, int64_t W, int kh, int kw, int stride, int pad,
                     float* a, hipStream_t st);
int launch_rl_step(const float* w, const float* sw, int64_t N, int64_t K, const QParams& q, float* alpha, const float* a,
                   int64_t M, float lr, float reg_weight, float* loss_out, float* grad_out, void* workspace, hipStream_t st);

// Zero count (Section VI, "Sparsity"): blocks of the counting pass, each with a contiguous share of the bytes.
static inline int count_zeros_parts(size_t nbytes)
{
    const size_t p = (nbytes + 16383) / 16384;
    return p < 1 ? 1 : (p > 1024 ? 1024 : (int)p);
}
int launch_count_zeros(const void* x, int is_fp32, size_t n, int em, bool four_bit, unsigned long long* out,
                       unsigned long long* partial, hipStream_t st);
int launch_absmax(const float* x, size_t n, float maxval, float* absmax_out, float* scale_out, float* partial,
                  hipStream_t st);
int launch_absmax_partials(const float* x, size_t n, float* partial, hipStream_t st);
int launch_quantize_dynamic_small(const float* x, size_t n, const QParams& q, float maxval, float* publish, uint8_t* codes,
                                  hipStream_t st);
int launch_quantize(const float* x, size_t n, const QParams& q, bool four_bit, const ScaleSrc& ss, uint8_t* codes,
                    hipStream_t st);
int launch_quantize_nhwc(const float* x, int64_t B, int64_t C, int64_t H, int64_t W, const QParams& q,
                         const ScaleSrc& ss, uint8_t* codes, hipStream_t st);
int launch_dequantize(const uint8_t* codes, size_t n, int e, int m, int b, float scale, float* out, hipStream_t st);
int launch_pack_weights(const float* w, int64_t N, int64_t Cin, int taps, const QParams& q, bool four_bit,
                        const float* scale_in, const uint8_t* mask, uint8_t* packed_rows, float* scale_out,
                        uint8_t* codes_out, hipStream_t st);
int launch_gemm(const GemmArgs& a, hipStream_t st);
// One launch for a dynamically scaled linear layer with at most 16 rows (x: the fp32 activations; a.x is not used;
// codes [M, K] and publish [scale, absmax] receive what the two-launch form leaves in the workspace).
int launch_gemm_skinny_dynamic(const GemmArgs& a, const float* x, const QParams& qx, float maxval, uint8_t* codes,
                               float* publish, hipStream_t st);
// Grouped forms (gemm.hip, quant.hip): one launch each over all problems of g.
int launch_gemm_grouped(const GroupedArgs& g, hipStream_t st);                 // register-staged 64 x 64 tiles, any shape
bool skinny_grouped_applicable(const GroupedArgs& g);                           // all problems: at most 16 rows, <= 16 Ki activations
int launch_gemm_skinny_dynamic_grouped(const GroupedArgs& g, const QParams& qx, float maxval, hipStream_t st);
int launch_quantize_dynamic_grouped(const GroupedArgs& g, const QParams& qx, float maxval, hipStream_t st);
// Structured-sparse weight operand (gemm_sparse.hip).
int launch_pack_weights_sparse(const float* w, int64_t N, int64_t Cin, int taps, const QParams& q, bool four_bit,
                               const float* scale_in, const uint8_t* mask, uint8_t* code_rows, uint32_t* pos_rows,
                               float* scale_out, uint8_t* codes_out, unsigned long long* altered, hipStream_t st);
int launch_gemm_sparse(const GemmArgs& a, const uint32_t* pos_rows, hipStream_t st);
// Uniform integer baseline of Eq. (4) (igemm.hip).
int launch_int_params(const float* x, size_t n, int bits, fpq_int_params* out, float* partial, hipStream_t st);
int launch_int_quantize(const float* x, size_t n, int bits, float scale, int zp, const fpq_int_params* params_dev, uint8_t* codes,
                        hipStream_t st);
int launch_int_pack_weights(const float* w, int64_t N, int64_t K, int bits, uint8_t* rows, float* scale_out, int32_t* zp_out,
                            int32_t* rowsum_out, uint8_t* codes_out, hipStream_t st);
int launch_int_gemm(const uint8_t* x, float sx, int zx, const fpq_int_params* px_dev, const uint8_t* wrows, const int32_t* wsum,
                    int wbits, const float* sw, const int32_t* zw, const float* bias, float* y, int64_t M, int64_t N, int64_t K,
                    int32_t* xsum, hipStream_t st);
// Machine-ceiling probes (peaks.hip): kind 0 / 1 = register-only bf16 / 8-bit MFMA loop, 2 = device copy,
// 3 / 4 = bf16 MFMA with the conversions of a 64 x 160 / 32 x 160 wave tile, 5 = device fill.
int launch_probe(int kind, int iters, const void* src, void* dst, size_t bytes, int* grid_out, hipStream_t st);
bool gemm_dma_applicable(const GemmArgs& a);
int launch_gemm_dma(const GemmArgs& a, hipStream_t st);
int launch_gemm_dma_q(const GemmArgs& a, hipStream_t st);   // the same with the result as codes (a.yq)

}  // namespace fpq
