// C ABI of libfpq (see include/fpq.h): argument validation on the host, then kernel launches on
// the caller's stream.  No entry point allocates, synchronizes or keeps a pointer.
#include <math.h>
#include <string.h>

#include "fpq_dev.h"
#include "fpq_host.h"

using namespace fpq;

namespace {

// |b| <= 64 keeps every grid value and the decoders' constants normal fp32 numbers; the last condition keeps the
// rounding constant of the encoder (2^23 times the step of the top binade, exponent field 2^e - 1 - b - m + 150)
// a finite fp32 number: it excludes only encodings whose largest value exceeds 2^(105 + m), e.g. E7M0 below bias 23.
bool em_ok(int e, int m, int b)
{
    return e >= 1 && m >= 0 && 1 + e + m <= 8 && b >= -64 && b <= 64 && (1 << e) - b - 1 <= 104 + m;
}

double eq7_max(int e, int m, int b) { return (2.0 - ldexp(1.0, -m)) * ldexp(1.0, (1 << e) - b - 1); }

// Is v a magnitude of the (e, m, b) grid (Eq. (5) plus the subnormal row)?
bool on_grid(int e, int m, int b, double v)
{
    if (!(v > 0.0) || v > eq7_max(e, m, b)) return false;
    double lowest_normal = ldexp(1.0, 1 - b);
    if (v < lowest_normal) {
        double f = ldexp(v, -(1 - b - m));
        return f == floor(f);
    }
    int ex;
    double fr = frexp(v, &ex);
    double f = ldexp(2.0 * fr - 1.0, m);
    return f == floor(f);
}

// Validates f and fills the kernel parameters (maxval 0 -> Eq. (7)).
int resolve_format(fpq_format_t f, QParams* q)
{
    if (!em_ok(f.ebits, f.mbits, f.bias)) return FPQ_ERR_FORMAT;
    double c = f.maxval == 0.0f ? eq7_max(f.ebits, f.mbits, f.bias) : (double)f.maxval;
    if (!(c == c) || !on_grid(f.ebits, f.mbits, f.bias, c)) return FPQ_ERR_FORMAT;
    if (q) {
        q->m = f.mbits;
        q->b = f.bias;
        q->em = f.ebits + f.mbits;
        q->c = (float)c;
    }
    return FPQ_OK;
}

bool scale_ok(float s)
{
    if (!(s > 0.0f) || isinf(s)) return false;
    float r = 1.0f / s;
    return !isinf(r);
}

bool is_four_bit(fpq_format_t f) { return 1 + f.ebits + f.mbits <= 4; }

// Which matrix-unit decoder reads this format's bit pattern, and the power of two between the
// hardware's value of a code and the format's value (hardware biases: E4M3 7, E5M2 15, E2M1 1).
// Hardware E4M3 has no value for the all-ones magnitude and hardware E5M2 none for the top
// exponent, so a format whose maxval reaches those codes decodes arithmetically instead.
int hardware_kind(fpq_format_t f, float c, bool weight, float* alpha)
{
    *alpha = 1.0f;
    if (f.ebits == 4 && f.mbits == 3 && c <= 448.0 * ldexp(1.0, 7 - f.bias)) {
        *alpha = (float)ldexp(1.0, 7 - f.bias);
        return OPK_FP8;
    }
    if (f.ebits == 5 && f.mbits == 2 && c <= 57344.0 * ldexp(1.0, 15 - f.bias)) {
        *alpha = (float)ldexp(1.0, 15 - f.bias);
        return OPK_BF8;
    }
    if (weight && f.ebits == 2 && f.mbits == 1) {
        *alpha = (float)ldexp(1.0, 1 - f.bias);
        return OPK_FP4;
    }
    return (weight && is_four_bit(f)) ? OPK_GENERIC4 : OPK_GENERIC8;
}

// Operand kinds the kernels are instantiated for, and the epilogue factor alpha.
int resolve_kinds(fpq_format_t fx, float cx, fpq_format_t fw, float cw, int acc_mode, int* xkind, int* wkind,
                  float* alpha)
{
    float ax, aw;
    int xk = hardware_kind(fx, cx, false, &ax);
    int wk = hardware_kind(fw, cw, true, &aw);
    if (is_four_bit(fx)) return FPQ_ERR_UNSUPPORTED;   // activations of <= 4 bits are not a case of the paper
    if (acc_mode == FPQ_ACC_FP8_MFMA) {
        if (xk == OPK_GENERIC8 || wk == OPK_GENERIC8 || wk == OPK_GENERIC4) return FPQ_ERR_UNSUPPORTED;
    } else if (acc_mode == FPQ_ACC_FP32) {
        if (!(xk == OPK_FP8 && (wk == OPK_FP8 || wk == OPK_FP4))) {
            xk = OPK_GENERIC8;
            wk = is_four_bit(fw) ? OPK_GENERIC4 : OPK_GENERIC8;
            ax = aw = 1.0f;
        }
    } else {
        return FPQ_ERR_UNSUPPORTED;
    }
    *xkind = xk;
    *wkind = wk;
    *alpha = ax * aw;
    return FPQ_OK;
}

__global__ void write_header_kernel(PackedHeader h, uint32_t* dst)
{
    const uint32_t* src = reinterpret_cast<const uint32_t*>(&h);
    if (threadIdx.x < 16) dst[threadIdx.x] = src[threadIdx.x];
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Scratch memory of fpq_gemm_noalloc: one copy per GPU the library runs on, held until the process ends.
// The array's name is only a host-side handle; scratch_on_current_device() asks the runtime for its address on the
// current device, once per device, and host code uses that pointer everywhere.
constexpr size_t kStaticScratchBytes = FPQ_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::atomic<void*> g_scratch_ptr[64];

int scratch_on_current_device(void** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FPQ_ERR_LAUNCH;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // two threads may both get here: they receive the same address
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FPQ_ERR_LAUNCH;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return FPQ_OK;
}

// Tail of the workspace in dynamic-scale mode: 1024 partial maxima, then [scale, absmax].
constexpr size_t kDynScaleBytes = 1024 * sizeof(float) + 256;

}  // namespace

extern "C" {

const char* fpq_strerror(int status)
{
    switch (status) {
        case FPQ_OK: return "ok";
        case FPQ_ERR_NULL: return "a required pointer is NULL";
        case FPQ_ERR_FORMAT: return "invalid ExMy format (bits, bias, or maxval not on the grid)";
        case FPQ_ERR_SCALE: return "scale must be positive and finite";
        case FPQ_ERR_SHAPE: return "invalid or inconsistent sizes";
        case FPQ_ERR_ALIGN: return "pointer or size not aligned as required";
        case FPQ_ERR_WORKSPACE: return "workspace missing or too small";
        case FPQ_ERR_LAUNCH: return "HIP launch failed";
        case FPQ_ERR_UNSUPPORTED: return "no kernel for these arguments";
        case FPQ_ERR_PACKED: return "packed weights do not match the arguments";
        default: return "unknown status";
    }
}

float fpq_format_max(int ebits, int mbits, int bias)
{
    if (!em_ok(ebits, mbits, bias)) return 0.0f;
    return (float)eq7_max(ebits, mbits, bias);
}

int fpq_format_check(fpq_format_t f) { return resolve_format(f, nullptr); }

int fpq_bias_to_scale(int ebits, int mbits, double real_bias, int32_t* int_bias, float* scale)
{
    if (!int_bias || !scale) return FPQ_ERR_NULL;
    if (!(real_bias == real_bias) || isinf(real_bias)) return FPQ_ERR_FORMAT;
    double fl = floor(real_bias);
    if (!em_ok(ebits, mbits, (int)fl)) return FPQ_ERR_FORMAT;
    *int_bias = (int32_t)fl;
    *scale = (float)exp2(fl - real_bias);
    return FPQ_OK;
}

size_t fpq_code_bytes(size_t n, fpq_format_t f) { return is_four_bit(f) ? (n + 1) / 2 : n; }

size_t fpq_absmax_workspace_size(size_t n)
{
    int p = absmax_parts(n);
    return (size_t)(p > 0 ? p : 1) * sizeof(float);
}

int fpq_absmax(const float* x, size_t n, float maxval, float* absmax_out, float* scale_out, void* workspace,
               size_t workspace_bytes, void* stream)
{
    if (!absmax_out || !workspace || (n && !x)) return FPQ_ERR_NULL;
    if (scale_out && !(maxval > 0.0f && !isinf(maxval))) return FPQ_ERR_FORMAT;
    if (workspace_bytes < fpq_absmax_workspace_size(n)) return FPQ_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(x) & 3) || (reinterpret_cast<uintptr_t>(workspace) & 3)) return FPQ_ERR_ALIGN;
    return launch_absmax(x, n, maxval, absmax_out, scale_out, static_cast<float*>(workspace),
                         static_cast<hipStream_t>(stream));
}

size_t fpq_rl_workspace_size(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return rl_workspace_bytes(M, N, K);
}

static int rl_check(const float* w, const float* sw, int64_t N, int64_t K, fpq_format_t f, QParams* q)
{
    int st = resolve_format(f, q);
    if (st) return st;
    if (N <= 0 || K <= 0 || N * K >= (int64_t)1 << 31) return FPQ_ERR_SHAPE;
    if (!w || !sw) return FPQ_ERR_NULL;
    return FPQ_OK;
}

int fpq_rl_init_alpha(const float* w, const float* sw, int64_t N, int64_t K, fpq_format_t f, float* alpha, void* stream)
{
    QParams q;
    int st = rl_check(w, sw, N, K, f, &q);
    if (st) return st;
    if (!alpha) return FPQ_ERR_NULL;
    return launch_rl_init(w, sw, N, K, q, alpha, static_cast<hipStream_t>(stream));
}

int fpq_rl_im2col(const float* x, int64_t B, int64_t C, int64_t H, int64_t W, int kh, int kw, int stride, int pad, float* a,
                  void* stream)
{
    if (B <= 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0) return FPQ_ERR_SHAPE;
    if (H + 2 * pad < kh || W + 2 * pad < kw || kh > 64 || kw > 64 || C * kh * kw >= (int64_t)1 << 24) return FPQ_ERR_SHAPE;
    if (!x || !a) return FPQ_ERR_NULL;
    return launch_rl_im2col(x, B, C, H, W, kh, kw, stride, pad, a, static_cast<hipStream_t>(stream));
}

int fpq_rl_mask(const float* alpha, size_t n, uint8_t* mask, void* stream)
{
    if (n && (!alpha || !mask)) return FPQ_ERR_NULL;
    if (n == 0) return FPQ_OK;
    return launch_rl_mask(alpha, n, mask, static_cast<hipStream_t>(stream));
}

int fpq_rl_step(const float* w, const float* sw, int64_t N, int64_t K, fpq_format_t f, float* alpha, const float* a,
                int64_t M, float lr, float reg_weight, float* loss_out, float* grad_out, void* workspace,
                size_t workspace_bytes, void* stream)
{
    QParams q;
    int st = rl_check(w, sw, N, K, f, &q);
    if (st) return st;
    if (M <= 0 || M * N >= (int64_t)1 << 31 || M >= (int64_t)1 << 23) return FPQ_ERR_SHAPE;
    if (!alpha || !a || !loss_out || !workspace) return FPQ_ERR_NULL;
    if (!(lr >= 0.0f) || isinf(lr) || !(reg_weight >= 0.0f) || isinf(reg_weight)) return FPQ_ERR_SCALE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return FPQ_ERR_ALIGN;
    if (workspace_bytes < rl_workspace_bytes(M, N, K)) return FPQ_ERR_WORKSPACE;
    return launch_rl_step(w, sw, N, K, q, alpha, a, M, lr, reg_weight, loss_out, grad_out, workspace,
                          static_cast<hipStream_t>(stream));
}

size_t fpq_count_zeros_workspace_size(size_t) { return 1024 * sizeof(unsigned long long); }

int fpq_count_zeros(const void* x, int x_kind, size_t n, fpq_format_t f, uint64_t* count_out, void* workspace,
                    size_t workspace_bytes, void* stream)
{
    if (!count_out || !workspace || (n && !x)) return FPQ_ERR_NULL;
    if (x_kind != FPQ_X_CODES && x_kind != FPQ_X_FP32 && x_kind != FPQ_X_CODES_BYTE) return FPQ_ERR_UNSUPPORTED;
    const bool fp32 = x_kind == FPQ_X_FP32;
    if (!fp32) {
        int st = fpq_format_check(f);
        if (st) return st;
    }
    if (workspace_bytes < fpq_count_zeros_workspace_size(n)) return FPQ_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 7) || (reinterpret_cast<uintptr_t>(count_out) & 7) ||
        (fp32 && (reinterpret_cast<uintptr_t>(x) & 3)))
        return FPQ_ERR_ALIGN;
    return launch_count_zeros(x, fp32, n, f.ebits + f.mbits, x_kind == FPQ_X_CODES && is_four_bit(f),
                              reinterpret_cast<unsigned long long*>(count_out),
                              static_cast<unsigned long long*>(workspace), static_cast<hipStream_t>(stream));
}

int fpq_quantize(const float* x, size_t n, fpq_format_t f, float scale, const float* scale_dev, uint8_t* codes,
                 void* stream)
{
    QParams q;
    int st = resolve_format(f, &q);
    if (st) return st;
    if (!scale_dev && !scale_ok(scale)) return FPQ_ERR_SCALE;
    if (n == 0) return FPQ_OK;
    if (!x || !codes) return FPQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(x) & 3) return FPQ_ERR_ALIGN;
    const ScaleSrc ss{scale, scale_dev, nullptr, 0, 0.0f, nullptr};
    return launch_quantize(x, n, q, is_four_bit(f), ss, codes, static_cast<hipStream_t>(stream));
}

int64_t fpq_padded_channels(int64_t C) { return C > 0 ? padded_channels(C) : 0; }

int fpq_quantize_nhwc(const float* x, int64_t B, int64_t C, int64_t H, int64_t W, fpq_format_t f, float scale,
                      const float* scale_dev, uint8_t* codes, void* stream)
{
    QParams q;
    int st = resolve_format(f, &q);
    if (st) return st;
    if (!scale_dev && !scale_ok(scale)) return FPQ_ERR_SCALE;
    if (B <= 0 || C <= 0 || H <= 0 || W <= 0) return FPQ_ERR_SHAPE;
    if (B >= (int64_t)1 << 31 || H * W > (1 << 24) || B * H * W * padded_channels(C) >= (int64_t)1 << 31) return FPQ_ERR_SHAPE;
    if (!x || !codes) return FPQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(x) & 3) || (reinterpret_cast<uintptr_t>(codes) & 15)) return FPQ_ERR_ALIGN;
    const ScaleSrc ss{scale, scale_dev, nullptr, 0, 0.0f, nullptr};
    return launch_quantize_nhwc(x, B, C, H, W, q, ss, codes, static_cast<hipStream_t>(stream));
}

int fpq_dequantize(const uint8_t* codes, size_t n, fpq_format_t f, float scale, float* out, void* stream)
{
    int st = resolve_format(f, nullptr);
    if (st) return st;
    if (!(scale == scale) || isinf(scale)) return FPQ_ERR_SCALE;
    if (n == 0) return FPQ_OK;
    if (!codes || !out) return FPQ_ERR_NULL;
    return launch_dequantize(codes, n, f.ebits, f.mbits, f.bias, scale, out, static_cast<hipStream_t>(stream));
}

size_t fpq_packed_size(int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f)
{
    if (N <= 0 || Cin <= 0 || kh <= 0 || kw <= 0 || resolve_format(f, nullptr)) return 0;
    size_t kpad = (size_t)padded_k(Cin, (int64_t)kh * kw);
    size_t row = is_four_bit(f) ? kpad / 2 : kpad;
    return kPackedRowsOffset + (size_t)N * row;
}

int fpq_pack_weights(const float* w, int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f, const float* scale,
                     const uint8_t* mask, void* packed, size_t packed_bytes, float* scale_out, uint8_t* codes_out,
                     void* stream)
{
    QParams q;
    int st = resolve_format(f, &q);
    if (st) return st;
    if (N <= 0 || Cin <= 0 || kh <= 0 || kw <= 0 || kh > 64 || kw > 64) return FPQ_ERR_SHAPE;
    if (N > 0x7fffffff || Cin * kh * kw > (1 << 28)) return FPQ_ERR_SHAPE;
    if (!w || !packed || !scale_out) return FPQ_ERR_NULL;
    if (packed_bytes < fpq_packed_size(N, Cin, kh, kw, f)) return FPQ_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(packed) & 15) || (reinterpret_cast<uintptr_t>(w) & 3)) return FPQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    PackedHeader h;
    memset(&h, 0, sizeof h);
    h.magic = kPackedMagic;
    h.layout = 1;
    h.ebits = f.ebits;
    h.mbits = f.mbits;
    h.bias = f.bias;
    h.maxval = q.c;
    h.N = N;
    h.Cin = Cin;
    h.kh = kh;
    h.kw = kw;
    h.Cp = (int32_t)padded_channels(Cin);
    h.Kpad = (int32_t)padded_k(Cin, (int64_t)kh * kw);
    hipLaunchKernelGGL(write_header_kernel, dim3(1), dim3(64), 0, s, h, static_cast<uint32_t*>(packed));
    return launch_pack_weights(w, N, Cin, kh * kw, q, is_four_bit(f), scale, mask,
                               static_cast<uint8_t*>(packed) + kPackedRowsOffset, scale_out, codes_out, s);
}

int fpq_packed_check(const void* packed, int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f, void* stream)
{
    QParams q;
    int st = resolve_format(f, &q);
    if (st) return st;
    if (!packed) return FPQ_ERR_NULL;
    PackedHeader h;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(&h, packed, sizeof h, hipMemcpyDeviceToHost, s) != hipSuccess) return FPQ_ERR_LAUNCH;
    if (hipStreamSynchronize(s) != hipSuccess) return FPQ_ERR_LAUNCH;
    if (h.magic != kPackedMagic || h.layout != 1) return FPQ_ERR_PACKED;
    if (h.ebits != f.ebits || h.mbits != f.mbits || h.bias != f.bias || h.maxval != q.c) return FPQ_ERR_PACKED;
    if (h.N != N || h.Cin != Cin || h.kh != kh || h.kw != kw) return FPQ_ERR_PACKED;
    return FPQ_OK;
}

// workspace of the search: [1024 partial maxima][absmax, 256 bytes][per-block error sums]
size_t fpq_search_workspace_size(size_t n, int n_enc, int n_bias)
{
    if (n_enc < 1 || n_enc > kSearchMaxEncodings || n_bias < 1 || n_bias > 128) return 0;
    const int nb = search_blocks(n);
    return 4096 + 256 + align_up((size_t)(nb > 0 ? nb : 1) * (size_t)(n_enc * n_bias) * sizeof(float), 256);
}

int fpq_search_format(const float* x, size_t n, const int32_t* ebits, const int32_t* mbits, int n_enc, int n_bias,
                      float* mse_out, fpq_search_result* result, void* workspace, size_t workspace_bytes, void* stream)
{
    if (n_enc < 1 || n_enc > kSearchMaxEncodings || n_bias < 1 || n_bias > 128) return FPQ_ERR_SHAPE;
    if (!ebits || !mbits || !result || !workspace || (n && !x)) return FPQ_ERR_NULL;
    SearchArgs a;
    memset(&a, 0, sizeof a);
    a.n_enc = n_enc;
    a.J = n_bias;
    for (int i = 0; i < n_enc; ++i) {
        const int e = ebits[i], m = mbits[i];
        if (e < 1 || m < 0 || 1 + e + m > 8) return FPQ_ERR_FORMAT;
        a.enc[i].e = e;
        a.enc[i].m = m;
        a.enc[i].b0 = 1 << (e - 1);
        a.enc[i].c0 = fpq_format_max(e, m, a.enc[i].b0);
    }
    if (workspace_bytes < fpq_search_workspace_size(n, n_enc, n_bias)) return FPQ_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(x) & 3) ||
        (reinterpret_cast<uintptr_t>(result) & 3))
        return FPQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* maxparts = static_cast<float*>(workspace);
    float* absmax = maxparts + 1024;
    float* partial = absmax + 64;
    int st = launch_absmax(x, n, 1.0f, absmax, nullptr, maxparts, s);
    if (st) return st;
    return launch_search(x, n, a, absmax, partial, mse_out, result, s);
}

size_t fpq_gemm_workspace_size(int64_t M, int64_t N, int64_t K, int x_is_fp32)
{
    if (M <= 0 || K <= 0 || N <= 0) return 0;
    size_t codes = x_is_fp32 ? align_up((size_t)M * (size_t)padded_channels(K), 256) : 0;
    return codes + align_up(split_workspace_bytes(plan_gemm(M, N, padded_k(K, 1)), M, N), 256) +
           (x_is_fp32 == FPQ_X_FP32_DYNAMIC ? kDynScaleBytes : 0);
}

size_t fpq_conv2d_workspace_size(int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh, int kw,
                                 int stride, int pad, int x_is_fp32)
{
    if (B <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0) return 0;
    if (H + 2 * pad < kh || W + 2 * pad < kw) return 0;
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    size_t codes = x_is_fp32 ? align_up((size_t)B * H * W * (size_t)padded_channels(Cin), 256) : 0;
    return codes +
           align_up(split_workspace_bytes(plan_gemm(B * Ho * Wo, Cout, padded_k(Cin, (int64_t)kh * kw)), B * Ho * Wo, Cout),
                    256) +
           (x_is_fp32 == FPQ_X_FP32_DYNAMIC ? kDynScaleBytes : 0);
}

static void fill_plan(const GemmPlan& p, int64_t M, bool linear, fpq_plan_t* out)
{
    out->kernel = p.tile == TILE_256x160_S3 ? FPQ_KERNEL_256x160
                  : p.tile == TILE_128x160_S2 ? FPQ_KERNEL_128x160
                  : (linear && M <= 16)       ? FPQ_KERNEL_ROWS16
                                              : FPQ_KERNEL_SMALL_TILE;
    out->k_slices = p.splits;
}

int fpq_gemm_plan(int64_t M, int64_t N, int64_t K, fpq_plan_t* plan)
{
    if (!plan) return FPQ_ERR_NULL;
    if (M <= 0 || K <= 0 || N <= 0) return FPQ_ERR_SHAPE;
    fill_plan(plan_gemm(M, N, padded_k(K, 1)), M, true, plan);
    return FPQ_OK;
}

int fpq_conv2d_plan(int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh, int kw, int stride, int pad,
                    fpq_plan_t* plan)
{
    if (!plan) return FPQ_ERR_NULL;
    if (B <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
        return FPQ_ERR_SHAPE;
    if (H + 2 * pad < kh || W + 2 * pad < kw) return FPQ_ERR_SHAPE;
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    fill_plan(plan_gemm(B * Ho * Wo, Cout, padded_k(Cin, (int64_t)kh * kw)), B * Ho * Wo, false, plan);
    return FPQ_OK;
}

// Where a layer's result goes when it leaves as codes for the next quantized layer.
struct CodesOut {
    fpq_format_t f;
    float s;
    const float* s_dev;
    uint8_t* yq;
};

// Geometry of the structured-sparse packed form: kept-code rows, then (256-byte aligned) the position words.
static size_t sparse_code_row_bytes(int64_t kpad, fpq_format_t f) { return (size_t)(is_four_bit(f) ? kpad / 4 : kpad / 2); }
static size_t sparse_pos_offset(int64_t N, int64_t kpad, fpq_format_t f)
{
    return kPackedRowsOffset + align_up((size_t)N * sparse_code_row_bytes(kpad, f), 256);
}

static int run_layer(const CodesOut* out, const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev,
                     const void* packed_w, fpq_format_t fw, const float* sw, const float* bias, float* y, int64_t B,
                     int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh, int kw, int stride, int pad,
                     int conv_out, int acc_mode, void* workspace, size_t workspace_bytes, void* stream, bool sparse = false)
{
    const int accumulate = (acc_mode & FPQ_OUT_ACCUMULATE) ? 1 : 0;
    const int act = acc_mode & (FPQ_ACT_SILU | FPQ_ACT_GEGLU);
    acc_mode &= ~(FPQ_OUT_ACCUMULATE | FPQ_ACT_SILU | FPQ_ACT_GEGLU);
    if (act && !out) return FPQ_ERR_UNSUPPORTED;                       // activations exist in the codes-out form only
    if (act == (FPQ_ACT_SILU | FPQ_ACT_GEGLU)) return FPQ_ERR_UNSUPPORTED;
    if (act == FPQ_ACT_GEGLU && (conv_out || Cout % 32 != 0)) return FPQ_ERR_UNSUPPORTED;
    QParams qx, qw;
    int st = resolve_format(fx, &qx);
    if (st) return st;
    st = resolve_format(fw, &qw);
    if (st) return st;
    if (x_is_fp32 < 0 || x_is_fp32 > FPQ_X_FP32_DYNAMIC) return FPQ_ERR_UNSUPPORTED;
    const bool dyn = x_is_fp32 == FPQ_X_FP32_DYNAMIC;
    if (!dyn && !sx_dev && !scale_ok(sx)) return FPQ_ERR_SCALE;
    if (B <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
        return FPQ_ERR_SHAPE;
    if (H + 2 * pad < kh || W + 2 * pad < kw || H > 16000 || W > 16000 || kh > 64 || kw > 64 || pad > 64)
        return FPQ_ERR_SHAPE;
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    const int64_t M = B * Ho * Wo;
    const int64_t Cp = padded_channels(Cin);
    if (M >= (int64_t)1 << 31 || B * H * W * Cp >= (int64_t)1 << 31 || M * Cout >= (int64_t)1 << 40 ||
        Cout >= (int64_t)1 << 24 || Cin * kh * kw > (1 << 28))   // the last: what fpq_pack_weights accepts
        return FPQ_ERR_SHAPE;
    if (!x || !packed_w || !sw || (out ? !out->yq : !y)) return FPQ_ERR_NULL;
    QParams qy{0, 0, 0, 0.0f};
    if (out) {
        st = resolve_format(out->f, &qy);
        if (st) return st;
        if (is_four_bit(out->f)) return FPQ_ERR_UNSUPPORTED;   // codes out are the next layer's activations: one per byte
        if (!out->s_dev && !scale_ok(out->s)) return FPQ_ERR_SCALE;
        if (accumulate) return FPQ_ERR_UNSUPPORTED;
        if (reinterpret_cast<uintptr_t>(out->yq) & 15) return FPQ_ERR_ALIGN;
    }
    int xkind, wkind;
    float alpha;
    st = resolve_kinds(fx, qx.c, fw, qw.c, acc_mode, &xkind, &wkind, &alpha);
    if (st) return st;
    if ((reinterpret_cast<uintptr_t>(packed_w) & 15) || (!out && (reinterpret_cast<uintptr_t>(y) & 3))) return FPQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* xcodes;
    // workspace = [activation codes when the input is fp32][split-K partial results]; a caller that passes
    // codes and no (or too small a) workspace gets the unsplit kernel
    GemmPlan plan = plan_gemm(M, Cout, padded_k(Cin, (int64_t)kh * kw));
    if (sparse) {
        // the structured-sparse form has one kernel: hardware E4M3 activations, E4M3 / E2M1 weights, exact accumulate
        if (out || accumulate || acc_mode != FPQ_ACC_FP32 || xkind != OPK_FP8 || (wkind != OPK_FP8 && wkind != OPK_FP4))
            return FPQ_ERR_UNSUPPORTED;
        plan = GemmPlan{TILE_GENERIC, 1};
    }
    const size_t codes_bytes = x_is_fp32 ? align_up((size_t)B * H * W * (size_t)Cp, 256) : 0;
    const size_t part_bytes = align_up(split_workspace_bytes(plan, M, Cout), 256);
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255)) return FPQ_ERR_ALIGN;
    if (x_is_fp32 && (!workspace || workspace_bytes < codes_bytes + part_bytes + (dyn ? kDynScaleBytes : 0)))
        return FPQ_ERR_WORKSPACE;
    if (!x_is_fp32 && (!workspace || workspace_bytes < part_bytes)) plan.splits = 1;
    float* partial = plan.splits > 1 ? reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + codes_bytes) : nullptr;
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.wrows = static_cast<const uint8_t*>(packed_w) + kPackedRowsOffset;
    a.sw = sw;
    a.bias = bias;
    a.sx = sx;
    a.alpha = alpha;
    a.y = y;
    a.M = (int)M;
    a.N = (int)Cout;
    a.Kpad = (int)padded_k(Cin, (int64_t)kh * kw);
    a.Kreal = (int)(Cp * kh * kw);
    a.B = (int)B; a.H = (int)H; a.W = (int)W; a.Cp = (int)Cp;
    a.Ho = (int)Ho; a.Wo = (int)Wo;
    a.kh = kh; a.kw = kw; a.stride = stride; a.pad = pad;
    a.conv_out = conv_out;
    a.xkind = xkind; a.wkind = wkind;
    a.xe = fx.ebits; a.xm = fx.mbits; a.xb = fx.bias;
    a.we = fw.ebits; a.wm = fw.mbits; a.wb = fw.bias;
    a.acc_mode = acc_mode;
    a.accumulate = accumulate;
    if (out) {
        a.yq = out->yq;
        a.act = act;
        a.ldq = (int)(act == FPQ_ACT_GEGLU ? Cout / 2 : padded_channels(Cout));
        a.ym = qy.m; a.yb = qy.b; a.yem = qy.em; a.yc = qy.c;
        a.ykind = (out->f.ebits == 4 && out->f.mbits == 3 && out->f.bias == 7 && qy.c <= 448.0f) ? 1
                  : (out->f.ebits == 5 && out->f.mbits == 2 && out->f.bias == 15 && qy.c <= 57344.0f) ? 2 : 0;
        a.sy = out->s;
        a.sy_dev = out->s_dev;
    }
    a.partial = partial;
    a.splits = plan.splits;
    a.tile = plan.tile;
    a.x_bytes = (uint32_t)(B * H * W * Cp);
    {
        const int64_t wrow = is_four_bit(fw) ? a.Kpad / 2 : a.Kpad;
        if (wrow * Cout >= (int64_t)1 << 31) return FPQ_ERR_SHAPE;
        a.w_bytes = (uint32_t)(wrow * Cout);
    }
    if (x_is_fp32) {
        if (reinterpret_cast<uintptr_t>(x) & 3) return FPQ_ERR_ALIGN;
        uint8_t* buf = static_cast<uint8_t*>(workspace);
        ScaleSrc ss{sx, sx_dev, nullptr, 0, 0.0f, nullptr};
        bool quantized = false;
        if (dyn && !conv_out && Cp == Cin && M <= 16 && !sparse) {
            // at most 16 rows: maximum, scale, codes and the layer itself in one launch
            st = launch_gemm_skinny_dynamic(a, static_cast<const float*>(x), qx, qx.c, buf,
                                            reinterpret_cast<float*>(buf + codes_bytes + part_bytes) + 1024, s);
            if (st != FPQ_ERR_UNSUPPORTED) return st;
        }
        if (dyn && !conv_out && Cp == Cin) {
            // a tensor of a few thousand elements: maximum, scale and codes by one workgroup in one launch
            float* dynbuf = reinterpret_cast<float*>(buf + codes_bytes + part_bytes);
            st = launch_quantize_dynamic_small(static_cast<const float*>(x), (size_t)M * Cin, qx, qx.c, dynbuf + 1024, buf, s);
            if (st == FPQ_OK) {
                quantized = true;
                sx_dev = dynbuf + 1024;
            } else if (st != FPQ_ERR_UNSUPPORTED) {
                return st;
            }
        }
        if (dyn && !quantized) {
            // per-tensor scale = absmax(x) / maxval found here: one reduction launch leaves per-block maxima,
            // the quantize kernel folds them and publishes the scale the layer kernel reads
            float* dynbuf = reinterpret_cast<float*>(buf + codes_bytes + part_bytes);
            const size_t nx = (size_t)B * Cin * H * W;
            st = launch_absmax_partials(static_cast<const float*>(x), nx, dynbuf, s);
            if (st) return st;
            ss.partials = dynbuf;
            ss.nparts = absmax_parts(nx);
            ss.maxval = qx.c;
            ss.publish = dynbuf + 1024;
            sx_dev = dynbuf + 1024;
        }
        if (quantized) {
            st = FPQ_OK;
        } else if (conv_out) {
            st = launch_quantize_nhwc(static_cast<const float*>(x), B, Cin, H, W, qx, ss, buf, s);
        } else if (Cp == Cin) {
            st = launch_quantize(static_cast<const float*>(x), (size_t)M * Cin, qx, false, ss, buf, s);
        } else {
            // rows padded to Cp codes: a linear layer is a 1x1 "image" per row with Cin channels
            st = launch_quantize_nhwc(static_cast<const float*>(x), M, Cin, 1, 1, qx, ss, buf, s);
        }
        if (st) return st;
        xcodes = buf;
    } else {
        if (!conv_out && Cp != Cin) return FPQ_ERR_ALIGN;
        if (reinterpret_cast<uintptr_t>(x) & 15) return FPQ_ERR_ALIGN;
        xcodes = static_cast<const uint8_t*>(x);
    }
    a.x = xcodes;
    a.sx_dev = sx_dev;
    if (sparse)
        return launch_gemm_sparse(a, reinterpret_cast<const uint32_t*>(static_cast<const uint8_t*>(packed_w) +
                                                                       sparse_pos_offset(Cout, a.Kpad, fw)), s);
    if (!gemm_dma_applicable(a)) {   // operand pairing only the generic kernels serve
        a.tile = TILE_GENERIC;
        a.splits = 1;
        a.partial = nullptr;
    }
    return launch_gemm(a, s);
}

int fpq_gemm(const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev, const void* packed_w,
             fpq_format_t fw, const float* sw, const float* bias, float* y, int64_t M, int64_t N, int64_t K,
             int acc_mode, void* workspace, size_t workspace_bytes, void* stream)
{
    if (M == 0 && N > 0 && K > 0) return FPQ_OK;
    return run_layer(nullptr, x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, y, M, K, 1, 1, N, 1, 1, 1, 0, 0, acc_mode,
                     workspace, workspace_bytes, stream);
}

int fpq_conv2d(const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev, const void* packed_w,
               fpq_format_t fw, const float* sw, const float* bias, float* y, int64_t B, int64_t Cin, int64_t H,
               int64_t W, int64_t Cout, int kh, int kw, int stride, int pad, int acc_mode, void* workspace,
               size_t workspace_bytes, void* stream)
{
    return run_layer(nullptr, x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, y, B, Cin, H, W, Cout, kh, kw, stride, pad,
                     1, acc_mode, workspace, workspace_bytes, stream);
}

int fpq_gemm_codes_out(const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev, const void* packed_w,
                       fpq_format_t fw, const float* sw, const float* bias, fpq_format_t fy, float sy, const float* sy_dev,
                       uint8_t* yq, int64_t M, int64_t N, int64_t K, int acc_mode, void* workspace, size_t workspace_bytes,
                       void* stream)
{
    if (M == 0 && N > 0 && K > 0) return FPQ_OK;
    const CodesOut out{fy, sy, sy_dev, yq};
    return run_layer(&out, x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, nullptr, M, K, 1, 1, N, 1, 1, 1, 0, 0,
                     acc_mode, workspace, workspace_bytes, stream);
}

int fpq_conv2d_codes_out(const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev,
                         const void* packed_w, fpq_format_t fw, const float* sw, const float* bias, fpq_format_t fy,
                         float sy, const float* sy_dev, uint8_t* yq, int64_t B, int64_t Cin, int64_t H, int64_t W,
                         int64_t Cout, int kh, int kw, int stride, int pad, int acc_mode, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    const CodesOut out{fy, sy, sy_dev, yq};
    return run_layer(&out, x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, nullptr, B, Cin, H, W, Cout, kh, kw, stride,
                     pad, 1, acc_mode, workspace, workspace_bytes, stream);
}

// Workspace of the grouped dynamic-scale form: per problem its activation codes (256-byte aligned), then per problem a
// 256-byte slot [32 partial maxima][scale, absmax].
static size_t grouped_codes_bytes(const fpq_gemm_problem_t& q) { return align_up((size_t)q.M * (size_t)q.K, 256); }

size_t fpq_gemm_grouped_workspace_size(const fpq_gemm_problem_t* problems, int count, int x_is_fp32)
{
    if (!problems || count <= 0 || x_is_fp32 != FPQ_X_FP32_DYNAMIC) return 0;
    size_t total = 0;
    for (int i = 0; i < count; ++i) {
        if (problems[i].M <= 0 || problems[i].K <= 0) return 0;
        total += grouped_codes_bytes(problems[i]) + 256;
    }
    return total;
}

int fpq_gemm_grouped(const fpq_gemm_problem_t* problems, int count, int x_is_fp32, fpq_format_t fx, fpq_format_t fw,
                     int acc_mode, void* workspace, size_t workspace_bytes, void* stream)
{
    if (count == 0) return FPQ_OK;
    if (!problems) return FPQ_ERR_NULL;
    if (count < 0) return FPQ_ERR_SHAPE;
    QParams qx, qw;
    int st = resolve_format(fx, &qx);
    if (st) return st;
    st = resolve_format(fw, &qw);
    if (st) return st;
    if (x_is_fp32 != FPQ_X_CODES && x_is_fp32 != FPQ_X_FP32_DYNAMIC) return FPQ_ERR_UNSUPPORTED;
    if (acc_mode != FPQ_ACC_FP32 && acc_mode != FPQ_ACC_FP8_MFMA) return FPQ_ERR_UNSUPPORTED;   // no flags in the grouped form
    const bool dyn = x_is_fp32 == FPQ_X_FP32_DYNAMIC;
    int xkind, wkind;
    float alpha;
    st = resolve_kinds(fx, qx.c, fw, qw.c, acc_mode, &xkind, &wkind, &alpha);
    if (st) return st;
    for (int i = 0; i < count; ++i) {
        const fpq_gemm_problem_t& q = problems[i];
        if (q.M <= 0 || q.N <= 0 || q.K <= 0 || q.M >= (int64_t)1 << 31 || q.N >= (int64_t)1 << 24 || q.K > (1 << 28) ||
            q.M * q.K >= (int64_t)1 << 31 || q.M * q.N >= (int64_t)1 << 40)
            return FPQ_ERR_SHAPE;
        if (!q.x || !q.packed_w || !q.sw || !q.y || (!dyn && !q.sx_dev)) return FPQ_ERR_NULL;
        if ((q.K & 15) || (reinterpret_cast<uintptr_t>(q.x) & 15) || (reinterpret_cast<uintptr_t>(q.packed_w) & 15) ||
            (reinterpret_cast<uintptr_t>(q.y) & 3))
            return FPQ_ERR_ALIGN;
        const int64_t kpad = padded_k(q.K, 1);
        if ((is_four_bit(fw) ? kpad / 2 : kpad) * q.N >= (int64_t)1 << 31) return FPQ_ERR_SHAPE;
    }
    if (dyn) {
        if (!workspace || workspace_bytes < fpq_gemm_grouped_workspace_size(problems, count, x_is_fp32)) return FPQ_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255) return FPQ_ERR_ALIGN;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    size_t codes_total = 0;
    for (int i = 0; i < count; ++i) codes_total += grouped_codes_bytes(problems[i]);
    uint8_t* codes_at = static_cast<uint8_t*>(workspace);
    uint8_t* slot_at = codes_at + codes_total;
    for (int first = 0; first < count; first += kGroupMax) {
        GroupedArgs g;
        memset(&g, 0, sizeof g);
        g.count = count - first < kGroupMax ? count - first : kGroupMax;
        GemmArgs& a = g.common;
        a.alpha = alpha;
        a.H = a.W = a.Ho = a.Wo = 1;
        a.kh = a.kw = a.stride = 1;
        a.xkind = xkind; a.wkind = wkind;
        a.xe = fx.ebits; a.xm = fx.mbits; a.xb = fx.bias;
        a.we = fw.ebits; a.wm = fw.mbits; a.wb = fw.bias;
        a.acc_mode = acc_mode;
        a.splits = 1;
        a.tile = TILE_GENERIC;
        for (int i = 0; i < g.count; ++i) {
            const fpq_gemm_problem_t& q = problems[first + i];
            GroupedProblem& d = g.p[i];
            d.wrows = static_cast<const uint8_t*>(q.packed_w) + kPackedRowsOffset;
            d.sw = q.sw;
            d.bias = q.bias;
            d.y = q.y;
            d.M = (int)q.M; d.N = (int)q.N; d.K = (int)q.K; d.Kpad = (int)padded_k(q.K, 1);
            if (dyn) {
                d.x32 = static_cast<const float*>(q.x);
                d.xcodes = codes_at;
                d.partials = reinterpret_cast<float*>(slot_at);
                d.sx_dev = reinterpret_cast<const float*>(slot_at + 128);
                codes_at += grouped_codes_bytes(q);
                slot_at += 256;
            } else {
                d.xcodes = static_cast<const uint8_t*>(q.x);
                d.sx_dev = q.sx_dev;
            }
        }
        if (dyn && skinny_grouped_applicable(g)) {
            // every problem of this chunk has at most 16 rows: maximum, scale, codes and the layer in one launch
            st = launch_gemm_skinny_dynamic_grouped(g, qx, qx.c, s);
        } else {
            if (dyn) {
                st = launch_quantize_dynamic_grouped(g, qx, qx.c, s);
                if (st) return st;
            }
            st = launch_gemm_grouped(g, s);
        }
        if (st) return st;
    }
    return FPQ_OK;
}

size_t fpq_packed_sparse_size(int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f)
{
    if (N <= 0 || Cin <= 0 || kh <= 0 || kw <= 0 || resolve_format(f, nullptr)) return 0;
    const int64_t kpad = padded_k(Cin, (int64_t)kh * kw);
    return sparse_pos_offset(N, kpad, f) + (size_t)N * (size_t)(kpad / 8);
}

int fpq_pack_weights_sparse(const float* w, int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f, const float* scale,
                            const uint8_t* mask, void* packed, size_t packed_bytes, float* scale_out, uint8_t* codes_out,
                            uint64_t* dropped_out, void* stream)
{
    QParams q;
    int st = resolve_format(f, &q);
    if (st) return st;
    if (N <= 0 || Cin <= 0 || kh <= 0 || kw <= 0 || kh > 64 || kw > 64) return FPQ_ERR_SHAPE;
    if (N > 0x7fffffff || Cin * kh * kw > (1 << 28)) return FPQ_ERR_SHAPE;
    if (!w || !packed || !scale_out || !dropped_out) return FPQ_ERR_NULL;
    if (packed_bytes < fpq_packed_sparse_size(N, Cin, kh, kw, f)) return FPQ_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(packed) & 255) || (reinterpret_cast<uintptr_t>(w) & 3) ||
        (reinterpret_cast<uintptr_t>(dropped_out) & 7))
        return FPQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    PackedHeader h;
    memset(&h, 0, sizeof h);
    h.magic = kPackedMagic;
    h.layout = 2;
    h.ebits = f.ebits; h.mbits = f.mbits; h.bias = f.bias;
    h.maxval = q.c;
    h.N = N; h.Cin = Cin; h.kh = kh; h.kw = kw;
    h.Cp = (int32_t)padded_channels(Cin);
    h.Kpad = (int32_t)padded_k(Cin, (int64_t)kh * kw);
    hipLaunchKernelGGL(write_header_kernel, dim3(1), dim3(64), 0, s, h, static_cast<uint32_t*>(packed));
    uint8_t* base = static_cast<uint8_t*>(packed);
    return launch_pack_weights_sparse(w, N, Cin, kh * kw, q, is_four_bit(f), scale, mask, base + kPackedRowsOffset,
                                      reinterpret_cast<uint32_t*>(base + sparse_pos_offset(N, h.Kpad, f)), scale_out, codes_out,
                                      reinterpret_cast<unsigned long long*>(dropped_out), s);
}

int fpq_gemm_sparse(const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev, const void* packed_sparse,
                    fpq_format_t fw, const float* sw, const float* bias, float* y, int64_t M, int64_t N, int64_t K,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    if (M == 0 && N > 0 && K > 0) return FPQ_OK;
    if (packed_sparse && (reinterpret_cast<uintptr_t>(packed_sparse) & 255)) return FPQ_ERR_ALIGN;
    return run_layer(nullptr, x, x_is_fp32, fx, sx, sx_dev, packed_sparse, fw, sw, bias, y, M, K, 1, 1, N, 1, 1, 1, 0, 0,
                     FPQ_ACC_FP32, workspace, workspace_bytes, stream, true);
}

int fpq_conv2d_sparse(const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev, const void* packed_sparse,
                      fpq_format_t fw, const float* sw, const float* bias, float* y, int64_t B, int64_t Cin, int64_t H, int64_t W,
                      int64_t Cout, int kh, int kw, int stride, int pad, void* workspace, size_t workspace_bytes, void* stream)
{
    if (packed_sparse && (reinterpret_cast<uintptr_t>(packed_sparse) & 255)) return FPQ_ERR_ALIGN;
    return run_layer(nullptr, x, x_is_fp32, fx, sx, sx_dev, packed_sparse, fw, sw, bias, y, B, Cin, H, W, Cout, kh, kw, stride, pad,
                     1, FPQ_ACC_FP32, workspace, workspace_bytes, stream, true);
}

// ---- uniform integer baseline (Section IV-A, Eq. (4))

static bool int_bits_ok(int bits) { return bits == 8 || bits == 4; }
static size_t int_rows_bytes(int64_t N, int64_t K, int bits)
{
    const size_t kpad = (size_t)padded_k(K, 1);
    return (size_t)N * (bits == 4 ? kpad / 2 : kpad);
}

size_t fpq_int_calibrate_workspace_size(size_t) { return 2 * 1024 * sizeof(float); }

int fpq_int_calibrate(const float* x, size_t n, int bits, fpq_int_params* params_out, void* workspace, size_t workspace_bytes,
                      void* stream)
{
    if (!int_bits_ok(bits)) return FPQ_ERR_FORMAT;
    if (!params_out || !workspace || (n && !x)) return FPQ_ERR_NULL;
    if (workspace_bytes < fpq_int_calibrate_workspace_size(n)) return FPQ_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(x) & 3) || (reinterpret_cast<uintptr_t>(workspace) & 3) ||
        (reinterpret_cast<uintptr_t>(params_out) & 3))
        return FPQ_ERR_ALIGN;
    return launch_int_params(x, n, bits, params_out, static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
}

int fpq_int_quantize(const float* x, size_t n, int bits, float scale, int32_t zero_point, const fpq_int_params* params_dev,
                     uint8_t* codes, void* stream)
{
    if (!int_bits_ok(bits)) return FPQ_ERR_FORMAT;
    if (!params_dev && !scale_ok(scale)) return FPQ_ERR_SCALE;
    if (!params_dev && (zero_point < -(1 << 24) || zero_point > (1 << 24))) return FPQ_ERR_SCALE;
    if (n == 0) return FPQ_OK;
    if (!x || !codes) return FPQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(x) & 3) return FPQ_ERR_ALIGN;
    return launch_int_quantize(x, n, bits, scale, zero_point, params_dev, codes, static_cast<hipStream_t>(stream));
}

size_t fpq_int_packed_size(int64_t N, int64_t K, int bits)
{
    if (N <= 0 || K <= 0 || !int_bits_ok(bits)) return 0;
    return kPackedRowsOffset + align_up(int_rows_bytes(N, K, bits), 256) + (size_t)N * sizeof(int32_t);
}

int fpq_int_pack_weights(const float* w, int64_t N, int64_t K, int bits, void* packed, size_t packed_bytes, float* scale_out,
                         int32_t* zero_point_out, uint8_t* codes_out, void* stream)
{
    if (!int_bits_ok(bits)) return FPQ_ERR_FORMAT;
    if (N <= 0 || K <= 0 || N > 0x7fffffff || K > 32768) return FPQ_ERR_SHAPE;
    if (!w || !packed || !scale_out || !zero_point_out) return FPQ_ERR_NULL;
    if (packed_bytes < fpq_int_packed_size(N, K, bits)) return FPQ_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(packed) & 255) || (reinterpret_cast<uintptr_t>(w) & 3)) return FPQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    PackedHeader h;
    memset(&h, 0, sizeof h);
    h.magic = kPackedMagic;
    h.layout = 3;                 // integer codes
    h.mbits = bits;
    h.N = N; h.Cin = K; h.kh = h.kw = 1;
    h.Cp = (int32_t)padded_channels(K);
    h.Kpad = (int32_t)padded_k(K, 1);
    hipLaunchKernelGGL(write_header_kernel, dim3(1), dim3(64), 0, s, h, static_cast<uint32_t*>(packed));
    uint8_t* base = static_cast<uint8_t*>(packed);
    int32_t* rowsum = reinterpret_cast<int32_t*>(base + kPackedRowsOffset + align_up(int_rows_bytes(N, K, bits), 256));
    return launch_int_pack_weights(w, N, K, bits, base + kPackedRowsOffset, scale_out, zero_point_out, rowsum, codes_out, s);
}

size_t fpq_int_gemm_workspace_size(int64_t M) { return M > 0 ? align_up((size_t)M * sizeof(int32_t), 256) : 0; }

int fpq_int_gemm(const uint8_t* xcodes, float sx, int32_t zx, const fpq_int_params* px_dev, const void* packed_w, int wbits,
                 const float* sw, const int32_t* zw, const float* bias, float* y, int64_t M, int64_t N, int64_t K,
                 void* workspace, size_t workspace_bytes, void* stream)
{
    if (!int_bits_ok(wbits)) return FPQ_ERR_FORMAT;
    if (M == 0 && N > 0 && K > 0) return FPQ_OK;
    if (M <= 0 || N <= 0 || K <= 0 || M >= (int64_t)1 << 31 || N >= (int64_t)1 << 24 || K > 32768 || M * N >= (int64_t)1 << 40 ||
        M * K >= (int64_t)1 << 40)
        return FPQ_ERR_SHAPE;
    if (!px_dev && !scale_ok(sx)) return FPQ_ERR_SCALE;
    if (!px_dev && (zx < -(1 << 24) || zx > (1 << 24))) return FPQ_ERR_SCALE;
    if (!xcodes || !packed_w || !sw || !zw || !y || !workspace) return FPQ_ERR_NULL;
    if ((K & 15) || (reinterpret_cast<uintptr_t>(xcodes) & 15) || (reinterpret_cast<uintptr_t>(packed_w) & 255) ||
        (reinterpret_cast<uintptr_t>(y) & 3) || (reinterpret_cast<uintptr_t>(workspace) & 3))
        return FPQ_ERR_ALIGN;
    if (workspace_bytes < fpq_int_gemm_workspace_size(M)) return FPQ_ERR_WORKSPACE;
    const uint8_t* base = static_cast<const uint8_t*>(packed_w);
    const int32_t* rowsum = reinterpret_cast<const int32_t*>(base + kPackedRowsOffset + align_up(int_rows_bytes(N, K, wbits), 256));
    return launch_int_gemm(xcodes, sx, zx, px_dev, base + kPackedRowsOffset, rowsum, wbits, sw, zw, bias, y, M, N, K,
                           static_cast<int32_t*>(workspace), static_cast<hipStream_t>(stream));
}

int fpq_probe_peak(int kind, int iterations, const void* src, void* dst, size_t bytes, double* work_out, void* stream)
{
    if (kind < FPQ_PROBE_MFMA_BF16 || kind > FPQ_PROBE_FILL) return FPQ_ERR_UNSUPPORTED;
    if (!dst || !work_out) return FPQ_ERR_NULL;
    const bool memory = kind == FPQ_PROBE_COPY || kind == FPQ_PROBE_FILL;
    if (memory) {
        if (kind == FPQ_PROBE_COPY && !src) return FPQ_ERR_NULL;
        if (bytes < 16 || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15)) return FPQ_ERR_ALIGN;
    } else {
        if (iterations < 1 || iterations > (1 << 20)) return FPQ_ERR_SHAPE;
        if (bytes < (size_t)2048 * 256 * sizeof(float)) return FPQ_ERR_WORKSPACE;
    }
    int grid = 0;
    const int st = launch_probe(kind, iterations, src, dst, bytes, &grid, static_cast<hipStream_t>(stream));
    if (st) return st;
    if (memory)                                                                        // bytes read + written
        *work_out = (kind == FPQ_PROBE_COPY ? 2.0 : 1.0) * (double)(bytes / 16 * 16);
    else if (kind == FPQ_PROBE_MFMA_DECODE_64 || kind == FPQ_PROBE_MFMA_DECODE_32)       // 10 or 5 MFMAs per iteration and wave
        *work_out = (double)grid * 4.0 * iterations * (kind == FPQ_PROBE_MFMA_DECODE_64 ? 10.0 : 5.0) * 2.0 * 32 * 32 * 16;
    else                                                                               // flops: 32 MFMAs per iteration and wave
        *work_out = (double)grid * 4.0 * iterations * 32.0 * 2.0 * 32 * 32 * (kind == FPQ_PROBE_MFMA_BF16 ? 16 : 64);
    return FPQ_OK;
}

int fpq_gemm_noalloc(const void* x, int x_is_fp32, fpq_format_t fx, float sx, const float* sx_dev, const void* packed_w,
                     fpq_format_t fw, const float* sw, const float* bias, float* y, int64_t M, int64_t N, int64_t K,
                     int acc_mode, void* stream)
{
    if (M == 0 && N > 0 && K > 0) return FPQ_OK;
    if (M < 0 || N <= 0 || K <= 0) return FPQ_ERR_SHAPE;
    // the scratch a call of this shape needs is what fpq_gemm would ask of its caller
    if (fpq_gemm_workspace_size(M, N, K, x_is_fp32) > kStaticScratchBytes) return FPQ_ERR_WORKSPACE;
    void* ws = nullptr;
    const int st = scratch_on_current_device(&ws);
    if (st) return st;
    return run_layer(nullptr, x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, y, M, K, 1, 1, N, 1, 1, 1, 0, 0, acc_mode,
                     ws, kStaticScratchBytes, stream);
}

}  // extern "C"
