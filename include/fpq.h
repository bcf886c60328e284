/*
 * fpq.h -- C ABI of libfpq: U-Net conv/linear layers computed on low-bitwidth floating-point
 * (signed ExMy) codes on one AMD MI355X (gfx950).
 *
 * The operations are those of the paper "Low-Bitwidth Floating Point Quantization for Efficient
 * High-Quality Diffusion Models": the tensor quantizer of Section IV-B (Eq. (5)-(9)), the
 * fixed-mask weight quantizer that rounding learning produces (Section V-B, Eq. (12)), and the
 * quantized linear / convolution layer Y = W^q A of Section V-B.
 *
 * Conventions
 *   - A format is (ebits e, mbits m, integer bias b, max value c); 1 + e + m <= 8, e >= 1, m >= 0,
 *     |b| <= 64 and 2^e - b - 1 <= 104 + m (the largest value stays below 2^(106 + m); of the
 *     encodings above only E7M0 below bias 23 and E6M1 below bias -42 are excluded).  maxval == 0 selects the paper's closed form, Eq. (7).  A non-zero maxval must be a
 *     value of the (e, m, b) grid and must not exceed Eq. (7) (hardware E4M3 is (4, 3, 7, 448)).
 *   - A code is sign << (e+m) | p << m | f, one per byte for every format in device buffers that
 *     feed fpq_gemm / fpq_conv2d.  fpq_quantize writes two codes per byte when 1 + e + m <= 4
 *     (element 2j in bits 0-3, element 2j+1 in bits 4-7 of byte j).
 *   - The real-valued per-tensor bias of Section V-A is carried as integer bias + positive fp32
 *     scale: the quantizer is applied to y = fl32(x * fl32(1 / scale)) and a code's value is
 *     decode(code) * scale.
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless it says "host".  The
 *     library keeps no pointer after a call returns and allocates no device memory: scratch space
 *     is the caller's workspace argument.  A scale may be given as a host float, or as a device
 *     float (scale_dev != NULL wins) so that a scale computed by fpq_absmax never visits the host.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue work.
 *   - Every function returns FPQ_OK (0) or a negative fpq_status; arguments are validated on the
 *     host before anything is launched, and nothing throws or aborts.  NaN inputs give
 *     unspecified codes (never a fault).
 */
#ifndef FPQ_H
#define FPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fpq_format {
    int32_t ebits;
    int32_t mbits;
    int32_t bias;
    float maxval; /* 0 => Eq. (7) */
} fpq_format_t;

typedef enum fpq_status {
    FPQ_OK = 0,
    FPQ_ERR_NULL = -1,        /* a required pointer is NULL */
    FPQ_ERR_FORMAT = -2,      /* bad (e, m, b) or maxval not on the grid / above Eq. (7) */
    FPQ_ERR_SCALE = -3,       /* host scale <= 0, NaN or Inf */
    FPQ_ERR_SHAPE = -4,       /* non-positive or inconsistent sizes */
    FPQ_ERR_ALIGN = -5,       /* pointer or leading dimension not aligned as documented */
    FPQ_ERR_WORKSPACE = -6,   /* workspace missing or too small */
    FPQ_ERR_LAUNCH = -7,      /* the HIP runtime reported an error at launch */
    FPQ_ERR_UNSUPPORTED = -8, /* valid arguments the library has no kernel for */
    FPQ_ERR_PACKED = -9       /* fpq_packed_check: the packed weight buffer does not match the arguments */
} fpq_status;

/* Accumulation arithmetic of fpq_gemm / fpq_conv2d.
 * FPQ_ACC_FP32: every product a_k * b_k is formed exactly and summed in fp32 (codes are expanded
 *   to bf16 in registers and fed to the bf16 MFMA).  Meets |y - exact| <= 1e-5 * sum|a_k b_k| + 1e-6.
 * FPQ_ACC_FP8_MFMA: codes go straight into the FP8/FP4 MFMA (only for formats that map onto the
 *   hardware E4M3 / E5M2 / E2M1 encodings).  Twice the peak rate, but the matrix unit aligns each
 *   group of 8 products to the group's largest exponent and drops bits more than 13 binary places
 *   below it, so the error bound is 7 * 2^-13 * sum|a_k b_k| instead. */
typedef enum fpq_acc_mode { FPQ_ACC_FP32 = 0, FPQ_ACC_FP8_MFMA = 1 } fpq_acc_mode;

/* May be OR-ed into the acc_mode argument of fpq_gemm / fpq_conv2d: the layer's result (bias included) is
 * added to what y holds instead of replacing it.  A convolution over a channel-wise concatenation whose
 * parts are quantized separately, each with its own per-tensor scale (Section VI-A: the skip connection
 * and the previous layer's output have different value distributions), is then one call per part on that
 * part's codes and that part's slice of the weights, the second and later calls with this flag. */
#define FPQ_OUT_ACCUMULATE 0x100
#define FPQ_ACT_SILU 0x200  /* codes-out entry points only, see there */
#define FPQ_ACT_GEGLU 0x400

/* What the x argument of fpq_gemm / fpq_conv2d holds (their x_is_fp32 argument).
 * FPQ_X_CODES: codes written by fpq_quantize / fpq_quantize_nhwc with scale sx.
 * FPQ_X_FP32: fp32 activations; the library quantizes them first with the given scale sx / sx_dev.
 * FPQ_X_FP32_DYNAMIC: fp32 activations and no scale: the library finds the per-tensor scale
 *   absmax(x) / maxval itself (what fpq_absmax computes, bit for bit) on the way; sx and sx_dev are
 *   ignored.  One launch fewer than fpq_absmax followed by FPQ_X_FP32.
 * FPQ_X_CODES_BYTE is a value of fpq_count_zeros' x_kind only (codes stored one per byte whatever the format);
 *   the layer calls return FPQ_ERR_UNSUPPORTED for it. */
typedef enum fpq_x_kind { FPQ_X_CODES = 0, FPQ_X_FP32 = 1, FPQ_X_FP32_DYNAMIC = 2, FPQ_X_CODES_BYTE = 3 } fpq_x_kind;

const char *fpq_strerror(int status);

/* ---- host helpers (no GPU needed) ------------------------------------------------------- */

/* Eq. (7): (2 - 2^-m) * 2^(2^e - b - 1); returns 0 for an invalid (e, m, b). */
float fpq_format_max(int ebits, int mbits, int bias);

/* Validates a format (rules above).  FPQ_OK or FPQ_ERR_FORMAT. */
int fpq_format_check(fpq_format_t f);

/* Section V-A: a real-valued bias equals an integer bias plus a power-of-two scale, because the
 * grid of bias b is the grid of bias b0 multiplied by 2^(b0 - b).  Writes int_bias = floor(b)
 * and scale = 2^(floor(b) - b) in (0.5, 1].  Host pointers. */
int fpq_bias_to_scale(int ebits, int mbits, double real_bias, int32_t *int_bias, float *scale);

/* Bytes fpq_quantize writes for n elements: n, or (n + 1) / 2 for formats of at most 4 bits. */
size_t fpq_code_bytes(size_t n, fpq_format_t f);

/* ---- calibration of the clip / scale ---------------------------------------------------- */

/* max_i |x_i| of n fp32 values -> absmax_out[0]; if scale_out != NULL also
 * scale_out[0] = fl32(absmax / maxval) (1 when absmax == 0).  This is the data range from which
 * Section V-A derives c and hence the bias (Eq. (7)).  workspace: fpq_absmax_workspace_size(n)
 * bytes, 4-byte aligned.  n == 0 writes absmax 0 (scale 1). */
size_t fpq_absmax_workspace_size(size_t n);
int fpq_absmax(const float *x, size_t n, float maxval, float *absmax_out, float *scale_out,
               void *workspace, size_t workspace_bytes, void *stream);

/* ---- encoding and bias selection: Section V-A, Algorithm 1 ------------------------------- */

/* Result of fpq_search_format (device memory, 40 bytes).  The chosen candidate is the encoding
 * (ebits, mbits) with max value maxval; its real-valued bias is real_bias (Eq. (7) solved for b).
 * To quantize with it, pass the format (ebits, mbits, int_bias, 0) and the scale to fpq_quantize /
 * fpq_gemm / fpq_conv2d: the grid of the real-valued bias is the grid of int_bias times scale. */
typedef struct fpq_search_result {
    int32_t encoding;   /* index into the encodings passed in */
    int32_t bias_index; /* j of the max-value candidate c_j */
    int32_t ebits, mbits;
    int32_t int_bias;   /* 2^(ebits-1) */
    float maxval;       /* c_j = absmax * (j + 1) / n_bias */
    float scale;        /* c_j / Eq. (7)(ebits, mbits, int_bias) */
    float real_bias;
    float mse;          /* mean squared error of the chosen candidate */
    int32_t reserved;
} fpq_search_result;

/* For each of n_enc encodings (ebits[i], mbits[i]; host arrays, n_enc <= 8) and each of n_bias
 * max-value candidates c_j = absmax(x) * (j + 1) / n_bias (n_bias <= 128; the paper uses 111):
 * the mean over the tensor of (x - dequantize(quantize(x)))^2, written to mse_out[i * n_bias + j]
 * (device, may be NULL); result receives the first candidate with the smallest error in the order
 * of Algorithm 1 (encodings outer, biases inner; the printed initial value prev_mse = 0 is read as
 * +infinity).  An all-zero tensor is searched as if absmax were 1.  One read of x; errors are summed
 * in fp32 within a workgroup (at most 1024 of them share the tensor) and in fp64 across workgroups.  workspace: fpq_search_workspace_size
 * bytes, 256-byte aligned. */
size_t fpq_search_workspace_size(size_t n, int n_enc, int n_bias);
int fpq_search_format(const float *x, size_t n, const int32_t *ebits, const int32_t *mbits, int n_enc,
                      int n_bias, float *mse_out, fpq_search_result *result, void *workspace,
                      size_t workspace_bytes, void *stream);

/* ---- gradient-based rounding learning for low-bitwidth weights (Section V-B, Eq. (10)-(14)) ------
 *
 * A linear layer without bias, as in the paper's exposition: weights w[N, K] fp32, one scale sw[n] per
 * output channel, format f, one learnable parameter alpha[N, K] per weight, calibration activations
 * a[M, K] in full precision.  With y' the clipped weight on the format's axis (fl32(w * fl32(1 / sw)),
 * Eq. (6)), s its step (Eq. (9)) and fl = floor(y' / s):
 *   Wq(alpha) = clamp(s * (fl + sigmoid(alpha)), -c, c) * sw                  (Eq. (12) with the sigmoid)
 *   loss = mean_{M,N}((a Wq^T - a w^T)^2) + reg_weight * mean_{N,K}(1 - (2 |sigmoid(alpha) - 0.5|)^20)
 * fpq_rl_step performs one step of gradient descent, alpha -= lr * d loss / d alpha (the outer clamp passes
 * no gradient where it is active), and writes loss_out[0] = the mean squared output error and loss_out[1]
 * = the mean regulariser of the alpha that came in (device memory, two floats); grad_out[N, K], if not
 * NULL, receives the gradient used.  fpq_rl_init_alpha sets sigmoid(alpha) to each weight's fractional
 * position between its two grid neighbours (kept inside [1e-3, 1 - 1e-3]), so that learning starts from
 * the unquantized weights.  fpq_rl_mask writes the decision used at inference, 1 where
 * sigmoid(alpha) >= 0.5: the mask that fpq_pack_weights takes.  All products are fp32 on the fp32
 * matrix instruction.  workspace: fpq_rl_workspace_size bytes, 256-byte aligned, no initialisation.
 * Size limits (FPQ_ERR_SHAPE beyond them): N K < 2^31, M N < 2^31, M < 2^23; lr and reg_weight finite and
 * >= 0 (FPQ_ERR_SCALE otherwise). */
/* A convolution takes part as the linear layer on its patch matrix (Section V-B presents the method on a linear
 * layer and notes that it carries over to other layer types, convolutions among them): fpq_rl_im2col writes, for x NCHW [B, C, H, W] fp32, the matrix
 * a[B * Ho * Wo, C * kh * kw] whose row (b, ho, wo) is the receptive field of that output pixel in the
 * order of the flattened weight [Cout, (ci, kh, kw)], zero where it reaches into the padding; w[N, K] is
 * then the weight tensor as it stands, K = C * kh * kw, and the learned mask has the weight's shape. */
int fpq_rl_im2col(const float *x, int64_t B, int64_t C, int64_t H, int64_t W, int kh, int kw, int stride,
                  int pad, float *a, void *stream);
size_t fpq_rl_workspace_size(int64_t M, int64_t N, int64_t K);
int fpq_rl_init_alpha(const float *w, const float *sw, int64_t N, int64_t K, fpq_format_t f, float *alpha,
                      void *stream);
int fpq_rl_step(const float *w, const float *sw, int64_t N, int64_t K, fpq_format_t f, float *alpha,
                const float *a, int64_t M, float lr, float reg_weight, float *loss_out, float *grad_out,
                void *workspace, size_t workspace_bytes, void *stream);
int fpq_rl_mask(const float *alpha, size_t n, uint8_t *mask, void *stream);

/* ---- sparsity (Section VI, "Sparsity"): how many values of a tensor are zero ---------------- */

/* Counts the zeros among the n elements of x and writes the count to count_out (one 64-bit unsigned
 * integer in device memory).  x_kind says what x holds:
 *   FPQ_X_CODES       codes of format f as fpq_quantize writes them (one per byte; two per byte for
 *                     formats of at most 4 bits, and then the high nibble of the last byte is not
 *                     counted when n is odd); a code is zero when its exponent and mantissa fields
 *                     are, whatever its sign bit;
 *   FPQ_X_CODES_BYTE  codes of format f, one per byte whatever the format (codes_out of
 *                     fpq_pack_weights);
 *   FPQ_X_FP32        fp32 values (+0 and -0 count; f is ignored), for the full-precision tensor the
 *                     quantized one is compared with.
 * x needs no alignment beyond that of its element type.  workspace: fpq_count_zeros_workspace_size
 * bytes, 8-byte aligned; n == 0 writes 0. */
size_t fpq_count_zeros_workspace_size(size_t n);
int fpq_count_zeros(const void *x, int x_kind, size_t n, fpq_format_t f, uint64_t *count_out,
                    void *workspace, size_t workspace_bytes, void *stream);

/* ---- activation quantizer: Eq. (6) clip, Eq. (9) step, Eq. (8) round-to-nearest(-even), clip - */

/* x[n] fp32 -> codes, same element order.  n == 0 is a no-op. */
int fpq_quantize(const float *x, size_t n, fpq_format_t f, float scale, const float *scale_dev,
                 uint8_t *codes, void *stream);

/* Same quantizer for a convolution input: x is NCHW [B, C, H, W] fp32, codes are written
 * channels-last as [B, H, W, Cp] with Cp = fpq_padded_channels(C) (C rounded up to 16); the
 * padding channels hold code 0.  Only 8-bit-class storage (one code per byte). */
int64_t fpq_padded_channels(int64_t C);
int fpq_quantize_nhwc(const float *x, int64_t B, int64_t C, int64_t H, int64_t W, fpq_format_t f,
                      float scale, const float *scale_dev, uint8_t *codes, void *stream);

/* codes (one per byte) -> fp32 values decode(code) * scale.  For tests and inspection. */
int fpq_dequantize(const uint8_t *codes, size_t n, fpq_format_t f, float scale, float *out,
                   void *stream);

/* ---- weight pre-quantization and packing (offline step) -------------------------------- */

/* Weights w[N, Cin, kh, kw] fp32 (a linear layer is kh = kw = 1, Cin = K).  Per output channel n:
 * scale[n] (given, or fl32(absmax_n / maxval), 1 for an all-zero row), then each element is
 * quantized with Eq. (12) and its mask entry h (0 = floor, non-zero = floor + 1 step), or with
 * Eq. (8) when mask == NULL (the paper applies no rounding learning to FP8 weights).
 * packed receives fpq_packed_size(...) bytes: a header (256 bytes, 64 used), then the codes in the
 * layout the GEMM kernels stream (K ordered (kh, kw, ci), ci padded to 16, K padded to 128; 4-bit
 * formats two per byte).  packed must be 16-byte aligned; 256-byte alignment is what the kernels
 * are tuned for (every 128-byte piece of a row is then one cache line).  scale_out[N] receives
 * the scales used.  codes_out, if not NULL, receives the plain codes [N, Cin, kh, kw], one per
 * byte, for inspection. */
size_t fpq_packed_size(int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f);
int fpq_pack_weights(const float *w, int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f,
                     const float *scale, const uint8_t *mask, void *packed, size_t packed_bytes,
                     float *scale_out, uint8_t *codes_out, void *stream);

/* Reads the header of a packed weight buffer back (synchronises `stream`; the only entry point that
 * waits for the device) and compares it with the arguments a layer call is about to pass: FPQ_OK, or
 * FPQ_ERR_PACKED (not a packed buffer, another format or max value, or other N, Cin, kh, kw).  The
 * layer calls themselves are asynchronous and do not check the header (reading it back would make every
 * layer call wait for the device): passing them a buffer packed for another shape or format is the
 * caller's error, which this call lets the caller rule out once per buffer. */
int fpq_packed_check(const void *packed, int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f,
                     void *stream);

/* ---- quantized layers: Y = sx * sw[n] * sum_k deq(xq) * deq(wq) (+ bias[n]) ------------- */

/* Linear layer.  x: x_is_fp32 == 0: codes [M, K], one per byte, K % 16 == 0, 16-byte aligned;
 *                   x_is_fp32 == 1: fp32 [M, K], quantized by the library first (any K) into the
 *                   workspace with scale sx / sx_dev;
 *                   x_is_fp32 == 2: the same with the scale absmax(x) / maxval found by the library.
 * packed_w from fpq_pack_weights(N, K, 1, 1, fw).  sw[N], bias[N] (or NULL) fp32.
 * y[M, N] fp32 row-major.  workspace: fpq_gemm_workspace_size bytes, 256-byte aligned (may be
 * NULL when that size is 0).  It holds the activation codes of the x_is_fp32 == 1 form and, for
 * shapes with few output tiles and a deep K, the partial sums of the K slices that a second
 * kernel adds up.  With x_is_fp32 == 0 a missing or smaller workspace is not an error: the layer
 * then runs unsliced (same result up to summation order, slower for those shapes).  With
 * x_is_fp32 == 1 a workspace below the stated size returns FPQ_ERR_WORKSPACE.  The contents need
 * no initialisation and mean nothing after the call; calls that share a workspace must be
 * ordered on one stream. */
size_t fpq_gemm_workspace_size(int64_t M, int64_t N, int64_t K, int x_is_fp32);
int fpq_gemm(const void *x, int x_is_fp32, fpq_format_t fx, float sx, const float *sx_dev,
             const void *packed_w, fpq_format_t fw, const float *sw, const float *bias, float *y,
             int64_t M, int64_t N, int64_t K, int acc_mode, void *workspace, size_t workspace_bytes,
             void *stream);

/* 2-D convolution, zero padding, square stride, as an implicit GEMM with M = B*Ho*Wo,
 * K = Cin*kh*kw, N = Cout.  x: x_is_fp32 == 0: codes [B, H, W, Cp] from fpq_quantize_nhwc;
 * x_is_fp32 == 1 or 2 (fpq_x_kind): fp32 NCHW [B, Cin, H, W], quantized by the library first into
 * the workspace.
 * y: fp32 NCHW [B, Cout, Ho, Wo], Ho = (H + 2 pad - kh) / stride + 1.
 * Size limits of both layer calls (FPQ_ERR_SHAPE beyond them): M = B Ho Wo < 2^31, B H W Cp < 2^31 (Cp = Cin
 * rounded up to 16), M Cout < 2^40, Cout < 2^24, Cin kh kw <= 2^28, kh, kw, pad <= 64, H, W <= 16000. */
size_t fpq_conv2d_workspace_size(int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh,
                                 int kw, int stride, int pad, int x_is_fp32);
int fpq_conv2d(const void *x, int x_is_fp32, fpq_format_t fx, float sx, const float *sx_dev,
               const void *packed_w, fpq_format_t fw, const float *sw, const float *bias, float *y,
               int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh, int kw, int stride,
               int pad, int acc_mode, void *workspace, size_t workspace_bytes, void *stream);

/* Read-only query (host, no GPU): which kernel fpq_gemm / fpq_conv2d launch for a shape and into how many K slices
 * they cut it, given a workspace of the size the *_workspace_size functions state and operands in the hardware's
 * E4M3 / E2M1 encodings (other operand pairings may take FPQ_KERNEL_SMALL_TILE, unsliced, whatever the shape).
 * With more than one slice the layer kernel writes partial sums to the workspace and a reduction kernel adds them.
 * For tests and benchmarks that have to state, or to cover, every launch configuration a workload uses. */
typedef enum fpq_kernel {
    FPQ_KERNEL_SMALL_TILE = 0, /* register-staged 128 x 128 / 64 x 64 tiles: any shape */
    FPQ_KERNEL_256x160 = 1,    /* persistent 256 x 160 tiles, three LDS stages */
    FPQ_KERNEL_128x160 = 2,    /* persistent 128 x 160 tiles, two LDS stages, two workgroups per compute unit */
    FPQ_KERNEL_ROWS16 = 3      /* linear layers with at most 16 rows: K split over the wavefronts of a workgroup */
} fpq_kernel;
typedef struct fpq_plan {
    int32_t kernel;   /* fpq_kernel */
    int32_t k_slices; /* >= 1 */
} fpq_plan_t;
int fpq_gemm_plan(int64_t M, int64_t N, int64_t K, fpq_plan_t *plan);
int fpq_conv2d_plan(int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh, int kw, int stride,
                    int pad, fpq_plan_t *plan);

/* ---- the same layers with the result handed to the next quantized layer as codes -------------
 *
 * Section V applies the activation quantizer to the input of every convolution and linear layer, so when
 * one such layer feeds another, the fp32 result exists only to be quantized again.  These entry points
 * quantize it in the layer kernel's epilogue instead: yq[m, n] = Q(v; fy, sy) with v the fp32 value
 * fpq_gemm / fpq_conv2d would have written (sx * sw[n] * sum + bias[n]), Q the activation quantizer of
 * Eq. (6)-(9) (as fpq_quantize), fy a format stored one code per byte, and sy (or *sy_dev when not
 * NULL) the next layer's static per-tensor scale.  One byte per output is written instead of four.
 *
 * yq: codes, row-major [M, Np] with Np = fpq_padded_channels(N); columns N .. Np - 1 receive code 0;
 * 16-byte aligned.  For a convolution the rows are the output pixels in (b, ho, wo) order, i.e. the
 * channels-last buffer [B, Ho, Wo, Np] that fpq_conv2d takes as codes; for a linear layer with
 * N % 16 == 0 it is the [M, K = N] code matrix that fpq_gemm takes.  All other arguments, the workspace
 * and its size are those of fpq_gemm / fpq_conv2d; FPQ_OUT_ACCUMULATE is not accepted.
 *
 * An activation can stand between the result and its codes (the U-Net has one between the two linear
 * layers of every feed-forward block), OR-ed into acc_mode:
 *   FPQ_ACT_SILU   yq = Q(v * sigmoid(v));
 *   FPQ_ACT_GEGLU  (fpq_gemm_codes_out only, N % 32 == 0) the columns of v come in blocks of 32, the
 *                  first 16 of a block values a, the last 16 gates g of the same 16 outputs:
 *                  yq[m, 16 B + i] = Q(v[m, 32 B + i] * gelu(v[m, 32 B + 16 + i])) with
 *                  gelu(g) = g * Phi(g) (the exact, erf-based form); yq is [M, N / 2].  A caller
 *                  whose projection holds all values before all gates reorders the weight rows,
 *                  scales and biases once, before fpq_pack_weights.
 * The activation is evaluated in fp32: sigmoid to a relative error below 1e-6, gelu(g) to an absolute
 * error below 4e-7 |g| (erf by a five-term rational approximation).  Because v
 * depends on the summation order within the fp32 tolerance, a code can differ from the one computed
 * from an exactly rounded v where v lies within that tolerance of a rounding boundary of fy. */
int fpq_gemm_codes_out(const void *x, int x_is_fp32, fpq_format_t fx, float sx, const float *sx_dev,
                       const void *packed_w, fpq_format_t fw, const float *sw, const float *bias,
                       fpq_format_t fy, float sy, const float *sy_dev, uint8_t *yq, int64_t M, int64_t N,
                       int64_t K, int acc_mode, void *workspace, size_t workspace_bytes, void *stream);
int fpq_conv2d_codes_out(const void *x, int x_is_fp32, fpq_format_t fx, float sx, const float *sx_dev,
                         const void *packed_w, fpq_format_t fw, const float *sw, const float *bias,
                         fpq_format_t fy, float sy, const float *sy_dev, uint8_t *yq, int64_t B,
                         int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh, int kw, int stride,
                         int pad, int acc_mode, void *workspace, size_t workspace_bytes, void *stream);

/* ---- structured-sparse weight operand (Section VI, "Sparsity") ----------------------------------
 *
 * Quantization to few bits turns many weights into zero (the paper measures up to 617 times more zeros in FP4 than in
 * full precision) and names the use of that sparsity as the next step.  These entry points store and multiply the
 * weight operand in the 2-of-4 form that the matrix unit's sparse instructions take: of every four consecutive input
 * channels (per output channel and kernel tap; a channel count that is not a multiple of four is completed with zeros)
 * the two codes of largest magnitude are kept (equal magnitudes: the lower channel), the other two are dropped.  A
 * group with at most two non-zero codes loses nothing, so a weight tensor whose groups are all like that gives
 * exactly the dense layer; *dropped_out counts the groups that lost a non-zero code.
 *
 * fpq_pack_weights_sparse: arguments as fpq_pack_weights (same per-channel scales, same Eq. (12) / Eq. (8) codes);
 *   packed receives fpq_packed_sparse_size bytes, 256-byte aligned (header; kept codes, half the bytes of the dense
 *   form; one 2-bit position per kept code); codes_out, if not NULL, the pruned codes [N, Cin, kh, kw] one per byte
 *   (dropped entries are code 0); dropped_out one 64-bit count in device memory.
 * fpq_gemm_sparse / fpq_conv2d_sparse: as fpq_gemm / fpq_conv2d with FPQ_ACC_FP32 on such a buffer: every kept
 *   product is formed exactly and summed in fp32, so the result is the dense layer on the pruned codes within
 *   1e-5 * sum|a_k b_k| + 1e-6.  Activations in the hardware's E4M3 encoding ((4, 3, b) with max value up to
 *   448 * 2^(7 - b)), weights E4M3 or E2M1; other formats return FPQ_ERR_UNSUPPORTED.  workspace: the size the dense
 *   call states for the same x_is_fp32 (only the activation codes and the dynamic-scale slot are used). */
size_t fpq_packed_sparse_size(int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f);
int fpq_pack_weights_sparse(const float *w, int64_t N, int64_t Cin, int kh, int kw, fpq_format_t f,
                            const float *scale, const uint8_t *mask, void *packed, size_t packed_bytes,
                            float *scale_out, uint8_t *codes_out, uint64_t *dropped_out, void *stream);
int fpq_gemm_sparse(const void *x, int x_is_fp32, fpq_format_t fx, float sx, const float *sx_dev,
                    const void *packed_sparse, fpq_format_t fw, const float *sw, const float *bias, float *y,
                    int64_t M, int64_t N, int64_t K, void *workspace, size_t workspace_bytes, void *stream);
int fpq_conv2d_sparse(const void *x, int x_is_fp32, fpq_format_t fx, float sx, const float *sx_dev,
                      const void *packed_sparse, fpq_format_t fw, const float *sw, const float *bias, float *y,
                      int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int kh, int kw, int stride,
                      int pad, void *workspace, size_t workspace_bytes, void *stream);

/* ---- the same-bitwidth integer baseline (Section IV-A, Eq. (4)) ------------------------------------
 *
 * The uniform integer quantizer the paper measures its floating-point formats against,
 *     X_int = s (clamp(round(X / s) + z; 0, 2^b - 1) - z),   s = (max X - min X) / (2^b - 1),   z = -round(min X / s),
 * and a linear layer on its codes, Y[m, n] = sx sw[n] sum_k (qx[m, k] - zx)(qw[n, k] - zw[n]) (+ bias[n]), computed
 * with the 8-bit integer matrix instruction: the sum is exact (32-bit integers), the scaling is one fp32 multiply.
 * bits is 8 or 4 (FPQ_ERR_FORMAT otherwise).  Codes are one per byte (0 .. 2^b - 1) in all caller-visible buffers.
 * Rounding is to nearest, ties to the even integer; in fp32: s = fl32(fl32(max - min) / (2^b - 1)) (1 for a constant
 * tensor), every quotient is fl32(x * fl32(1 / s)), z is not clamped to the code range.  NaN inputs give code 0.
 *
 * fpq_int_calibrate: min, max, s and z of x[n] into *params_out (device memory); workspace
 *   fpq_int_calibrate_workspace_size bytes.
 * fpq_int_quantize: codes of x with (scale, zero_point), or with *params_dev when that is not NULL.
 * fpq_int_pack_weights: w[N, K] fp32 -> per-output-channel (s, z) by the same equation, codes in the layout the layer
 *   kernel streams (fpq_int_packed_size bytes, 256-byte aligned) with each row's code sum; scale_out[N],
 *   zero_point_out[N]; codes_out (or NULL) the plain codes [N, K].  K <= 32768.
 * fpq_int_gemm: xcodes [M, K] 8-bit activation codes (K % 16 == 0, 16-byte aligned) with (sx, zx) or *px_dev;
 *   packed_w / wbits / sw / zw from fpq_int_pack_weights; y[M, N] fp32; workspace fpq_int_gemm_workspace_size(M)
 *   bytes (the row sums of the activation codes). */
typedef struct fpq_int_params {
    float scale;
    int32_t zero_point;
    float min, max;
} fpq_int_params;
size_t fpq_int_calibrate_workspace_size(size_t n);
int fpq_int_calibrate(const float *x, size_t n, int bits, fpq_int_params *params_out, void *workspace,
                      size_t workspace_bytes, void *stream);
int fpq_int_quantize(const float *x, size_t n, int bits, float scale, int32_t zero_point,
                     const fpq_int_params *params_dev, uint8_t *codes, void *stream);
size_t fpq_int_packed_size(int64_t N, int64_t K, int bits);
int fpq_int_pack_weights(const float *w, int64_t N, int64_t K, int bits, void *packed, size_t packed_bytes,
                         float *scale_out, int32_t *zero_point_out, uint8_t *codes_out, void *stream);
size_t fpq_int_gemm_workspace_size(int64_t M);
int fpq_int_gemm(const uint8_t *xcodes, float sx, int32_t zx, const fpq_int_params *px_dev, const void *packed_w,
                 int wbits, const float *sw, const int32_t *zw, const float *bias, float *y, int64_t M, int64_t N,
                 int64_t K, void *workspace, size_t workspace_bytes, void *stream);

/* ---- a group of independent linear layers in one call -----------------------------------------
 *
 * Several linear layers that do not depend on each other (in the U-Net: the key / value projections of all
 * cross-attention blocks, which all read the text context, and the time-embedding projections of all residual
 * blocks) as one call with a handful of launches for the whole group instead of up to three per layer; for layers
 * this small the launches are what a call costs.  problems is a HOST array of count entries (any count; the
 * pointers inside are device pointers); it is read during the call only and travels to the device as a kernel
 * argument, so the call can be captured into a graph.  All problems share the formats fx, fw and acc_mode
 * (FPQ_ACC_FP32 or FPQ_ACC_FP8_MFMA, no flags).  x_is_fp32:
 *   FPQ_X_FP32_DYNAMIC  x is fp32 [M, K]; every problem gets its own per-tensor scale absmax(x) / maxval, its codes
 *                       and its [scale, absmax] are left in the workspace (fpq_gemm_grouped_workspace_size bytes,
 *                       256-byte aligned, no initialisation: first the codes of every problem, each rounded up to
 *                       256 bytes, then one 256-byte slot per problem with [scale, absmax] at byte 128);
 *   FPQ_X_CODES         x holds codes [M, K] with the scale sx_dev[0]; no workspace.
 * Every K must be a multiple of 16 and every x 16-byte aligned (FPQ_ERR_ALIGN).  Each y[M, N] receives exactly what
 * fpq_gemm computes for that problem with the register-staged kernel (bit for bit for shapes that fpq_gemm itself
 * gives to that kernel; the same sums in another order otherwise).  Meant for small problems: every problem runs on
 * 64 x 64 tiles (or, when all problems of a chunk of 32 have at most 16 rows, on the one-launch kernel for such layers). */
typedef struct fpq_gemm_problem {
    const void *x;
    const float *sx_dev;  /* FPQ_X_CODES only */
    const void *packed_w; /* from fpq_pack_weights(N, K, 1, 1, fw) */
    const float *sw;      /* [N] */
    const float *bias;    /* [N] or NULL */
    float *y;             /* [M, N] */
    int64_t M, N, K;
} fpq_gemm_problem_t;
size_t fpq_gemm_grouped_workspace_size(const fpq_gemm_problem_t *problems, int count, int x_is_fp32);
int fpq_gemm_grouped(const fpq_gemm_problem_t *problems, int count, int x_is_fp32, fpq_format_t fx,
                     fpq_format_t fw, int acc_mode, void *workspace, size_t workspace_bytes, void *stream);

/* ---- machine-ceiling probes (for the benchmark's roofline object) -------------------------------
 *
 * What this GPU sustains with nothing but the instruction in question in the loop, to set beside the published peaks
 * that roofline fractions are quoted against.  kind:
 *   FPQ_PROBE_MFMA_BF16  register-only loop of the bf16 matrix instruction of the fp32-accumulate mode, operands
 *                        that change with every instruction; dst receives 2048 * 256 floats (bytes = size of dst);
 *   FPQ_PROBE_MFMA_FP8   the same with the 8-bit matrix instruction of FPQ_ACC_FP8_MFMA;
 *   FPQ_PROBE_COPY       dst[0 .. bytes) = src[0 .. bytes), 16-byte aligned;
 *   FPQ_PROBE_MFMA_DECODE_64 / _32
 *                        the bf16 matrix instruction together with the code-to-bf16 conversions that the
 *                        fp32-accumulate mode pays per k-step of a wave tile of 64 x 160 / 32 x 160 outputs (the two
 *                        large-tile layer kernels), codes in registers: the ceiling of that instruction mix; dst as
 *                        for FPQ_PROBE_MFMA_BF16;
 *   FPQ_PROBE_FILL       dst[0 .. bytes) = a constant pattern, 16-byte aligned; src is not used.
 * One launch on stream; work_out (host) receives the flops (MFMA kinds) or the bytes read plus written (copy, fill) of
 * that launch, for the caller to divide by the time it measures. */
typedef enum fpq_probe_kind {
    FPQ_PROBE_MFMA_BF16 = 0, FPQ_PROBE_MFMA_FP8 = 1, FPQ_PROBE_COPY = 2, FPQ_PROBE_MFMA_DECODE_64 = 3, FPQ_PROBE_MFMA_DECODE_32 = 4,
    FPQ_PROBE_FILL = 5
} fpq_probe_kind;
int fpq_probe_peak(int kind, int iterations, const void *src, void *dst, size_t bytes, double *work_out,
                   void *stream);

/* ---- fpq_gemm for callers that cannot allocate device memory ----------------------------------
 *
 * For callers that cannot call hipMalloc or hand over a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation.  Same arguments, result and kernels as fpq_gemm, without the
 * workspace: the scratch memory (activation codes of the fp32 forms, partial sums of the K slices, partial
 * maxima and scale of the dynamic-scale form) lives in a static device array of FPQ_NOALLOC_SCRATCH_BYTES inside
 * the library, of which every GPU the library runs on holds its own copy until the process ends.  The call
 * allocates nothing and frees nothing.  The first call on a device looks the array's address up (make it outside
 * a graph capture).  A shape whose fpq_gemm_workspace_size exceeds FPQ_NOALLOC_SCRATCH_BYTES returns
 * FPQ_ERR_WORKSPACE and launches nothing.  All calls on one GPU share that GPU's array: nothing in it has to
 * start at zero and every call overwrites what it uses, but two calls that overlap in time on one GPU (different
 * streams, or different host threads on unordered streams) race; order them on one stream. */
#define FPQ_NOALLOC_SCRATCH_BYTES ((size_t)64 << 20)
int fpq_gemm_noalloc(const void *x, int x_is_fp32, fpq_format_t fx, float sx, const float *sx_dev,
                     const void *packed_w, fpq_format_t fw, const float *sw, const float *bias, float *y,
                     int64_t M, int64_t N, int64_t K, int acc_mode, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FPQ_H */
