/*
 * fpq_oracle.c -- CPU oracle for low-bitwidth floating-point (ExMy) quantized layers.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision statement of
 * what the quantized hot path computes, written from the paper's equations.  It shares no
 * code with the GPU library and must never be linked into, or called from, the product
 * path; only the tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Notation follows the paper (Section IV-B "Floating Point Quantization" and Section V-B
 * "Gradient-Based Rounding Learning"):
 *   e, m   exponent / mantissa bit counts of a signed ExMy format (1 + e + m <= 8)
 *   b      integer exponent bias
 *   c      largest representable magnitude; the paper's closed form is Eq. (7)
 *   s_i    per-element step of Eq. (9)
 *   h      per-weight rounding decision (0 = down, 1 = up), the thresholded sigma(alpha)
 *          of Eq. (12)
 *
 * Readings taken where the paper is silent or garbled (each also listed in the design
 * notes of the repository):
 *   - exponent field p runs over 0 .. 2^e - 1 (the text's upper limit 2^e is one too many
 *     for e bits and contradicts Eq. (7));
 *   - p = 0 holds zero and the subnormals f * 2^(1-b-m), the flat-step branch of Eq. (9);
 *   - every code is a finite value (Eq. (7): the all-ones code is the maximum), but a
 *     caller may pass a smaller c that lies on the grid (hardware E4M3 tops out at 448);
 *   - round-to-nearest breaks ties towards the even integer multiple of s_i;
 *   - the real-valued bias of Section V-A is an integer bias plus a positive fp32 scale:
 *     y = fl32(x * fl32(1/scale)) is formed first, in fp32, then Eq. (6)-(9) are applied
 *     to y exactly;
 *   - Eq. (12) prints the quantized weight inside its own floor; it is read as the
 *     clipped full-precision weight (as in AdaRound, which the section adapts), the floor
 *     is towards minus infinity, and s_i is taken from the clipped, unrounded weight;
 *   - a value that rounds to zero keeps the sign bit of the input;
 *   - NaN inputs are outside the contract (result unspecified);
 *   - Algorithm 1 (Section V-A) starts from prev_mse = 0 and keeps a candidate only when
 *     prev_mse > curr_mse, which as printed never accepts anything: read as prev_mse =
 *     +infinity (first strict minimum in scan order, encodings outer, biases inner);
 *   - its bias candidates come from equally spaced points of the data's range, each turned
 *     into a bias by Eq. (7): read on magnitudes (the grid is symmetric) as
 *     the max values c_j = absmax * (j + 1) / J, j = 0 .. J-1; the real-valued bias of c_j
 *     is carried as the integer bias b0 = 2^(e-1) plus the scale c_j / c0, c0 = Eq. (7) at
 *     b0 (the grid of a real bias is a scaled copy of the grid of an integer one);
 *   - the error of a candidate is the mean over the tensor of (x - dequantized x)^2.
 *
 * Codes are held one per byte everywhere in this file (also for 4-bit formats);
 * oracle_pack4 produces the two-per-byte boundary form (even index in the low nibble).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC (see build.py).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ format */

/* Eq. (7): c = (2 - 2^-m) * 2^(2^e - b - 1). */
double oracle_format_max(int e, int m, int b)
{
    return (2.0 - ldexp(1.0, -m)) * ldexp(1.0, (1 << e) - b - 1);
}

/* Eq. (5) with p in 0..2^e-1, plus the p = 0 row (zero and subnormals). */
double oracle_decode(int e, int m, int b, unsigned code)
{
    unsigned f = code & ((1u << m) - 1u);
    unsigned p = (code >> m) & ((1u << e) - 1u);
    unsigned sgn = (code >> (e + m)) & 1u;
    double mag;
    if (p == 0)
        mag = ldexp((double)f, 1 - b - m);
    else
        mag = ldexp(1.0 + (double)f / (double)(1u << m), (int)p - b);
    return sgn ? -mag : mag;
}

/* Code of a magnitude q that lies on the grid (sign bit not included).
 * Returns 0xFFFF if q is not representable (never happens for q produced below). */
static unsigned encode_magnitude(int e, int m, int b, double q)
{
    double lowest_normal = ldexp(1.0, 1 - b);
    unsigned p, f;
    if (q < lowest_normal) {
        double fq = ldexp(q, -(1 - b - m));
        f = (unsigned)fq;
        if ((double)f != fq || f >= (1u << m)) return 0xFFFFu;
        p = 0;
    } else {
        int ex;
        double frac = frexp(q, &ex);          /* q = frac * 2^ex, frac in [0.5,1) */
        int E = ex - 1;                       /* q = (2 frac) * 2^E, 2 frac in [1,2) */
        double fq = ldexp(2.0 * frac - 1.0, m);
        int pe = E + b;
        f = (unsigned)fq;
        if ((double)f != fq || pe < 1 || pe > (1 << e) - 1) return 0xFFFFu;
        p = (unsigned)pe;
    }
    return (p << m) | f;
}

/* Step of Eq. (9) for a clipped magnitude a >= 0: the binade of a is taken exactly. */
static double step_of(int m, int b, double a)
{
    int P = 1;
    if (a > 0.0) {
        int ex;
        (void)frexp(a, &ex);                  /* floor(log2 a) = ex - 1 */
        P = (ex - 1) + b;
        if (P < 1) P = 1;
    }
    return ldexp(1.0, P - b - m);
}

/* fp32 pre-scaling: y = fl32(x * fl32(1/scale)).  volatile keeps each rounding. */
static double prescale(float x, float scale)
{
    volatile float r = 1.0f / scale;
    volatile float y = x * r;
    return (double)y;
}

/* ------------------------------------------------- Eq. (6), (8), (9): nearest */

unsigned oracle_quantize_one(float x, int e, int m, int b, double c, float scale)
{
    double y = prescale(x, scale);
    unsigned sgn = signbit(x) ? 1u : 0u;
    double a = fabs(y);
    if (a > c) a = c;                          /* Eq. (6) */
    double s = step_of(m, b, a);               /* Eq. (9) */
    double n = nearbyint(a / s);               /* ties to even; a/s is exact */
    double q = n * s;
    if (q > c) q = c;                          /* Eq. (8), outer clamp */
    return (sgn << (e + m)) | encode_magnitude(e, m, b, q);
}

void oracle_quantize(const float *x, size_t n, int e, int m, int b, double c, float scale,
                     uint8_t *codes)
{
    for (size_t i = 0; i < n; ++i)
        codes[i] = (uint8_t)oracle_quantize_one(x[i], e, m, b, c, scale);
}

/* --------------------------------------------- Eq. (12): floor + fixed mask h */

unsigned oracle_quantize_mask_one(float w, unsigned h, int e, int m, int b, double c, float scale)
{
    double y = prescale(w, scale);
    if (y > c) y = c;                          /* Eq. (6) */
    if (y < -c) y = -c;
    double s = step_of(m, b, fabs(y));         /* Eq. (9) on the clipped, unrounded weight */
    double n = floor(y / s) + (h ? 1.0 : 0.0); /* Eq. (12) */
    double q = n * s;
    if (q > c) q = c;
    if (q < -c) q = -c;
    unsigned sgn = (q < 0.0 || (q == 0.0 && signbit(w))) ? 1u : 0u;
    return (sgn << (e + m)) | encode_magnitude(e, m, b, fabs(q));
}

void oracle_quantize_mask(const float *w, const uint8_t *h, size_t n, int e, int m, int b,
                          double c, float scale, uint8_t *codes)
{
    for (size_t i = 0; i < n; ++i)
        codes[i] = (uint8_t)oracle_quantize_mask_one(w[i], h[i], e, m, b, c, scale);
}

/* ------------------------------------------------------- scales, absmax, pack */

float oracle_absmax(const float *x, size_t n)
{
    float a = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float v = fabsf(x[i]);
        if (v > a) a = v;
    }
    return a;
}

/* scale = fl32(absmax / c), or 1 when the tensor is all zero. */
float oracle_scale_from_absmax(float absmax, double c)
{
    volatile float s = absmax / (float)c;
    return (absmax == 0.0f) ? 1.0f : s;
}

/* Weights [N,K]: one scale per output channel (row), then Eq. (8) (h == NULL) or
 * Eq. (12) (h given) on every element with its row's scale. */
void oracle_pack_weights(const float *w, const uint8_t *h, long N, long K, int e, int m, int b,
                         double c, const float *scale_in, float *scale_out, uint8_t *codes)
{
    for (long n = 0; n < N; ++n) {
        const float *row = w + (size_t)n * (size_t)K;
        float s = scale_in ? scale_in[n]
                           : oracle_scale_from_absmax(oracle_absmax(row, (size_t)K), c);
        scale_out[n] = s;
        if (h)
            oracle_quantize_mask(row, h + (size_t)n * (size_t)K, (size_t)K, e, m, b, c, s,
                                 codes + (size_t)n * (size_t)K);
        else
            oracle_quantize(row, (size_t)K, e, m, b, c, s, codes + (size_t)n * (size_t)K);
    }
}

/* Two 4-bit codes per byte, element 2j in bits 0-3 and 2j+1 in bits 4-7 of byte j. */
void oracle_pack4(const uint8_t *codes, size_t n, uint8_t *packed)
{
    for (size_t j = 0; j < (n + 1) / 2; ++j) {
        unsigned lo = codes[2 * j] & 0xFu;
        unsigned hi = (2 * j + 1 < n) ? (codes[2 * j + 1] & 0xFu) : 0u;
        packed[j] = (uint8_t)(lo | (hi << 4));
    }
}

void oracle_dequantize(const uint8_t *codes, size_t n, int e, int m, int b, double scale,
                       double *out)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = oracle_decode(e, m, b, codes[i]) * scale;
}

/* ---------------------------------------------- quantized linear layer Y = W^q A
 * Y[r,n] = sx * sw[n] * sum_k deq(xq[r,k]) * deq(wq[n,k]) (+ bias[n]); double accumulator,
 * index order.  T[r,n] = sx * sw[n] * sum_k |deq(xq) * deq(wq)| is the tolerance scale.
 * rows == NULL: all M rows, Y and T are [M,N]; otherwise only the listed rows, [nrows,N]. */
void oracle_gemm(const uint8_t *xq, int ex, int mx, int bx, float sx,
                 const uint8_t *wq, int ew, int mw, int bw, const float *sw, const float *bias,
                 long M, long N, long K, const long *rows, long nrows, double *Y, double *T)
{
    double lx[256], lw[256];
    for (unsigned cde = 0; cde < 256; ++cde) {
        lx[cde] = oracle_decode(ex, mx, bx, cde & ((1u << (1 + ex + mx)) - 1u));
        lw[cde] = oracle_decode(ew, mw, bw, cde & ((1u << (1 + ew + mw)) - 1u));
    }
    long R = rows ? nrows : M;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < R; ++i) {
        long r = rows ? rows[i] : i;
        const uint8_t *xr = xq + (size_t)r * (size_t)K;
        for (long n = 0; n < N; ++n) {
            const uint8_t *wr = wq + (size_t)n * (size_t)K;
            double acc = 0.0, accabs = 0.0;
            for (long k = 0; k < K; ++k) {
                double p = lx[xr[k]] * lw[wr[k]];
                acc += p;
                accabs += fabs(p);
            }
            double sc = (double)sx * (double)sw[n];
            Y[(size_t)i * (size_t)N + (size_t)n] = sc * acc + (bias ? (double)bias[n] : 0.0);
            T[(size_t)i * (size_t)N + (size_t)n] = sc * accabs;
        }
    }
}

/* ---------------------------------------------- quantized conv2d, zero padding
 * x codes NCHW [B,Cin,H,W]; w codes [Cout,Cin,kh,kw]; output NCHW [B,Cout,Ho,Wo] with
 * Ho = (H + 2 pad - kh)/stride + 1 (same for Wo).  A padded position contributes zero.
 * pix == NULL: every output pixel, Y/T are full NCHW tensors; otherwise pix lists npix
 * flattened (b*Ho + ho)*Wo + wo positions and Y/T are [npix, Cout]. */
void oracle_conv2d(const uint8_t *xq, int ex, int mx, int bx, float sx,
                   const uint8_t *wq, int ew, int mw, int bw, const float *sw, const float *bias,
                   long B, long Cin, long H, long W, long Cout, long kh, long kw, long stride,
                   long pad, const long *pix, long npix, double *Y, double *T)
{
    double lx[256], lw[256];
    for (unsigned cde = 0; cde < 256; ++cde) {
        lx[cde] = oracle_decode(ex, mx, bx, cde & ((1u << (1 + ex + mx)) - 1u));
        lw[cde] = oracle_decode(ew, mw, bw, cde & ((1u << (1 + ew + mw)) - 1u));
    }
    long Ho = (H + 2 * pad - kh) / stride + 1;
    long Wo = (W + 2 * pad - kw) / stride + 1;
    long P = pix ? npix : B * Ho * Wo;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < P; ++i) {
        long flat = pix ? pix[i] : i;
        long wo = flat % Wo, ho = (flat / Wo) % Ho, bb = flat / (Wo * Ho);
        for (long co = 0; co < Cout; ++co) {
            double acc = 0.0, accabs = 0.0;
            for (long ci = 0; ci < Cin; ++ci)
                for (long r = 0; r < kh; ++r)
                    for (long t = 0; t < kw; ++t) {
                        long hi = ho * stride - pad + r, wi = wo * stride - pad + t;
                        if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                        double xv = lx[xq[(((size_t)bb * Cin + ci) * H + hi) * W + wi]];
                        double wv = lw[wq[(((size_t)co * Cin + ci) * kh + r) * kw + t]];
                        double p = xv * wv;
                        acc += p;
                        accabs += fabs(p);
                    }
            double sc = (double)sx * (double)sw[co];
            double yv = sc * acc + (bias ? (double)bias[co] : 0.0);
            size_t o = pix ? (size_t)i * (size_t)Cout + (size_t)co
                           : (((size_t)bb * Cout + co) * Ho + ho) * Wo + wo;
            Y[o] = yv;
            T[o] = sc * accabs;
        }
    }
}

/* ----------------------------- Section V-A, Algorithm 1: encoding and bias search */

/* Max-value candidate j of J for a tensor whose largest magnitude is absmax (1 if the
 * tensor is all zero): evenly spaced in (0, absmax], the last one equal to absmax. */
float oracle_search_candidate(float absmax, int j, int J)
{
    double a = absmax > 0.0f ? (double)absmax : 1.0;
    return (float)(a * (double)(j + 1) / (double)J);
}

/* Integer bias + scale form of "encoding (e, m) with max value cj": b0 = 2^(e-1),
 * scale = fl32(cj / c0) with c0 = Eq. (7) at b0. */
float oracle_search_scale(int e, int m, float cj)
{
    int b0 = 1 << (e - 1);
    return (float)((double)cj / oracle_format_max(e, m, b0));
}

/* Mean squared error between x and its quantized-dequantized copy for one candidate. */
double oracle_candidate_mse(const float *x, size_t n, int e, int m, float cj)
{
    int b0 = 1 << (e - 1);
    double c0 = oracle_format_max(e, m, b0);
    float scale = oracle_search_scale(e, m, cj);
    double sum = 0.0;
    for (size_t i = 0; i < n; ++i) {
        unsigned code = oracle_quantize_one(x[i], e, m, b0, c0, scale);
        double q = oracle_decode(e, m, b0, code) * (double)scale;
        double d = (double)x[i] - q;
        sum += d * d;
    }
    return n ? sum / (double)n : 0.0;
}

/* Algorithm 1 over n_enc encodings x J bias candidates.  mse[i * J + j] receives every
 * candidate's error; best[0], best[1] the chosen encoding and bias index. */
void oracle_search(const float *x, size_t n, const int *enc_e, const int *enc_m, int n_enc, int J,
                   double *mse, int *best)
{
    float absmax = oracle_absmax(x, n);
    int total = n_enc * J;
#pragma omp parallel for schedule(dynamic)
    for (int cnd = 0; cnd < total; ++cnd) {
        int i = cnd / J, j = cnd % J;
        mse[cnd] = oracle_candidate_mse(x, n, enc_e[i], enc_m[i], oracle_search_candidate(absmax, j, J));
    }
    double prev_mse = INFINITY;
    best[0] = best[1] = 0;
    for (int i = 0; i < n_enc; ++i)
        for (int j = 0; j < J; ++j)
            if (prev_mse > mse[i * J + j]) {
                best[0] = i;
                best[1] = j;
                prev_mse = mse[i * J + j];
            }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
