"""ctypes binding of the CPU oracle (oracle/fpq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing on the product path may import this package, and this package
imports nothing from the GPU library.

A format is a tuple (e, m, b, c): exponent bits, mantissa bits, integer bias, maximum
magnitude (Section IV-B, Eq. (5)-(7)).  Codes are numpy uint8, one code per element.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.oracle_format_max.restype = C.c_double
        L.oracle_format_max.argtypes = [C.c_int] * 3
        L.oracle_decode.restype = C.c_double
        L.oracle_decode.argtypes = [C.c_int, C.c_int, C.c_int, C.c_uint]
        L.oracle_quantize_one.restype = C.c_uint
        L.oracle_quantize_one.argtypes = [C.c_float, C.c_int, C.c_int, C.c_int, C.c_double, C.c_float]
        L.oracle_quantize_mask_one.restype = C.c_uint
        L.oracle_quantize_mask_one.argtypes = [C.c_float, C.c_uint, C.c_int, C.c_int, C.c_int,
                                               C.c_double, C.c_float]
        L.oracle_quantize.restype = None
        L.oracle_quantize.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_double,
                                      C.c_float, C.c_void_p]
        L.oracle_quantize_mask.restype = None
        L.oracle_quantize_mask.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int,
                                           C.c_int, C.c_double, C.c_float, C.c_void_p]
        L.oracle_absmax.restype = C.c_float
        L.oracle_absmax.argtypes = [C.c_void_p, C.c_size_t]
        L.oracle_scale_from_absmax.restype = C.c_float
        L.oracle_scale_from_absmax.argtypes = [C.c_float, C.c_double]
        L.oracle_pack_weights.restype = None
        L.oracle_pack_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_long, C.c_long, C.c_int, C.c_int,
                                          C.c_int, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_pack4.restype = None
        L.oracle_pack4.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
        L.oracle_dequantize.restype = None
        L.oracle_dequantize.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_double,
                                        C.c_void_p]
        L.oracle_gemm.restype = None
        L.oracle_gemm.argtypes = ([C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                   C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                   C.c_long, C.c_long, C.c_long, C.c_void_p, C.c_long,
                                   C.c_void_p, C.c_void_p])
        L.oracle_conv2d.restype = None
        L.oracle_conv2d.argtypes = ([C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                     C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
                                    + [C.c_long] * 9 + [C.c_void_p, C.c_long, C.c_void_p, C.c_void_p])
        L.oracle_num_threads.restype = C.c_int
        L.oracle_num_threads.argtypes = []
        L.oracle_search_candidate.restype = C.c_float
        L.oracle_search_candidate.argtypes = [C.c_float, C.c_int, C.c_int]
        L.oracle_search_scale.restype = C.c_float
        L.oracle_search_scale.argtypes = [C.c_int, C.c_int, C.c_float]
        L.oracle_candidate_mse.restype = C.c_double
        L.oracle_candidate_mse.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_float]
        L.oracle_search.restype = None
        L.oracle_search.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                    C.c_void_p]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def format_max(e, m, b):
    """Eq. (7)."""
    return lib().oracle_format_max(e, m, b)


def decode(fmt, code):
    e, m, b, _ = fmt
    return lib().oracle_decode(e, m, b, int(code))


def grid(fmt):
    """All non-negative magnitudes of the format, indexed by code (sign bit clear)."""
    e, m, b, _ = fmt
    return np.array([lib().oracle_decode(e, m, b, k) for k in range(1 << (e + m))])


def quantize_one(x, fmt, scale=1.0):
    e, m, b, c = fmt
    return lib().oracle_quantize_one(float(np.float32(x)), e, m, b, float(c), float(np.float32(scale)))


def quantize_mask_one(w, h, fmt, scale=1.0):
    e, m, b, c = fmt
    return lib().oracle_quantize_mask_one(float(np.float32(w)), int(h), e, m, b, float(c),
                                          float(np.float32(scale)))


def quantize(x, fmt, scale=1.0):
    """Eq. (6), (8), (9): nearest-value codes of x / scale, same shape as x."""
    e, m, b, c = fmt
    x = _f32(x)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().oracle_quantize(_p(x), x.size, e, m, b, float(c), float(np.float32(scale)), _p(out))
    return out


def quantize_mask(w, h, fmt, scale=1.0):
    """Eq. (12) with a fixed 0/1 mask h."""
    e, m, b, c = fmt
    w = _f32(w)
    h = _u8(h)
    assert h.shape == w.shape
    out = np.empty(w.shape, dtype=np.uint8)
    lib().oracle_quantize_mask(_p(w), _p(h), w.size, e, m, b, float(c), float(np.float32(scale)), _p(out))
    return out


def absmax(x):
    x = _f32(x)
    return float(lib().oracle_absmax(_p(x), x.size))


def scale_from_absmax(a, c):
    return float(lib().oracle_scale_from_absmax(float(np.float32(a)), float(c)))


def pack_weights(w, fmt, h=None, scale=None):
    """Per-output-channel weight quantization of w[N, ...]; returns (codes, scale[N])."""
    e, m, b, c = fmt
    w = _f32(w)
    N = w.shape[0]
    K = w.size // N
    hh = None if h is None else _u8(h)
    sc_in = None if scale is None else _f32(scale)
    sc_out = np.empty(N, dtype=np.float32)
    codes = np.empty(w.shape, dtype=np.uint8)
    lib().oracle_pack_weights(_p(w), _p(hh), N, K, e, m, b, float(c), _p(sc_in), _p(sc_out), _p(codes))
    return codes, sc_out


def pack4(codes):
    codes = _u8(codes).reshape(-1)
    out = np.empty((codes.size + 1) // 2, dtype=np.uint8)
    lib().oracle_pack4(_p(codes), codes.size, _p(out))
    return out


def dequantize(codes, fmt, scale=1.0):
    e, m, b, _ = fmt
    codes = _u8(codes)
    out = np.empty(codes.shape, dtype=np.float64)
    lib().oracle_dequantize(_p(codes), codes.size, e, m, b, float(scale), _p(out))
    return out


def gemm(xq, fx, sx, wq, fw, sw, bias=None, rows=None):
    """Quantized linear layer on codes: returns (Y, T) as float64 [M or len(rows), N]."""
    xq = _u8(xq)
    wq = _u8(wq)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    sw = _f32(sw)
    assert sw.shape == (N,)
    bias_ = None if bias is None else _f32(bias)
    rows_ = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    R = M if rows_ is None else rows_.size
    Y = np.empty((R, N), dtype=np.float64)
    T = np.empty((R, N), dtype=np.float64)
    lib().oracle_gemm(_p(xq), fx[0], fx[1], fx[2], float(np.float32(sx)),
                      _p(wq), fw[0], fw[1], fw[2], _p(sw), _p(bias_),
                      M, N, K, _p(rows_), R, _p(Y), _p(T))
    return Y, T


def conv2d(xq, fx, sx, wq, fw, sw, bias=None, stride=1, pad=0, pix=None):
    """Quantized conv2d on NCHW codes; returns (Y, T) NCHW float64, or [len(pix), Cout]."""
    xq = _u8(xq)
    wq = _u8(wq)
    B, Cin, H, W = xq.shape
    Cout, Cin2, kh, kw = wq.shape
    assert Cin == Cin2
    sw = _f32(sw)
    bias_ = None if bias is None else _f32(bias)
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    pix_ = None if pix is None else np.ascontiguousarray(pix, dtype=np.int64)
    shape = (B, Cout, Ho, Wo) if pix_ is None else (pix_.size, Cout)
    Y = np.empty(shape, dtype=np.float64)
    T = np.empty(shape, dtype=np.float64)
    lib().oracle_conv2d(_p(xq), fx[0], fx[1], fx[2], float(np.float32(sx)),
                        _p(wq), fw[0], fw[1], fw[2], _p(sw), _p(bias_),
                        B, Cin, H, W, Cout, kh, kw, stride, pad,
                        _p(pix_), 0 if pix_ is None else pix_.size, _p(Y), _p(T))
    return Y, T


def silu(v):
    """v * sigmoid(v) in double."""
    v = np.asarray(v, dtype=np.float64)
    return v / (1.0 + np.exp(-v))


def gelu(g):
    """g * Phi(g), Phi the standard normal distribution function (the exact, erf-based form), in double."""
    from scipy.special import erfc
    g = np.asarray(g, dtype=np.float64)
    return 0.5 * g * erfc(-g / np.sqrt(2.0))


def geglu(V):
    """Gated GELU on a layer result whose columns come in blocks of 32, the first 16 of a block values, the last 16
    the gates of the same outputs: [M, N] -> [M, N / 2]."""
    V = np.asarray(V, dtype=np.float64)
    M, N = V.shape
    blocks = V.reshape(M, N // 32, 2, 16)
    return (blocks[:, :, 0, :] * gelu(blocks[:, :, 1, :])).reshape(M, N // 2)


def geglu_plain(V):
    """Gated GELU as a feed-forward block defines it: the projection's result holds all values in the first half of
    its columns and all gates in the second half: [M, N] -> [M, N / 2], out[:, i] = V[:, i] * gelu(V[:, N / 2 + i])."""
    V = np.asarray(V, dtype=np.float64)
    half = V.shape[1] // 2
    return V[:, :half] * gelu(V[:, half:])


def geglu_interleaved_rows(N):
    """The one-time reordering of a projection's N output channels (weight rows, scales, biases) from the plain
    layout of geglu_plain to the blocked layout of geglu: entry r of the result is the plain index that moves to
    position r.  Position 32 B + i (i < 16) takes value channel 16 B + i, position 32 B + 16 + i its gate N / 2 + 16 B + i."""
    half = N // 2
    order = np.empty(N, dtype=np.int64)
    for r in range(N):
        blk, i = divmod(r, 32)
        order[r] = 16 * blk + i if i < 16 else half + 16 * blk + (i - 16)
    return order


def requantize(Y, fmt, scale):
    """A layer's result as the next quantized layer's input codes (Section V: every convolution / linear input is
    quantized): the fp32 value of each output through the activation quantizer of Eq. (6)-(9)."""
    return quantize(np.asarray(Y, dtype=np.float64).astype(np.float32), fmt, scale)


def requantize_bounds(Y, T, fmt, scale, rel, abs_):
    """Codes of the lowest and highest fp32 values within the layer tolerance rel * T + abs_ of Y: the quantizer is
    monotone, so a result inside the tolerance has a code whose value lies between theirs."""
    Y = np.asarray(Y, dtype=np.float64)
    tol = rel * np.asarray(T, dtype=np.float64) + abs_
    lo = np.nextafter((Y - tol).astype(np.float32), np.float32(-np.inf))
    hi = np.nextafter((Y + tol).astype(np.float32), np.float32(np.inf))
    return quantize(lo, fmt, scale), quantize(hi, fmt, scale)


def prune_2of4(codes, fmt):
    """Structured sparsity for the weight operand (Section VI, "Sparsity", and the future work of Section VIII: use the
    zeros that quantization produces).  codes: weight codes [N, Cin] or [N, Cin, kh, kw].  The input channels of every
    output channel and kernel tap are taken in groups of four consecutive ones (the last group of a channel count that
    is not a multiple of four is completed with zeros); in each group the two codes of largest magnitude are kept, the
    other two become code 0.  Equal magnitudes: the lower channel index wins.  A group that has at most two non-zero
    codes to begin with, which is what quantization to few bits makes common, is unchanged.
    Returns (pruned codes, same shape; number of groups that lost a non-zero value)."""
    e, m, b, _ = fmt
    codes = _u8(codes)
    shape = codes.shape
    c4 = codes.reshape(shape[0], shape[1], -1)                      # [N, Cin, taps]
    N, Cin, taps = c4.shape
    mag = np.array([decode(fmt, k) for k in range(1 << (e + m))])   # magnitude of every code without its sign bit
    out = c4.copy()
    altered = 0
    for n in range(N):
        for t in range(taps):
            for c0 in range(0, Cin, 4):
                grp = list(range(c0, min(c0 + 4, Cin)))
                mags = [mag[int(c4[n, c, t]) & ((1 << (e + m)) - 1)] for c in grp]
                order = sorted(range(len(grp)), key=lambda i: (-mags[i], i))   # largest first, lower index first among equals
                keep = set(order[:2])
                lost = False
                for i, c in enumerate(grp):
                    if i not in keep:
                        lost = lost or mags[i] != 0.0
                        out[n, c, t] = 0
                altered += int(lost)
    return out.reshape(shape), altered


def prune_2of4_fast(codes, fmt):
    """The same rule vectorised with numpy (stable sort on the negated magnitudes), for tensors the loop above is too
    slow for; the tests check it against the loop."""
    e, m, b, _ = fmt
    codes = _u8(codes)
    shape = codes.shape
    c4 = codes.reshape(shape[0], shape[1], -1)
    N, Cin, taps = c4.shape
    pad = (-Cin) % 4
    g = np.concatenate([c4, np.zeros((N, pad, taps), dtype=np.uint8)], axis=1) if pad else c4
    g = g.transpose(0, 2, 1).reshape(N, taps, -1, 4)                # [N, taps, groups, 4]
    mag = np.array([decode(fmt, k) for k in range(1 << (e + m))])[g & ((1 << (e + m)) - 1)]
    order = np.argsort(-mag, axis=-1, kind="stable")                # largest first; equal magnitudes keep index order
    drop = order[..., 2:]
    pruned = g.copy()
    np.put_along_axis(pruned, drop, 0, axis=-1)
    altered = int((np.take_along_axis(mag, drop, axis=-1) != 0).any(axis=-1).sum())
    pruned = pruned.reshape(N, taps, -1).transpose(0, 2, 1)[:, :Cin, :]
    return np.ascontiguousarray(pruned).reshape(shape), altered


def count_zeros(values):
    """Section VI, "Sparsity": the number of values of a tensor that are zero (+0 and -0 alike)."""
    return int(np.count_nonzero(np.asarray(values) == 0))


def count_zero_codes(codes, fmt):
    """The same on codes (one per byte): every code is decoded (Eq. (5)) and its value compared with zero."""
    return count_zeros(dequantize(codes, fmt))


def sparsity(values):
    """Fraction of the values that are zero."""
    v = np.asarray(values)
    return count_zeros(v) / v.size


def search_candidate(absmax, j, J):
    """Section V-A: max-value candidate j of J, evenly spaced in (0, absmax]."""
    return float(lib().oracle_search_candidate(float(absmax), int(j), int(J)))


def search_scale(e, m, cj):
    """Scale that, with the integer bias 2^(e-1), realises encoding (e, m) with max value cj."""
    return float(lib().oracle_search_scale(int(e), int(m), float(cj)))


def candidate_mse(x, e, m, cj):
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    return float(lib().oracle_candidate_mse(_p(x), x.size, int(e), int(m), float(cj)))


def search(x, encodings, J=111):
    """Algorithm 1 (Section V-A) over encodings [(e, m), ...] x J bias candidates.
    Returns (mse[n_enc, J] float64, (best encoding index, best bias index))."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    ee = np.ascontiguousarray([e for e, _ in encodings], dtype=np.int32)
    mm = np.ascontiguousarray([m for _, m in encodings], dtype=np.int32)
    mse = np.empty(len(encodings) * J, dtype=np.float64)
    best = np.zeros(2, dtype=np.int32)
    lib().oracle_search(_p(x), x.size, _p(ee), _p(mm), len(encodings), int(J), _p(mse), _p(best))
    return mse.reshape(len(encodings), J), (int(best[0]), int(best[1]))


def num_threads():
    return lib().oracle_num_threads()
