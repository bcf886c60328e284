"""Thin ctypes binding of libfpq.so: same names as the C ABI (include/fpq.h), argument marshalling only.

Tensors are torch tensors on the GPU (PyTorch supplies device memory and streams, nothing else);
every function below forwards their data pointers to the C entry point of the same name on the
current torch stream and raises FpqError on a non-zero status.  There is no CPU fallback: if the
shared library is missing or does not load, importing the functions' library handle fails.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FPQ_LIB_PATH") or os.path.join(HERE, "libfpq.so")   # FPQ_LIB_PATH: a library built elsewhere

FPQ_ACC_FP32 = 0
FPQ_ACC_FP8_MFMA = 1
FPQ_OUT_ACCUMULATE = 0x100
FPQ_ACT_SILU = 0x200
FPQ_ACT_GEGLU = 0x400
FPQ_X_CODES = 0
FPQ_X_FP32 = 1
FPQ_X_FP32_DYNAMIC = 2
FPQ_X_CODES_BYTE = 3


class fpq_format_t(C.Structure):
    _fields_ = [("ebits", C.c_int32), ("mbits", C.c_int32), ("bias", C.c_int32), ("maxval", C.c_float)]


class fpq_plan_t(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("k_slices", C.c_int32)]


FPQ_KERNEL_SMALL_TILE, FPQ_KERNEL_256x160, FPQ_KERNEL_128x160, FPQ_KERNEL_ROWS16 = 0, 1, 2, 3
FPQ_NOALLOC_SCRATCH_BYTES = 64 << 20


class fpq_gemm_problem_t(C.Structure):
    _fields_ = [("x", C.c_void_p), ("sx_dev", C.c_void_p), ("packed_w", C.c_void_p), ("sw", C.c_void_p),
                ("bias", C.c_void_p), ("y", C.c_void_p), ("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64)]


class FpqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().fpq_strerror(status).decode()
        super().__init__("%s: status %d (%s)" % (where, status, msg))


_lib = None


def lib():
    """Load libfpq.so (built by paper_2408_06995_amd.build); loud failure if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libfpq.so not built: run `python -m paper_2408_06995_amd.build` (%s)" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, f32p, u8p, sz, i64, i32, fl = C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int64, C.c_int, C.c_float
    F = fpq_format_t
    L.fpq_strerror.restype = C.c_char_p
    L.fpq_strerror.argtypes = [i32]
    L.fpq_format_max.restype = fl
    L.fpq_format_max.argtypes = [i32, i32, i32]
    L.fpq_format_check.restype = i32
    L.fpq_format_check.argtypes = [F]
    L.fpq_bias_to_scale.restype = i32
    L.fpq_bias_to_scale.argtypes = [i32, i32, C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_float)]
    L.fpq_code_bytes.restype = sz
    L.fpq_code_bytes.argtypes = [sz, F]
    L.fpq_absmax_workspace_size.restype = sz
    L.fpq_absmax_workspace_size.argtypes = [sz]
    L.fpq_absmax.restype = i32
    L.fpq_absmax.argtypes = [f32p, sz, fl, f32p, f32p, vp, sz, vp]
    L.fpq_quantize.restype = i32
    L.fpq_quantize.argtypes = [f32p, sz, F, fl, f32p, u8p, vp]
    L.fpq_padded_channels.restype = i64
    L.fpq_padded_channels.argtypes = [i64]
    L.fpq_quantize_nhwc.restype = i32
    L.fpq_quantize_nhwc.argtypes = [f32p, i64, i64, i64, i64, F, fl, f32p, u8p, vp]
    L.fpq_dequantize.restype = i32
    L.fpq_dequantize.argtypes = [u8p, sz, F, fl, f32p, vp]
    L.fpq_packed_size.restype = sz
    L.fpq_packed_size.argtypes = [i64, i64, i32, i32, F]
    L.fpq_pack_weights.restype = i32
    L.fpq_pack_weights.argtypes = [f32p, i64, i64, i32, i32, F, f32p, u8p, vp, sz, f32p, u8p, vp]
    L.fpq_packed_check.restype = i32
    L.fpq_packed_check.argtypes = [vp, i64, i64, i32, i32, F, vp]
    L.fpq_gemm_workspace_size.restype = sz
    L.fpq_gemm_workspace_size.argtypes = [i64, i64, i64, i32]
    L.fpq_gemm.restype = i32
    L.fpq_gemm.argtypes = [vp, i32, F, fl, f32p, vp, F, f32p, f32p, f32p, i64, i64, i64, i32, vp, sz, vp]
    L.fpq_conv2d_workspace_size.restype = sz
    L.fpq_conv2d_workspace_size.argtypes = [i64, i64, i64, i64, i64, i32, i32, i32, i32, i32]
    L.fpq_conv2d.restype = i32
    L.fpq_conv2d.argtypes = ([vp, i32, F, fl, f32p, vp, F, f32p, f32p, f32p] + [i64] * 5 + [i32] * 5 + [vp, sz, vp])
    L.fpq_search_workspace_size.restype = sz
    L.fpq_search_workspace_size.argtypes = [sz, i32, i32]
    L.fpq_search_format.restype = i32
    L.fpq_search_format.argtypes = [f32p, sz, vp, vp, i32, i32, f32p, vp, vp, sz, vp]
    L.fpq_gemm_codes_out.restype = i32
    L.fpq_gemm_codes_out.argtypes = [vp, i32, F, fl, f32p, vp, F, f32p, f32p, F, fl, f32p, u8p, i64, i64, i64, i32, vp, sz, vp]
    L.fpq_conv2d_codes_out.restype = i32
    L.fpq_conv2d_codes_out.argtypes = ([vp, i32, F, fl, f32p, vp, F, f32p, f32p, F, fl, f32p, u8p] + [i64] * 5 + [i32] * 5 +
                                       [vp, sz, vp])
    L.fpq_rl_workspace_size.restype = sz
    L.fpq_rl_workspace_size.argtypes = [i64, i64, i64]
    L.fpq_rl_init_alpha.restype = i32
    L.fpq_rl_init_alpha.argtypes = [f32p, f32p, i64, i64, F, f32p, vp]
    L.fpq_rl_step.restype = i32
    L.fpq_rl_step.argtypes = [f32p, f32p, i64, i64, F, f32p, f32p, i64, fl, fl, f32p, f32p, vp, sz, vp]
    L.fpq_rl_im2col.restype = i32
    L.fpq_rl_im2col.argtypes = [f32p, i64, i64, i64, i64, i32, i32, i32, i32, f32p, vp]
    L.fpq_rl_mask.restype = i32
    L.fpq_rl_mask.argtypes = [f32p, sz, u8p, vp]
    L.fpq_count_zeros_workspace_size.restype = sz
    L.fpq_count_zeros_workspace_size.argtypes = [sz]
    L.fpq_count_zeros.restype = i32
    L.fpq_count_zeros.argtypes = [vp, i32, sz, F, vp, vp, sz, vp]
    L.fpq_gemm_plan.restype = i32
    L.fpq_gemm_plan.argtypes = [i64, i64, i64, C.POINTER(fpq_plan_t)]
    L.fpq_conv2d_plan.restype = i32
    L.fpq_conv2d_plan.argtypes = [i64] * 5 + [i32] * 4 + [C.POINTER(fpq_plan_t)]
    L.fpq_gemm_grouped_workspace_size.restype = sz
    L.fpq_gemm_grouped_workspace_size.argtypes = [C.POINTER(fpq_gemm_problem_t), i32, i32]
    L.fpq_gemm_grouped.restype = i32
    L.fpq_gemm_grouped.argtypes = [C.POINTER(fpq_gemm_problem_t), i32, i32, F, F, i32, vp, sz, vp]
    L.fpq_packed_sparse_size.restype = sz
    L.fpq_packed_sparse_size.argtypes = [i64, i64, i32, i32, F]
    L.fpq_pack_weights_sparse.restype = i32
    L.fpq_pack_weights_sparse.argtypes = [f32p, i64, i64, i32, i32, F, f32p, u8p, vp, sz, f32p, u8p, vp, vp]
    L.fpq_gemm_sparse.restype = i32
    L.fpq_gemm_sparse.argtypes = [vp, i32, F, fl, f32p, vp, F, f32p, f32p, f32p, i64, i64, i64, vp, sz, vp]
    L.fpq_conv2d_sparse.restype = i32
    L.fpq_conv2d_sparse.argtypes = ([vp, i32, F, fl, f32p, vp, F, f32p, f32p, f32p] + [i64] * 5 + [i32] * 4 + [vp, sz, vp])
    L.fpq_int_calibrate_workspace_size.restype = sz
    L.fpq_int_calibrate_workspace_size.argtypes = [sz]
    L.fpq_int_calibrate.restype = i32
    L.fpq_int_calibrate.argtypes = [f32p, sz, i32, vp, vp, sz, vp]
    L.fpq_int_quantize.restype = i32
    L.fpq_int_quantize.argtypes = [f32p, sz, i32, fl, C.c_int32, vp, u8p, vp]
    L.fpq_int_packed_size.restype = sz
    L.fpq_int_packed_size.argtypes = [i64, i64, i32]
    L.fpq_int_pack_weights.restype = i32
    L.fpq_int_pack_weights.argtypes = [f32p, i64, i64, i32, vp, sz, f32p, vp, u8p, vp]
    L.fpq_int_gemm_workspace_size.restype = sz
    L.fpq_int_gemm_workspace_size.argtypes = [i64]
    L.fpq_int_gemm.restype = i32
    L.fpq_int_gemm.argtypes = [u8p, fl, C.c_int32, vp, vp, i32, f32p, vp, f32p, f32p, i64, i64, i64, vp, sz, vp]
    L.fpq_probe_peak.restype = i32
    L.fpq_probe_peak.argtypes = [i32, i32, vp, vp, sz, C.POINTER(C.c_double), vp]
    L.fpq_gemm_noalloc.restype = i32
    L.fpq_gemm_noalloc.argtypes = [vp, i32, F, fl, f32p, vp, F, f32p, f32p, f32p, i64, i64, i64, i32, vp]
    _lib = L
    return L


EXPORTS = ["fpq_strerror", "fpq_format_max", "fpq_format_check", "fpq_bias_to_scale", "fpq_code_bytes",
           "fpq_absmax_workspace_size", "fpq_absmax", "fpq_quantize", "fpq_padded_channels", "fpq_quantize_nhwc",
           "fpq_dequantize", "fpq_packed_size", "fpq_pack_weights", "fpq_gemm_workspace_size", "fpq_gemm",
           "fpq_conv2d_workspace_size", "fpq_conv2d", "fpq_search_workspace_size", "fpq_search_format",
           "fpq_count_zeros_workspace_size", "fpq_count_zeros", "fpq_gemm_codes_out", "fpq_conv2d_codes_out",
           "fpq_rl_workspace_size", "fpq_rl_init_alpha", "fpq_rl_step", "fpq_rl_mask", "fpq_packed_check", "fpq_rl_im2col",
           "fpq_gemm_plan", "fpq_conv2d_plan", "fpq_gemm_noalloc", "fpq_gemm_grouped_workspace_size", "fpq_gemm_grouped", "fpq_probe_peak",
           "fpq_packed_sparse_size", "fpq_pack_weights_sparse", "fpq_gemm_sparse", "fpq_conv2d_sparse",
           "fpq_int_calibrate_workspace_size", "fpq_int_calibrate", "fpq_int_quantize", "fpq_int_packed_size",
           "fpq_int_pack_weights", "fpq_int_gemm_workspace_size", "fpq_int_gemm"]


def fmt(f):
    """(e, m, b, c) tuple or fpq_format_t -> fpq_format_t."""
    if isinstance(f, fpq_format_t):
        return f
    e, m, b, c = f
    return fpq_format_t(int(e), int(m), int(b), float(c))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != 0:
        raise FpqError(status, where)


# ---- host helpers

def fpq_format_max(e, m, b):
    return lib().fpq_format_max(e, m, b)


def fpq_format_check(f):
    return lib().fpq_format_check(fmt(f))


def fpq_bias_to_scale(e, m, real_bias):
    ib, sc = C.c_int32(0), C.c_float(0)
    _check(lib().fpq_bias_to_scale(e, m, float(real_bias), C.byref(ib), C.byref(sc)), "fpq_bias_to_scale")
    return ib.value, sc.value


def fpq_code_bytes(n, f):
    return lib().fpq_code_bytes(n, fmt(f))


def fpq_padded_channels(c):
    return lib().fpq_padded_channels(c)


def fpq_packed_size(N, Cin, kh, kw, f):
    return lib().fpq_packed_size(N, Cin, kh, kw, fmt(f))


def fpq_absmax_workspace_size(n):
    return lib().fpq_absmax_workspace_size(n)


def fpq_gemm_workspace_size(M, N, K, x_is_fp32):
    return lib().fpq_gemm_workspace_size(M, N, K, int(x_is_fp32))


def fpq_conv2d_workspace_size(B, Cin, H, W, Cout, kh, kw, stride, pad, x_is_fp32):
    return lib().fpq_conv2d_workspace_size(B, Cin, H, W, Cout, kh, kw, stride, pad, int(x_is_fp32))


def fpq_gemm_plan(M, N, K):
    """(kernel, k_slices) of a linear layer."""
    p = fpq_plan_t()
    _check(lib().fpq_gemm_plan(M, N, K, C.byref(p)), "fpq_gemm_plan")
    return p.kernel, p.k_slices


def fpq_conv2d_plan(B, Cin, H, W, Cout, kh, kw, stride, pad):
    """(kernel, k_slices) of a convolution."""
    p = fpq_plan_t()
    _check(lib().fpq_conv2d_plan(B, Cin, H, W, Cout, kh, kw, stride, pad, C.byref(p)), "fpq_conv2d_plan")
    return p.kernel, p.k_slices


# ---- device entry points (torch tensors in, status checked)

class fpq_search_result(C.Structure):
    _fields_ = [("encoding", C.c_int32), ("bias_index", C.c_int32), ("ebits", C.c_int32), ("mbits", C.c_int32),
                ("int_bias", C.c_int32), ("maxval", C.c_float), ("scale", C.c_float), ("real_bias", C.c_float),
                ("mse", C.c_float), ("reserved", C.c_int32)]


def fpq_search_workspace_size(n, n_enc, n_bias):
    return lib().fpq_search_workspace_size(n, int(n_enc), int(n_bias))


def fpq_search_format(x, encodings, n_bias, mse_out, result, workspace):
    """encodings: [(e, m), ...]; mse_out: float32 tensor [n_enc * n_bias] or None; result: uint8 tensor of 40 bytes
    (read it back with search_result())."""
    ee = (C.c_int32 * len(encodings))(*[int(e) for e, _ in encodings])
    mm = (C.c_int32 * len(encodings))(*[int(m) for _, m in encodings])
    _check(lib().fpq_search_format(_ptr(x), x.numel(), C.cast(ee, C.c_void_p), C.cast(mm, C.c_void_p), len(encodings),
                                   int(n_bias), _ptr(mse_out), _ptr(result), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()), "fpq_search_format")


def search_result(result):
    """Device result buffer of fpq_search_format -> fpq_search_result (synchronises)."""
    return fpq_search_result.from_buffer_copy(bytes(result.cpu().numpy().tobytes()[:C.sizeof(fpq_search_result)]))


def fpq_count_zeros_workspace_size(n):
    return lib().fpq_count_zeros_workspace_size(n)


def fpq_count_zeros(x, x_kind, n, f, count_out, workspace):
    """x: uint8 codes or float32 values; count_out: int64 tensor of one element (the count is unsigned)."""
    _check(lib().fpq_count_zeros(_ptr(x), int(x_kind), int(n), fmt(f) if f is not None else fpq_format_t(0, 0, 0, 0.0),
                                 _ptr(count_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream()), "fpq_count_zeros")


def fpq_absmax(x, maxval, absmax_out, scale_out, workspace):
    _check(lib().fpq_absmax(_ptr(x), x.numel(), float(maxval), _ptr(absmax_out), _ptr(scale_out), _ptr(workspace),
                            workspace.numel() * workspace.element_size(), _stream()), "fpq_absmax")


def fpq_quantize(x, f, scale, scale_dev, codes):
    _check(lib().fpq_quantize(_ptr(x), x.numel(), fmt(f), float(scale), _ptr(scale_dev), _ptr(codes), _stream()),
           "fpq_quantize")


def fpq_quantize_nhwc(x, f, scale, scale_dev, codes):
    B, Cc, H, W = x.shape
    _check(lib().fpq_quantize_nhwc(_ptr(x), B, Cc, H, W, fmt(f), float(scale), _ptr(scale_dev), _ptr(codes), _stream()),
           "fpq_quantize_nhwc")


def fpq_dequantize(codes, f, scale, out):
    _check(lib().fpq_dequantize(_ptr(codes), codes.numel(), fmt(f), float(scale), _ptr(out), _stream()), "fpq_dequantize")


def fpq_pack_weights(w, f, scale, mask, packed, scale_out, codes_out=None):
    N, Cin = w.shape[0], w.shape[1]
    kh, kw = (w.shape[2], w.shape[3]) if w.dim() == 4 else (1, 1)
    _check(lib().fpq_pack_weights(_ptr(w), N, Cin, kh, kw, fmt(f), _ptr(scale), _ptr(mask), _ptr(packed),
                                  packed.numel() * packed.element_size(), _ptr(scale_out), _ptr(codes_out), _stream()),
           "fpq_pack_weights")


def fpq_gemm(x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, y, M, N, K, acc_mode=FPQ_ACC_FP32, workspace=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fpq_gemm(_ptr(x), int(x_is_fp32), fmt(fx), float(sx), _ptr(sx_dev), _ptr(packed_w), fmt(fw), _ptr(sw),
                          _ptr(bias), _ptr(y), M, N, K, int(acc_mode), _ptr(workspace), wb, _stream()), "fpq_gemm")


def gemm_problems(items):
    """[(x, sx_dev or None, packed_w, sw, bias or None, y, M, N, K), ...] of torch tensors -> ctypes array for the
    grouped call (the tensors must stay alive until the call has been made)."""
    arr = (fpq_gemm_problem_t * len(items))()
    for i, (x, sx_dev, packed_w, sw, bias, y, M, N, K) in enumerate(items):
        arr[i] = fpq_gemm_problem_t(x.data_ptr(), None if sx_dev is None else sx_dev.data_ptr(), packed_w.data_ptr(),
                                    sw.data_ptr(), None if bias is None else bias.data_ptr(), y.data_ptr(), M, N, K)
    return arr


def fpq_gemm_grouped_workspace_size(problems, x_is_fp32):
    return lib().fpq_gemm_grouped_workspace_size(problems, len(problems), int(x_is_fp32))


def fpq_gemm_grouped(problems, x_is_fp32, fx, fw, acc_mode=FPQ_ACC_FP32, workspace=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fpq_gemm_grouped(problems, len(problems), int(x_is_fp32), fmt(fx), fmt(fw), int(acc_mode), _ptr(workspace),
                                  wb, _stream()), "fpq_gemm_grouped")


def fpq_packed_sparse_size(N, Cin, kh, kw, f):
    return lib().fpq_packed_sparse_size(N, Cin, kh, kw, fmt(f))


def fpq_pack_weights_sparse(w, f, scale, mask, packed, scale_out, codes_out, dropped_out):
    """dropped_out: int64 tensor of one element."""
    N, Cin = w.shape[0], w.shape[1]
    kh, kw = (w.shape[2], w.shape[3]) if w.dim() == 4 else (1, 1)
    _check(lib().fpq_pack_weights_sparse(_ptr(w), N, Cin, kh, kw, fmt(f), _ptr(scale), _ptr(mask), _ptr(packed),
                                         packed.numel() * packed.element_size(), _ptr(scale_out), _ptr(codes_out),
                                         _ptr(dropped_out), _stream()), "fpq_pack_weights_sparse")


def fpq_gemm_sparse(x, x_is_fp32, fx, sx, sx_dev, packed_sparse, fw, sw, bias, y, M, N, K, workspace=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fpq_gemm_sparse(_ptr(x), int(x_is_fp32), fmt(fx), float(sx), _ptr(sx_dev), _ptr(packed_sparse), fmt(fw),
                                 _ptr(sw), _ptr(bias), _ptr(y), M, N, K, _ptr(workspace), wb, _stream()), "fpq_gemm_sparse")


def fpq_conv2d_sparse(x, x_is_fp32, fx, sx, sx_dev, packed_sparse, fw, sw, bias, y, B, Cin, H, W, Cout, kh, kw, stride, pad,
                      workspace=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fpq_conv2d_sparse(_ptr(x), int(x_is_fp32), fmt(fx), float(sx), _ptr(sx_dev), _ptr(packed_sparse), fmt(fw),
                                   _ptr(sw), _ptr(bias), _ptr(y), B, Cin, H, W, Cout, kh, kw, stride, pad, _ptr(workspace), wb,
                                   _stream()), "fpq_conv2d_sparse")


class fpq_int_params(C.Structure):
    _fields_ = [("scale", C.c_float), ("zero_point", C.c_int32), ("min", C.c_float), ("max", C.c_float)]


def fpq_int_calibrate(x, bits, params_out, workspace):
    """params_out: uint8 tensor of 16 bytes (read it back with int_params())."""
    _check(lib().fpq_int_calibrate(_ptr(x), x.numel(), int(bits), _ptr(params_out), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()), "fpq_int_calibrate")


def int_params(params):
    return fpq_int_params.from_buffer_copy(bytes(params.cpu().numpy().tobytes()[:C.sizeof(fpq_int_params)]))


def fpq_int_quantize(x, bits, scale, zero_point, params_dev, codes):
    _check(lib().fpq_int_quantize(_ptr(x), x.numel(), int(bits), float(scale), int(zero_point), _ptr(params_dev), _ptr(codes),
                                  _stream()), "fpq_int_quantize")


def fpq_int_packed_size(N, K, bits):
    return lib().fpq_int_packed_size(N, K, int(bits))


def fpq_int_pack_weights(w, bits, packed, scale_out, zero_point_out, codes_out=None):
    N, K = w.shape
    _check(lib().fpq_int_pack_weights(_ptr(w), N, K, int(bits), _ptr(packed), packed.numel() * packed.element_size(),
                                      _ptr(scale_out), _ptr(zero_point_out), _ptr(codes_out), _stream()), "fpq_int_pack_weights")


def fpq_int_gemm_workspace_size(M):
    return lib().fpq_int_gemm_workspace_size(M)


def fpq_int_gemm(xcodes, sx, zx, px_dev, packed_w, wbits, sw, zw, bias, y, M, N, K, workspace):
    _check(lib().fpq_int_gemm(_ptr(xcodes), float(sx), int(zx), _ptr(px_dev), _ptr(packed_w), int(wbits), _ptr(sw), _ptr(zw),
                              _ptr(bias), _ptr(y), M, N, K, _ptr(workspace), workspace.numel() * workspace.element_size(),
                              _stream()), "fpq_int_gemm")


FPQ_PROBE_MFMA_BF16, FPQ_PROBE_MFMA_FP8, FPQ_PROBE_COPY, FPQ_PROBE_MFMA_DECODE_64, FPQ_PROBE_MFMA_DECODE_32, FPQ_PROBE_FILL = 0, 1, 2, 3, 4, 5


def fpq_probe_peak(kind, iterations, src, dst):
    """One probe launch; returns its work (flops, or bytes read + written)."""
    work = C.c_double(0.0)
    _check(lib().fpq_probe_peak(int(kind), int(iterations), _ptr(src), _ptr(dst), dst.numel() * dst.element_size(),
                                C.byref(work), _stream()), "fpq_probe_peak")
    return work.value


def fpq_gemm_noalloc(x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, y, M, N, K, acc_mode=FPQ_ACC_FP32):
    _check(lib().fpq_gemm_noalloc(_ptr(x), int(x_is_fp32), fmt(fx), float(sx), _ptr(sx_dev), _ptr(packed_w), fmt(fw),
                                  _ptr(sw), _ptr(bias), _ptr(y), M, N, K, int(acc_mode), _stream()), "fpq_gemm_noalloc")


def fpq_conv2d(x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, y, B, Cin, H, W, Cout, kh, kw, stride, pad,
               acc_mode=FPQ_ACC_FP32, workspace=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fpq_conv2d(_ptr(x), int(x_is_fp32), fmt(fx), float(sx), _ptr(sx_dev), _ptr(packed_w), fmt(fw), _ptr(sw),
                            _ptr(bias), _ptr(y), B, Cin, H, W, Cout, kh, kw, stride, pad, int(acc_mode),
                            _ptr(workspace), wb, _stream()), "fpq_conv2d")


def fpq_gemm_codes_out(x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, fy, sy, sy_dev, yq, M, N, K,
                       acc_mode=FPQ_ACC_FP32, workspace=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fpq_gemm_codes_out(_ptr(x), int(x_is_fp32), fmt(fx), float(sx), _ptr(sx_dev), _ptr(packed_w), fmt(fw),
                                    _ptr(sw), _ptr(bias), fmt(fy), float(sy), _ptr(sy_dev), _ptr(yq), M, N, K,
                                    int(acc_mode), _ptr(workspace), wb, _stream()), "fpq_gemm_codes_out")


def fpq_conv2d_codes_out(x, x_is_fp32, fx, sx, sx_dev, packed_w, fw, sw, bias, fy, sy, sy_dev, yq, B, Cin, H, W, Cout,
                         kh, kw, stride, pad, acc_mode=FPQ_ACC_FP32, workspace=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fpq_conv2d_codes_out(_ptr(x), int(x_is_fp32), fmt(fx), float(sx), _ptr(sx_dev), _ptr(packed_w), fmt(fw),
                                      _ptr(sw), _ptr(bias), fmt(fy), float(sy), _ptr(sy_dev), _ptr(yq), B, Cin, H, W,
                                      Cout, kh, kw, stride, pad, int(acc_mode), _ptr(workspace), wb, _stream()),
           "fpq_conv2d_codes_out")


def fpq_rl_workspace_size(M, N, K):
    return lib().fpq_rl_workspace_size(M, N, K)


def fpq_rl_init_alpha(w, sw, f, alpha):
    N, K = w.shape
    _check(lib().fpq_rl_init_alpha(_ptr(w), _ptr(sw), N, K, fmt(f), _ptr(alpha), _stream()), "fpq_rl_init_alpha")


def fpq_rl_step(w, sw, f, alpha, a, lr, reg_weight, loss_out, grad_out, workspace):
    N, K = w.shape
    _check(lib().fpq_rl_step(_ptr(w), _ptr(sw), N, K, fmt(f), _ptr(alpha), _ptr(a), a.shape[0], float(lr), float(reg_weight),
                             _ptr(loss_out), _ptr(grad_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                             _stream()), "fpq_rl_step")


def fpq_rl_mask(alpha, mask):
    _check(lib().fpq_rl_mask(_ptr(alpha), alpha.numel(), _ptr(mask), _stream()), "fpq_rl_mask")


def fpq_packed_check(packed, N, Cin, kh, kw, f):
    """Status code (0 = the buffer was packed for these arguments); synchronises the current stream."""
    return lib().fpq_packed_check(_ptr(packed), N, Cin, kh, kw, fmt(f), _stream())


def fpq_rl_im2col(x, kh, kw, stride, pad, a):
    B_, C_, H, W = x.shape
    _check(lib().fpq_rl_im2col(_ptr(x), B_, C_, H, W, kh, kw, stride, pad, _ptr(a), _stream()), "fpq_rl_im2col")
