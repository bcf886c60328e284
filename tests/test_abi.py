"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, its host helpers
agree with the paper's closed forms, and argument validation returns the documented codes before
anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2408_06995_amd import binding as B
from paper_2408_06995_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fpq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fpq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(L, n), n
    assert sorted(names) == sorted(B.EXPORTS)


def test_format_max_and_check():
    for line in open(os.path.join(ROOT, "tests", "golden", "format_max.txt")):
        if line.strip() and line[0] != "#":
            e, m, b, c = line.split()
            assert B.fpq_format_max(int(e), int(m), int(b)) == float(c)
    assert B.fpq_format_max(0, 3, 1) == 0.0 and B.fpq_format_max(5, 3, 1) == 0.0
    for f in (synth.E4M3, synth.E5M2, synth.E2M1, synth.E1M2, synth.E3M4, synth.E2M5, synth.E3M0, (4, 3, 7, 0.0),
              (4, 3, 7, 480.0), (4, 3, 7, 0.001953125)):
        assert B.fpq_format_check(f) == 0, f
    for f in ((4, 3, 7, 449.0), (4, 3, 7, 512.0), (4, 3, 7, -448.0), (4, 4, 7, 0.0), (0, 3, 1, 0.0), (2, -1, 1, 0.0),
              (4, 3, 65, 0.0), (4, 3, 7, float("nan")), (4, 3, 7, float("inf"))):
        assert B.fpq_format_check(f) == -2, f


def test_bias_to_scale():
    assert B.fpq_bias_to_scale(4, 3, 7.0) == (7, 1.0)
    ib, sc = B.fpq_bias_to_scale(4, 3, 6.5)
    assert ib == 6 and abs(sc - 2.0 ** -0.5) < 1e-7
    # the grid of real bias b equals scale * grid of the integer bias: c(b) = scale * c(int bias)
    for rb in (3.25, 7.9, -1.5):
        ib, sc = B.fpq_bias_to_scale(4, 3, rb)
        c_real = (2 - 2.0 ** -3) * 2.0 ** (16 - rb - 1)
        assert abs(sc * B.fpq_format_max(4, 3, ib) / c_real - 1) < 1e-6


def test_sizes():
    assert B.fpq_code_bytes(10, synth.E4M3) == 10
    assert B.fpq_code_bytes(11, synth.E2M1) == 6
    assert B.fpq_padded_channels(4) == 16 and B.fpq_padded_channels(320) == 320
    assert B.fpq_packed_size(320, 320, 1, 1, synth.E4M3) == 256 + 320 * 384
    assert B.fpq_packed_size(320, 320, 3, 3, synth.E4M3) == 256 + 320 * 2944
    assert B.fpq_packed_size(1280, 1280, 3, 3, synth.E2M1) == 256 + 1280 * 11520 // 2
    assert B.fpq_packed_size(0, 320, 1, 1, synth.E4M3) == 0
    assert B.fpq_absmax_workspace_size(0) == 4 and B.fpq_absmax_workspace_size(10 ** 9) == 4096
    assert B.fpq_gemm_workspace_size(256, 320, 320, 0) == 0
    assert B.fpq_gemm_workspace_size(256, 320, 320, 1) == 256 * 320
    assert B.fpq_conv2d_workspace_size(1, 4, 64, 64, 320, 3, 3, 1, 1, 1) == 64 * 64 * 16


def test_argument_validation_without_gpu():
    L = B.lib()
    f = B.fmt(synth.E4M3)
    bad = B.fmt((4, 3, 7, 449.0))
    bad_fmt = bad
    p = C.c_void_p(4096)          # never dereferenced: every call below fails validation first
    assert L.fpq_quantize(p, 16, bad, 1.0, None, p, None) == -2
    assert L.fpq_quantize(p, 16, f, 0.0, None, p, None) == -3
    assert L.fpq_quantize(p, 16, f, float("nan"), None, p, None) == -3
    assert L.fpq_quantize(p, 16, f, float("inf"), None, p, None) == -3
    assert L.fpq_quantize(None, 16, f, 1.0, None, p, None) == -1
    assert L.fpq_quantize(p, 16, f, 1.0, None, None, None) == -1
    assert L.fpq_quantize(None, 0, f, 1.0, None, None, None) == 0
    assert L.fpq_quantize(C.c_void_p(4098), 16, f, 1.0, None, p, None) == -5
    assert L.fpq_absmax(p, 16, 448.0, None, None, p, 4, None) == -1
    assert L.fpq_absmax(p, 10 ** 6, 448.0, p, p, p, 4, None) == -6
    assert L.fpq_absmax(p, 16, 0.0, p, p, p, 4, None) == -2
    assert L.fpq_quantize_nhwc(p, 0, 4, 8, 8, f, 1.0, None, p, None) == -4
    assert L.fpq_quantize_nhwc(p, 1, 4, 8, 8, f, 1.0, None, C.c_void_p(4100), None) == -5
    assert L.fpq_pack_weights(p, 8, 0, 1, 1, f, None, None, p, 1 << 20, p, None, None) == -4
    assert L.fpq_pack_weights(p, 8, 32, 1, 1, f, None, None, p, 64, p, None, None) == -6
    assert L.fpq_pack_weights(p, 8, 32, 1, 1, f, None, None, None, 1 << 20, p, None, None) == -1
    e2m1 = B.fmt(synth.E2M1)
    # fpq_gemm: shape, null, scale, alignment, workspace, unsupported format pairing
    assert L.fpq_gemm(p, 0, f, 1.0, None, p, f, p, None, p, 8, 8, 0, 0, None, 0, None) == -4
    assert L.fpq_gemm(None, 0, f, 1.0, None, p, f, p, None, p, 8, 8, 32, 0, None, 0, None) == -1
    assert L.fpq_gemm(p, 0, f, -1.0, None, p, f, p, None, p, 8, 8, 32, 0, None, 0, None) == -3
    assert L.fpq_gemm(p, 0, f, 1.0, None, p, f, p, None, p, 8, 8, 24, 0, None, 0, None) == -5
    assert L.fpq_gemm(p, 1, f, 1.0, None, p, f, p, None, p, 8, 8, 32, 0, None, 0, None) == -6
    assert L.fpq_gemm(p, 2, f, 0.0, None, p, f, p, None, p, 8, 8, 32, 0, None, 0, None) == -6   # dynamic scale: no sx needed
    assert L.fpq_gemm(p, 3, f, 1.0, None, p, f, p, None, p, 8, 8, 32, 0, None, 0, None) == -8
    # encoding / bias search: every check below returns before a launch
    import ctypes as CT
    ee, mm = (CT.c_int32 * 2)(4, 5), (CT.c_int32 * 2)(3, 2)
    bad = (CT.c_int32 * 2)(4, 6)
    ev, mv, bv = CT.cast(ee, CT.c_void_p), CT.cast(mm, CT.c_void_p), CT.cast(bad, CT.c_void_p)
    assert L.fpq_search_format(p, 100, ev, mv, 0, 111, None, p, p, 1 << 20, None) == -4
    assert L.fpq_search_format(p, 100, ev, mv, 2, 129, None, p, p, 1 << 20, None) == -4
    assert L.fpq_search_format(p, 100, ev, mv, 2, 111, None, None, p, 1 << 20, None) == -1
    assert L.fpq_search_format(p, 100, ev, bv, 2, 111, None, p, p, 1 << 20, None) == -2
    assert L.fpq_search_format(p, 100, ev, mv, 2, 111, None, p, p, 64, None) == -6
    assert B.fpq_search_workspace_size(5000, 4, 111) == 4096 + 256 + 3 * 444 * 4 + (256 - 3 * 444 * 4 % 256) % 256
    assert B.fpq_search_workspace_size(5000, 9, 111) == 0
    assert B.fpq_gemm_workspace_size(8, 8, 32, 2) == B.fpq_gemm_workspace_size(8, 8, 32, 1) + 4096 + 256
    assert L.fpq_gemm(p, 0, e2m1, 1.0, None, p, f, p, None, p, 8, 8, 32, 0, None, 0, None) == -8
    assert L.fpq_gemm(p, 0, B.fmt(synth.E3M4), 1.0, None, p, f, p, None, p, 8, 8, 32, 1, None, 0, None) == -8
    assert L.fpq_gemm(p, 0, f, 1.0, None, p, f, p, None, p, 8, 8, 32, 7, None, 0, None) == -8
    assert L.fpq_gemm(p, 0, f, 1.0, None, p, f, p, None, p, 0, 8, 32, 0, None, 0, None) == 0
    assert L.fpq_conv2d(p, 0, f, 1.0, None, p, f, p, None, p, 1, 16, 2, 2, 8, 3, 3, 1, 0, 0, None, 0, None) == -4
    assert L.fpq_conv2d(p, 0, f, 1.0, None, p, f, p, None, p, 1, 16, 8, 8, 8, 3, 3, 0, 1, 0, None, 0, None) == -4
    # a contraction longer than fpq_pack_weights can have packed (2^28 codes per output channel)
    assert L.fpq_conv2d(p, 0, f, 1.0, None, p, e2m1, p, None, p, 1, 1 << 20, 1, 1, 1, 48, 48, 1, 24, 0, None, 0, None) == -4
    assert L.fpq_pack_weights(p, 1, 1 << 20, 48, 48, e2m1, None, None, p, 1 << 40, p, None, None) == -4
    # zero count: null, kind, format, workspace, alignment
    assert B.fpq_count_zeros_workspace_size(10 ** 9) == 8192
    assert L.fpq_count_zeros(p, 0, 100, f, None, p, 8192, None) == -1
    assert L.fpq_count_zeros(None, 0, 100, f, p, p, 8192, None) == -1
    assert L.fpq_count_zeros(p, 2, 100, f, p, p, 8192, None) == -8
    assert L.fpq_count_zeros(p, 0, 100, bad_fmt, p, p, 8192, None) == -2
    assert L.fpq_count_zeros(p, 0, 100, f, p, p, 8184, None) == -6
    assert L.fpq_count_zeros(p, 0, 100, f, C.c_void_p(4100), p, 8192, None) == -5
    assert L.fpq_count_zeros(C.c_void_p(4098), 1, 100, f, p, p, 8192, None) == -5
    assert L.fpq_strerror(-2).decode().startswith("invalid ExMy")
    assert L.fpq_strerror(0) == b"ok"


def test_plan_query_and_format_range():
    L = B.lib()
    assert B.fpq_gemm_plan(8, 1280, 1280) == (B.FPQ_KERNEL_ROWS16, 1)
    assert B.fpq_gemm_plan(616, 320, 768) == (B.FPQ_KERNEL_SMALL_TILE, 1)
    assert B.fpq_gemm_plan(4096, 333, 640) == (B.FPQ_KERNEL_SMALL_TILE, 1)          # N not a multiple of 160
    k, s = B.fpq_gemm_plan(512, 1280, 5120)
    assert k == B.FPQ_KERNEL_128x160 and s > 1
    assert B.fpq_gemm_workspace_size(512, 1280, 5120, 0) == s * 512 * 1280 * 4
    k, s = B.fpq_conv2d_plan(8, 1280, 32, 32, 1280, 3, 3, 1, 1)
    assert k == B.FPQ_KERNEL_256x160 and s == 1
    p = B.fpq_plan_t()
    assert L.fpq_gemm_plan(0, 8, 8, C.byref(p)) == -4
    assert L.fpq_gemm_plan(8, 8, 8, None) == -1
    assert L.fpq_conv2d_plan(1, 16, 2, 2, 8, 3, 3, 1, 0, C.byref(p)) == -4
    # encodings whose largest value would overflow the encoder's fp32 rounding constant are rejected
    assert B.fpq_format_check((7, 0, 23, 0.0)) == 0 and B.fpq_format_check((7, 0, 22, 0.0)) == -2
    assert B.fpq_format_check((6, 1, -42, 0.0)) == 0 and B.fpq_format_check((6, 1, -43, 0.0)) == -2
    assert B.fpq_format_max(7, 0, 0) == 0.0
    assert B.fpq_format_check((5, 2, -64, 0.0)) == 0 and B.fpq_format_check((4, 3, -64, 0.0)) == 0


def test_noalloc_entry_validates_before_touching_the_gpu():
    L = B.lib()
    f = B.fmt(synth.E4M3)
    p = C.c_void_p(4096)
    assert L.fpq_gemm_noalloc(p, 1, f, 1.0, None, p, f, p, None, p, 1 << 20, 320, 4096, 0, None) == -6   # 4 GiB of codes
    assert L.fpq_gemm_noalloc(p, 0, f, 1.0, None, p, f, p, None, p, 0, 8, 32, 0, None) == 0
    assert L.fpq_gemm_noalloc(p, 0, f, 1.0, None, p, f, p, None, p, 8, 0, 32, 0, None) == -4
    assert L.fpq_strerror(-9).decode().startswith("packed weights")
