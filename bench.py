#!/usr/bin/env python3
"""Benchmark of the quantized-layer hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input: for every layer of the
workload, absmax calibration of the fp32 activation (the per-tensor scale never leaves the device),
activation quantize to E4M3 codes, and the quantized linear / conv layer on pre-packed weights --
all three inside one fpq_gemm / fpq_conv2d call in its dynamic-scale mode -- once with E4M3 weights
(W8A8) and once with E2M1 weights (W4A8).  Weight packing is the offline step and is done
before the timed region; inputs are resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg4|cfg3|cfg2|cfg1]
                    [--acc fp32|fp8mfma] [--no-cpu-baseline]

Prints ONE JSON line: metric / value (whole-step TFLOP/s), the roofline object of the dominant
kernel (live hipEvent timing of every GEMM launch, on the stream the launches use), the CPU oracle
baseline timed on the host cores, the quantize kernel's bandwidth, and the same step through the
FP8-MFMA accumulate mode for reference.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense fp8 MFMA (also the rate of fp8 x fp4)
PEAK_HBM_GBS = 8000.0
ALU_LANE_RATE = 256 * 4 * 16 * 2.4e9   # vector instructions per lane and second: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
SEARCH_OPS = 11                        # vector instructions per element and candidate in the search kernel's inner loop
# HBM-side bytes per layer launch from two hardware-counter passes of a profiler (FETCH_SIZE, then WRITE_SIZE, the
# split-K reductions included): not measurable from inside this script, hence a constant, valid only for the workload,
# accumulate mode and call structure it was taken on; the summary file named here holds the command and the arithmetic.
MEASURED_TRAFFIC = {
    ("cfg5", "fp32", "grouped"): {"bytes_per_launch": 65.00e6,
                                  "source": "profiles/cfg5_layer_kernels_hbm_traffic_pmc.txt: 30.35 MB fetched + 34.65 MB written "
                                            "per layer over 4 x 500 layers"},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--acc", default="fp32", choices=["fp32", "fp8mfma"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the quantize-bandwidth probe and the other acc mode")
    ap.add_argument("--per-class", metavar="FILE",
                    help="also time every distinct layer shape of the workload on its own (layer kernel on prepared codes) "
                         "and write a table to FILE: time, TFLOP/s, share of the MFMA peak, share of the roofline "
                         "t_min = max(2MNK / peak, algorithmic bytes / 8 TB/s) and which term binds")
    ap.add_argument("--eager", action="store_true",
                    help="launch every step call by call instead of replaying a captured graph (for hardware-counter "
                         "passes of a profiler, where timing does not matter and every dispatch is serialized anyway)")
    ap.add_argument("--no-grouping", action="store_true",
                    help="one call per layer also for the layers that the default step hands to fpq_gemm_grouped (the "
                         "cross-attention key / value projections and the time-embedding projections, which do not "
                         "depend on the layers between them)")
    ap.add_argument("--layer-kernels-only", action="store_true",
                    help="for hardware-counter passes of a profiler: set up, then launch every GEMM / conv call of one "
                         "step (the launches the roofline object is about) exactly --steps times, call by call, and "
                         "exit; nothing else of the benchmark runs, so per-launch counter figures are the profiler's "
                         "sums over the layer kernels divided by steps x layers")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (the known-size kernel that hardware-counter "
                         "readings of a profiler run are scaled by)")
    return ap.parse_args()


WORKLOAD_NAMES = {
    "cfg1": "configs[0]: single linear layer 256x320x320, W8A8 + W4A8",
    "cfg2": "configs[1]: 3x3 conv 320->320 on 64x64, batch 1 (M=4096 K=2880 N=320), W8A8 + W4A8",
    "cfg3": "configs[2]: transformer-block projections (QKV, GEGLU, FF-out, cross-attn K/V), W8A8 + W4A8",
    "cfg4": "configs[3]: deep-stage 3x3 conv 1280->1280 on 16x16, batch 8 (M=2048 K=11520 N=1280), W8A8 + W4A8",
    "cfg5": "configs[4]: full SD-like U-Net denoising-step layer set (250 conv/linear layers, batch 8, 64x64 latent), "
            "W8A8 (E4M3 weights) then W4A8 (E2M1 weights)",
}


class LayerState:
    pass


def board_state():
    """Board power in watts and shader clock in MHz as the driver reports them (sysfs), or None where they cannot be read."""
    import glob
    try:
        hw = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")[0]
        watts = int(open(hw + "/power1_input").read()) / 1e6
        cap = int(open(hw + "/power1_cap").read()) / 1e6
        cur = [l for l in open(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")[0]) if "*" in l]
        mhz = int(cur[0].split(":")[1].strip().lower().split("mhz")[0]) if cur else None
        return {"W": round(watts), "cap_W": round(cap), "sclk_MHz": mhz}
    except Exception:
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported (no multi-GPU path exists)"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2408_06995_amd import binding as B
    from paper_2408_06995_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()   # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = int(args.workload[3:])
    layers = synth.unet_layers() if cfg == 5 else synth.config_layers(cfg)
    FX, FW8, FW4 = synth.E4M3, synth.E4M3, synth.E2M1
    acc = B.FPQ_ACC_FP32 if args.acc == "fp32" else B.FPQ_ACC_FP8_MFMA

    # ---- set-up (untimed): inputs resident in HBM, weights quantized and packed offline
    states = []
    max_y = 0
    max_ws = 0
    max_part = 0
    for li, L in enumerate(layers):
        s = LayerState()
        s.L = L
        sx_seed, sw_seed, sh_seed = synth.seeds(cfg, li)
        if L.kind == "conv":
            s.x = synth.activations_torch((L.B, L.Cin, L.H, L.W), sx_seed, dev)
            wshape = (L.Cout, L.Cin, L.k, L.k)
            ws = B.fpq_conv2d_workspace_size(L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, 2)
        else:
            s.x = synth.activations_torch((L.M, L.K), sx_seed, dev)
            wshape = (L.N, L.K)
            ws = B.fpq_gemm_workspace_size(L.M, L.N, L.K, 2)
        w = synth.weights_torch(wshape, sw_seed, dev)
        h = synth.rounding_mask_torch(wshape, sh_seed, dev)
        kk = L.k if L.kind == "conv" else 1
        s.packed = {}
        s.sw = {}
        for tag, fw, mask in (("w8", FW8, None), ("w4", FW4, h)):   # rounding mask only for FP4 (Section V-B)
            p = torch.empty(B.fpq_packed_size(L.N, L.Cin, kk, kk, fw), dtype=torch.uint8, device=dev)
            sw = torch.empty(L.N, dtype=torch.float32, device=dev)
            B.fpq_pack_weights(w, fw, None, mask, p, sw, None)
            s.packed[tag], s.sw[tag] = p, sw
        del w, h
        s.scale = torch.empty(2, dtype=torch.float32, device=dev)   # [absmax, scale]
        # layers that do not depend on the layers between them are handed to the library as one group: all key / value
        # projections of the cross-attention blocks read the text context, all time-embedding projections of the
        # residual blocks read the embedding that the two time-embedding layers produce
        s.group = None
        if cfg == 5 and not args.no_grouping and L.kind == "linear":
            if L.name.endswith("attn2.k") or L.name.endswith("attn2.v"):
                s.group = "context_kv"
            elif L.name.endswith(".temb"):
                s.group = "time_embedding"
        if s.group:
            s.y_own = torch.empty(L.M * L.N, dtype=torch.float32, device=dev)   # the members' results coexist
        max_y = max(max_y, L.M * L.N)
        max_ws = max(max_ws, ws)
        if L.kind == "conv":
            max_part = max(max_part, B.fpq_conv2d_workspace_size(L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, 0))
        else:
            max_part = max(max_part, B.fpq_gemm_workspace_size(L.M, L.N, L.K, 0))
        states.append(s)
    torch.cuda.synchronize()
    y = torch.empty(max_y, dtype=torch.float32, device=dev)
    ws_buf = torch.empty(max(max_ws, 256), dtype=torch.uint8, device=dev)
    amax_ws = torch.empty(1026, dtype=torch.float32, device=dev)   # partial maxima of the absmax reduction
    part_buf = torch.empty(max(max_part, 256), dtype=torch.uint8, device=dev)   # split-K partial sums (codes-input calls)

    def run_layer(s, tag, fw, acc_mode, static_scale=False):
        """One layer call.  Default: dynamic scale (absmax found inside the call).  static_scale: the per-tensor
        scale was calibrated beforehand (s.scale), as the paper does offline; the call quantizes and runs the layer."""
        L = s.L
        xk = B.FPQ_X_FP32 if static_scale else B.FPQ_X_FP32_DYNAMIC
        sdev = s.scale[1:2] if static_scale else None
        if L.kind == "conv":
            B.fpq_conv2d(s.x, xk, FX, 0.0, sdev, s.packed[tag], fw, s.sw[tag], None, y, L.B, L.Cin,
                         L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, acc_mode, ws_buf)
        else:
            B.fpq_gemm(s.x, xk, FX, 0.0, sdev, s.packed[tag], fw, s.sw[tag], None, y, L.M, L.N, L.K,
                       acc_mode, ws_buf)

    groups = {}
    for s in states:
        if s.group:
            groups.setdefault(s.group, []).append(s)
    group_args, group_ws = {}, {}
    for gname, members in groups.items():
        for tag in ("w8", "w4"):
            group_args[gname, tag, "fp32"] = B.gemm_problems(
                [(m.x, None, m.packed[tag], m.sw[tag], None, m.y_own, m.L.M, m.L.N, m.L.K) for m in members])
        group_ws[gname] = torch.empty(B.fpq_gemm_grouped_workspace_size(group_args[gname, "w8", "fp32"], B.FPQ_X_FP32_DYNAMIC),
                                      dtype=torch.uint8, device=dev)

    def step(acc_mode, static_scale=False):
        for tag, fw in (("w8", FW8), ("w4", FW4)):
            done = set()
            for s in states:
                if s.group and not static_scale:
                    if s.group not in done:      # the whole group at the place of its first member
                        done.add(s.group)
                        B.fpq_gemm_grouped(group_args[s.group, tag, "fp32"], B.FPQ_X_FP32_DYNAMIC, FX, fw, acc_mode,
                                           group_ws[s.group])
                    continue
                run_layer(s, tag, fw, acc_mode, static_scale)

    flops_step = 2 * sum(synth.flops(L) for L in layers)

    def timed(acc_mode, steps, warmup, static_scale=False):
        """Warm up eagerly, capture one step into a HIP graph (the step is ~2000 short launches; issued from
        Python the host cannot keep the GPU fed), then time `steps` replays."""
        for _ in range(max(1, warmup)):
            step(acc_mode, static_scale)
        torch.cuda.synchronize()
        if args.eager:
            t0 = time.perf_counter()
            for _ in range(steps):
                step(acc_mode, static_scale)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(acc_mode, static_scale)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    sec = None if args.layer_kernels_only else timed(acc, args.steps, args.warmup)

    # ---- the GEMM kernels alone: every layer's activation codes are prepared first (untimed), then all GEMM /
    # conv launches of one step (and the split-K reductions that belong to them) are captured into one graph
    # and timed with hipEvents on the stream they run on
    codes_bufs = {}

    def prepare_codes():
        for s in states:
            L = s.L
            B.fpq_absmax(s.x, FX[3], s.scale[0:1], s.scale[1:2], amax_ws)
            if L.kind == "conv":
                buf = torch.empty(L.B * L.H * L.W * B.fpq_padded_channels(L.Cin), dtype=torch.uint8, device=dev)
                B.fpq_quantize_nhwc(s.x, FX, 0.0, s.scale[1:2], buf)
            elif B.fpq_padded_channels(L.K) == L.K:
                buf = torch.empty(L.M * L.K, dtype=torch.uint8, device=dev)
                B.fpq_quantize(s.x, FX, 0.0, s.scale[1:2], buf)
            else:
                buf = None   # rows need padding: only reachable through the fused entry point
            codes_bufs[L.name] = buf
        torch.cuda.synchronize()

    def gemm_only(acc_mode):
        n = 0
        for tag, fw in (("w8", FW8), ("w4", FW4)):
            done = set()
            for s in states:
                L = s.L
                buf = codes_bufs[L.name]
                if buf is None:
                    continue
                if s.group:
                    if s.group not in done:
                        done.add(s.group)
                        key = (s.group, tag, "codes")
                        if key not in group_args:
                            group_args[key] = B.gemm_problems(
                                [(codes_bufs[m.L.name], m.scale[1:2], m.packed[tag], m.sw[tag], None, m.y_own, m.L.M, m.L.N,
                                  m.L.K) for m in groups[s.group]])
                        B.fpq_gemm_grouped(group_args[key], B.FPQ_X_CODES, FX, fw, acc_mode, None)
                    n += 1       # counted per layer: the roofline object averages over layers, however they are launched
                    continue
                if L.kind == "conv":
                    B.fpq_conv2d(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, y, L.B, L.Cin, L.H,
                                 L.W, L.Cout, L.k, L.k, L.stride, L.pad, acc_mode, part_buf)
                else:
                    B.fpq_gemm(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, y, L.M, L.N, L.K,
                               acc_mode, part_buf)
                n += 1
        return n

    def gemm_breakdown(acc_mode, reps=5):
        if not codes_bufs:
            prepare_codes()
        nlaunch = gemm_only(acc_mode)
        torch.cuda.synchronize()
        if args.eager:
            replay = lambda: gemm_only(acc_mode)
        else:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                gemm_only(acc_mode)
            replay = graph.replay
        replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            replay()
        e1.record()
        e1.synchronize()
        tot_ms = e0.elapsed_time(e1) / reps
        tot_fl = 2 * sum(synth.flops(s.L) for s in states if codes_bufs[s.L.name] is not None)
        # board power and clock while the same replays run (a second, untimed round: the reads take host time)
        board = None
        if not args.eager:
            for _ in range(40):
                replay()
            time.sleep(0.25)
            board = board_state()
            torch.cuda.synchronize()
        return tot_ms, tot_fl, nlaunch, {"board": board}

    if args.layer_kernels_only:
        prepare_codes()
        for _ in range(args.steps):
            n_layers = gemm_only(acc)
        torch.cuda.synchronize()
        print(json.dumps({"layer_kernels_only": True, "executions": args.steps, "layers_per_execution": n_layers,
                          "acc_mode": args.acc, "grouped_calls": {g: len(m) for g, m in groups.items()}}))
        return
    g_ms, g_fl, g_n, per_layer = gemm_breakdown(acc)
    # algorithmic bytes of those launches: activation codes once (not the im2col expansion), packed weights, fp32 output
    alg_bytes = 0
    for s in states:
        L = s.L
        if codes_bufs[L.name] is None:
            continue
        alg_bytes += 2 * (codes_bufs[L.name].numel() + 4 * L.M * L.N) + s.packed["w8"].numel() + s.packed["w4"].numel()
    peak = PEAK_BF16_TFLOPS if acc == B.FPQ_ACC_FP32 else PEAK_FP8_TFLOPS
    achieved = g_fl / (g_ms * 1e-3) / 1e12
    traffic = MEASURED_TRAFFIC.get((args.workload, args.acc, "grouped" if groups else "one call per layer"))
    roofline = {"bound": "mfma", "kernel": "fpq::gemm_dma_kernel / gemm_kernel (all GEMM and conv launches of one step, one graph)", "achieved": round(achieved, 2),
                "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                # the target of this workload is stated against the 8-bit matrix peak, which the exact (fp32-accumulate)
                # mode cannot use: its products go through the bf16 matrix instruction, whose peak is half of it
                "frac_of_fp8_peak": round(achieved / PEAK_FP8_TFLOPS, 4),
                "traffic": None if traffic is None else traffic["bytes_per_launch"],
                "traffic_source": None if traffic is None else traffic["source"],
                "traffic_unit": "bytes per layer launch (L2 <-> fabric, rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, "
                                "factors from a 256 MiB copy kernel)",
                "algorithmic_bytes_per_launch": round(alg_bytes / g_n),
                "launches": g_n, "avg_launch_us": round(g_ms * 1e3 / g_n, 2),
                "gemm_ms_per_step": round(g_ms, 4),
                # the part runs these kernels at its board power limit with the shader clock below the 2.4 GHz of the
                # published peaks (what the driver reports in the middle of 40 further replays of the same graph)
                "board_during_layer_kernels": per_layer.get("board")}

    out = {
        "metric": "W8A8+W4A8 GEMM/conv TFLOP/s incl. absmax + activation quantize (whole step)",
        "value": round(flops_step / sec / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8/fp4 codes -> bf16 MFMA, fp32 accumulate" if acc == B.FPQ_ACC_FP32 else "fp8/fp4 MFMA",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.workload], "layers": len(layers), "flop_per_step": flops_step,
                   "acc_mode": args.acc,
                   "grouped_calls": {g: len(m) for g, m in groups.items()}},
        "roofline": roofline,
    }

    def measure_peaks():
        """What the part sustains on the bare matrix instructions and on a plain copy (probe kernels of the library)."""
        pk = {}
        pdst = torch.empty(2048 * 256, dtype=torch.float32, device=dev)
        for name, kind, iters in (("bf16_mfma_TFLOP/s", B.FPQ_PROBE_MFMA_BF16, 1500), ("fp8_mfma_TFLOP/s", B.FPQ_PROBE_MFMA_FP8, 1500),
                                  ("bf16_mfma_with_conversions_64x160_TFLOP/s", B.FPQ_PROBE_MFMA_DECODE_64, 4000),
                                  ("bf16_mfma_with_conversions_32x160_TFLOP/s", B.FPQ_PROBE_MFMA_DECODE_32, 8000)):
            B.fpq_probe_peak(kind, 100, None, pdst)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            work = sum(B.fpq_probe_peak(kind, iters, None, pdst) for _ in range(3))
            e1.record()
            e1.synchronize()
            pk[name] = round(work / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
            for _ in range(30):        # long enough for the power reading to settle, then read it with the probe still running
                B.fpq_probe_peak(kind, iters, None, pdst)
            time.sleep(0.12)
            pk[name.replace("_TFLOP/s", "_board")] = board_state()
            torch.cuda.synchronize()
        csrc = [torch.empty(128 << 20, dtype=torch.float32, device=dev).normal_() for _ in range(2)]   # 512 MiB each
        cdst = [torch.empty(128 << 20, dtype=torch.float32, device=dev) for _ in range(2)]
        B.fpq_probe_peak(B.FPQ_PROBE_COPY, 1, csrc[0], cdst[0])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        work = sum(B.fpq_probe_peak(B.FPQ_PROBE_COPY, 1, csrc[i & 1], cdst[i & 1]) for i in range(8))
        e1.record()
        e1.synchronize()
        pk["copy_GB/s_read_plus_write"] = round(work / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        B.fpq_probe_peak(B.FPQ_PROBE_FILL, 1, None, cdst[0])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        work = sum(B.fpq_probe_peak(B.FPQ_PROBE_FILL, 1, None, cdst[i & 1]) for i in range(8))
        e1.record()
        e1.synchronize()
        pk["fill_GB/s_write_only"] = round(work / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        del csrc, cdst
        pk["note"] = ("register-only MFMA loops with operands that change every instruction (bare, and with the code-to-bf16 "
                      "conversions a k-step of the layer kernels' wave tiles pays), a 512 MiB device copy and a 512 MiB fill; "
                      "the nominal peaks are %g / %g TFLOP/s and %g GB/s" % (PEAK_BF16_TFLOPS, PEAK_FP8_TFLOPS, PEAK_HBM_GBS))
        return pk

    if args.per_class:
        # one representative layer per distinct (kind, kernel, stride, M, K, N); 8 launches in a graph, 4 replays
        seen, lines = {}, []
        for s in states:
            L = s.L
            key = (L.kind, L.k if L.kind == "conv" else 1, L.stride if L.kind == "conv" else 1, L.M, L.K, L.N)
            seen.setdefault(key, [s, 0])[1] += 1
        peak_fl = (PEAK_BF16_TFLOPS if acc == B.FPQ_ACC_FP32 else PEAK_FP8_TFLOPS) * 1e12
        mp = measure_peaks()
        m_fl = mp["bf16_mfma_TFLOP/s" if acc == B.FPQ_ACC_FP32 else "fp8_mfma_TFLOP/s"] * 1e12
        m_bw = mp["copy_GB/s_read_plus_write"] * 1e9
        m_fill = mp["fill_GB/s_write_only"] * 1e9
        m_cvt = mp["bf16_mfma_with_conversions_64x160_TFLOP/s"]
        lines.append("# per shape class of %s, accumulate mode %s: layer kernel alone on prepared codes" % (args.workload, args.acc))
        lines.append("# t_min = max(2MNK / %.0f TFLOP/s, (activation codes + packed weights + fp32 output) / 8 TB/s): the published peaks" % (peak_fl / 1e12))
        lines.append("# %%machine = the same with what this part sustained in this run: 2MNK on the bare matrix instruction (%.0f TFLOP/s; "
                     "%.0f with the conversions of a 64 x 160 wave tile in the loop), the fp32 output at the rate of a device fill "
                     "(%.0f GB/s) plus codes and weights at that of a device copy (%.0f GB/s read + write)"
                     % (m_fl / 1e12, m_cvt, m_fill / 1e9, m_bw / 1e9))
        lines.append("%-4s %-6s %1s %1s %6s %6s %6s %4s %9s %9s %7s %9s %6s %9s" % (
            "w", "kind", "k", "s", "M", "K", "N", "x", "us", "TFLOP/s", "%peak", "%roofline", "bound", "%machine"))
        tot_t, tot_min, tot_mach = 0.0, 0.0, 0.0
        for key, (s, cnt) in seen.items():
            L = s.L
            buf = codes_bufs.get(L.name)
            if buf is None:
                continue
            for tag, fw in (("w8", FW8), ("w4", FW4)):
                def one():
                    if L.kind == "conv":
                        B.fpq_conv2d(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, y, L.B, L.Cin, L.H, L.W,
                                     L.Cout, L.k, L.k, L.stride, L.pad, acc, part_buf)
                    else:
                        B.fpq_gemm(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, y, L.M, L.N, L.K, acc,
                                   part_buf)
                one()
                torch.cuda.synchronize()
                gc = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gc):
                    for _ in range(8):
                        one()
                gc.replay()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(4):
                    gc.replay()
                e1.record()
                e1.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 32
                fl = synth.flops(L)
                nbytes = buf.numel() + s.packed[tag].numel() + 4 * L.M * L.N
                t_f, t_b = fl / peak_fl * 1e6, nbytes / (PEAK_HBM_GBS * 1e9) * 1e6
                t_min = max(t_f, t_b)
                t_mach = max(fl / m_fl * 1e6, (4 * L.M * L.N / m_fill + (nbytes - 4 * L.M * L.N) / m_bw) * 1e6)
                lines.append("%-4s %-6s %1d %1d %6d %6d %6d %4d %9.1f %9.1f %7.1f %9.1f %6s %9.1f" % (
                    tag, L.kind, key[1], key[2], L.M, L.K, L.N, cnt, us, fl / us / 1e6, 100 * fl / (us * 1e-6) / peak_fl,
                    100 * t_min / us, "mfma" if t_f >= t_b else "hbm", 100 * t_mach / us))
                tot_t += us * cnt
                tot_min += t_min * cnt
                tot_mach += t_mach * cnt
        lines.append("# all layers of the step, each class weighted by its count: %.1f us against a roofline t_min of %.1f us (%.1f %%); "
                     "against the machine's measured ceilings %.1f us (%.1f %%)"
                     % (tot_t, tot_min, 100 * tot_min / tot_t, tot_mach, 100 * tot_mach / tot_t))
        with open(args.per_class, "w") as f:
            f.write("\n".join(lines) + "\n")

    if not args.no_extras:
        # the same step with per-tensor scales calibrated beforehand (the paper finds them offline): the timed region
        # then holds quantize + layer only.  prepare_codes() above has left absmax / scale of every layer in s.scale.
        sec_s = timed(acc, max(2, args.steps // 2), 1, static_scale=True)
        out["static_scale_step"] = {"ms_per_step": round(sec_s * 1e3, 4), "value": round(flops_step / sec_s / 1e12, 3),
                                    "unit": "TFLOP/s"}
        # every layer from codes to codes: activation codes in, the result quantized in the epilogue for a following
        # quantized layer (E4M3, per-tensor scale found beforehand from the layer's own fp32 result) and written as one
        # byte per output.  One launch per layer and a quarter of the output bytes: what a chain of quantized layers
        # costs once scales are static, against the fp32-out launches of the roofline object.
        def codes_to_codes():
            yq = torch.empty(max(s.L.M * ((s.L.N + 15) // 16 * 16) for s in states), dtype=torch.uint8, device=dev)
            sy = {}
            ymax = torch.empty(2, dtype=torch.float32, device=dev)
            for s in states:          # calibrate the output scales (untimed): absmax of the layer's fp32 result
                L = s.L
                buf = codes_bufs[L.name]
                if buf is None:
                    continue
                for tag, fw in (("w8", FW8), ("w4", FW4)):
                    if L.kind == "conv":
                        B.fpq_conv2d(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, y, L.B, L.Cin, L.H,
                                     L.W, L.Cout, L.k, L.k, L.stride, L.pad, acc, part_buf)
                    else:
                        B.fpq_gemm(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, y, L.M, L.N, L.K, acc,
                                   part_buf)
                    sy[L.name, tag] = torch.empty(2, dtype=torch.float32, device=dev)
                    B.fpq_absmax(y[:L.M * L.N], FX[3], sy[L.name, tag][0:1], sy[L.name, tag][1:2], amax_ws)

            def run():
                for tag, fw in (("w8", FW8), ("w4", FW4)):
                    for s in states:
                        L = s.L
                        buf = codes_bufs[L.name]
                        if buf is None:
                            continue
                        if L.kind == "conv":
                            B.fpq_conv2d_codes_out(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, FX, 0.0,
                                                   sy[L.name, tag][1:2], yq, L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride,
                                                   L.pad, acc, part_buf)
                        else:
                            B.fpq_gemm_codes_out(buf, 0, FX, 0.0, s.scale[1:2], s.packed[tag], fw, s.sw[tag], None, FX, 0.0,
                                                 sy[L.name, tag][1:2], yq, L.M, L.N, L.K, acc, part_buf)
            run()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                run()
            graph.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                graph.replay()
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1) / 3
        c_ms = codes_to_codes()
        out["codes_to_codes_step"] = {"ms_per_step": round(c_ms, 4), "value": round(g_fl / (c_ms * 1e-3) / 1e12, 2),
                                      "unit": "TFLOP/s", "frac_of_bf16_peak": round(g_fl / (c_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                                      "note": "all layers, codes in, E4M3 codes out with static scales, one launch per layer"}
        # the other accumulate mode, same step
        other = B.FPQ_ACC_FP8_MFMA if acc == B.FPQ_ACC_FP32 else B.FPQ_ACC_FP32
        sec_o = timed(other, max(2, args.steps // 2), 1)
        o_ms, o_fl, o_n, _ = gemm_breakdown(other, reps=3)
        peak_o = PEAK_FP8_TFLOPS if other == B.FPQ_ACC_FP8_MFMA else PEAK_BF16_TFLOPS
        out["other_acc_mode"] = {"acc_mode": "fp8mfma" if other == B.FPQ_ACC_FP8_MFMA else "fp32",
                                 "value": round(flops_step / sec_o / 1e12, 3), "unit": "TFLOP/s",
                                 "gemm_achieved": round(o_fl / (o_ms * 1e-3) / 1e12, 2), "peak": peak_o,
                                 "frac": round(o_fl / (o_ms * 1e-3) / 1e12 / peak_o, 4)}
        # single layers, layer kernel alone on prepared codes (16 launches in one graph), both accumulate modes:
        # configurations 2 and 4, and from configuration 5 a deep-K conv and an output-bound linear layer
        singles = {}
        picks = [("cfg2_conv_320_64x64_b1", synth.config_layers(2)[0]), ("cfg4_conv_1280_16x16_b8", synth.config_layers(4)[0]),
                 ("cfg5_conv_1280_32x32_b8", synth.conv("c", 8, 1280, 32, 32, 1280, 3, 1)),
                 ("cfg5_linear_32768x320x2560", synth.linear("l", 32768, 320, 2560))]
        for cname, L in picks:
            if L.kind == "conv":
                xs = synth.activations_torch((L.B, L.Cin, L.H, L.W), 1, dev)
                wshape, kk = (L.Cout, L.Cin, L.k, L.k), L.k
                cb = torch.empty(L.B * L.H * L.W * B.fpq_padded_channels(L.Cin), dtype=torch.uint8, device=dev)
                wsz = B.fpq_conv2d_workspace_size(L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, 0)
            else:
                xs = synth.activations_torch((L.M, L.K), 1, dev)
                wshape, kk = (L.N, L.K), 1
                cb = torch.empty(L.M * L.K, dtype=torch.uint8, device=dev)
                wsz = B.fpq_gemm_workspace_size(L.M, L.N, L.K, 0)
            w = synth.weights_torch(wshape, 2, dev)
            st2 = torch.empty(2, dtype=torch.float32, device=dev)
            B.fpq_absmax(xs, FX[3], st2[0:1], st2[1:2], amax_ws)
            if L.kind == "conv":
                B.fpq_quantize_nhwc(xs, FX, 0.0, st2[1:2], cb)
            else:
                B.fpq_quantize(xs, FX, 0.0, st2[1:2], cb)
            yb = torch.empty(L.M * L.N, dtype=torch.float32, device=dev)
            yq = torch.empty(L.M * B.fpq_padded_channels(L.N), dtype=torch.uint8, device=dev)
            wsb = torch.empty(max(256, wsz), dtype=torch.uint8, device=dev)
            entry = {}
            for tag, fw in (("w8a8", FW8), ("w4a8", FW4)):
                pk = torch.empty(B.fpq_packed_size(L.N, L.Cin, kk, kk, fw), dtype=torch.uint8, device=dev)
                sw = torch.empty(L.N, dtype=torch.float32, device=dev)
                B.fpq_pack_weights(w, fw, None, None, pk, sw, None)
                for mname, mode, q in (("fp32", B.FPQ_ACC_FP32, False), ("fp8mfma", B.FPQ_ACC_FP8_MFMA, False),
                                       ("fp32_codes_out", B.FPQ_ACC_FP32, True), ("fp8mfma_codes_out", B.FPQ_ACC_FP8_MFMA, True)):
                    def one():
                        if q and L.kind == "conv":      # result quantized for the next layer (E4M3, static scale) in the epilogue
                            B.fpq_conv2d_codes_out(cb, 0, FX, 0.0, st2[1:2], pk, fw, sw, None, FX, 0.05, None, yq, L.B, L.Cin,
                                                   L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, mode, wsb)
                        elif q:
                            B.fpq_gemm_codes_out(cb, 0, FX, 0.0, st2[1:2], pk, fw, sw, None, FX, 0.05, None, yq, L.M, L.N, L.K,
                                                 mode, wsb)
                        elif L.kind == "conv":
                            B.fpq_conv2d(cb, 0, FX, 0.0, st2[1:2], pk, fw, sw, None, yb, L.B, L.Cin, L.H, L.W, L.Cout, L.k,
                                         L.k, L.stride, L.pad, mode, wsb)
                        else:
                            B.fpq_gemm(cb, 0, FX, 0.0, st2[1:2], pk, fw, sw, None, yb, L.M, L.N, L.K, mode, wsb)
                    one()
                    torch.cuda.synchronize()
                    g1 = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g1):
                        for _ in range(16):
                            one()
                    g1.replay()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(4):
                        g1.replay()
                    e1.record()
                    e1.synchronize()
                    us = e0.elapsed_time(e1) * 1e3 / 64
                    entry["%s_%s" % (tag, mname)] = {"us": round(us, 2), "TFLOP/s": round(synth.flops(L) / us / 1e6, 1)}
                if L.kind == "linear":
                    # the feed-forward projection as the U-Net runs it: gated GELU between the result and its codes
                    def gated():
                        B.fpq_gemm_codes_out(cb, 0, FX, 0.0, st2[1:2], pk, fw, sw, None, FX, 0.05, None, yq, L.M, L.N, L.K,
                                             B.FPQ_ACC_FP32 | B.FPQ_ACT_GEGLU, wsb)
                    gated()
                    torch.cuda.synchronize()
                    g3 = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g3):
                        for _ in range(16):
                            gated()
                    g3.replay()
                    e0.record()
                    for _ in range(4):
                        g3.replay()
                    e1.record()
                    e1.synchronize()
                    us = e0.elapsed_time(e1) * 1e3 / 64
                    entry["%s_fp32_geglu_codes_out" % tag] = {"us": round(us, 2), "TFLOP/s": round(synth.flops(L) / us / 1e6, 1)}
                if L.kind == "linear" and tag == "w8a8":
                    # what the codes-out form replaces when the next layer is quantized too: the fp32 result written,
                    # then read again by the next layer's quantize pass (static scale)
                    def two():
                        B.fpq_gemm(cb, 0, FX, 0.0, st2[1:2], pk, fw, sw, None, yb, L.M, L.N, L.K, B.FPQ_ACC_FP32, wsb)
                        B.fpq_quantize(yb, FX, 0.05, None, yq)
                    two()
                    torch.cuda.synchronize()
                    g2 = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g2):
                        for _ in range(16):
                            two()
                    g2.replay()
                    e0.record()
                    for _ in range(4):
                        g2.replay()
                    e1.record()
                    e1.synchronize()
                    entry["w8a8_fp32_then_quantize_us"] = round(e0.elapsed_time(e1) * 1e3 / 64, 2)
            singles[cname] = entry
            del xs, w, cb, yb, yq, wsb
        out["single_layers"] = singles
        roofline["measured_peak"] = measure_peaks()
        roofline["frac_of_measured_peak"] = round(achieved / roofline["measured_peak"][
            "bf16_mfma_TFLOP/s" if acc == B.FPQ_ACC_FP32 else "fp8_mfma_TFLOP/s"], 4)
        # structured-sparse weight operand (2 of every 4 input channels kept): the configuration-4 convolution and a
        # 1280-wide linear layer, E2M1 weights, layer kernel alone on prepared codes, next to the dense call on the same
        # shape; TFLOP/s count the dense layer's 2MNK
        sp = {}
        for cname, L in (("cfg4_conv_1280_16x16_b8", synth.config_layers(4)[0]), ("linear_2048x1280x1280", synth.linear("l", 2048, 1280, 1280))):
            if L.kind == "conv":
                xs = synth.activations_torch((L.B, L.Cin, L.H, L.W), 1, dev)
                wshape, kk = (L.Cout, L.Cin, L.k, L.k), L.k
                cb = torch.empty(L.B * L.H * L.W * B.fpq_padded_channels(L.Cin), dtype=torch.uint8, device=dev)
                wsz = B.fpq_conv2d_workspace_size(L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k, L.stride, L.pad, 0)
            else:
                xs = synth.activations_torch((L.M, L.K), 1, dev)
                wshape, kk = (L.N, L.K), 1
                cb = torch.empty(L.M * L.K, dtype=torch.uint8, device=dev)
                wsz = B.fpq_gemm_workspace_size(L.M, L.N, L.K, 0)
            w = synth.weights_torch(wshape, 2, dev)
            st2 = torch.empty(2, dtype=torch.float32, device=dev)
            B.fpq_absmax(xs, FX[3], st2[0:1], st2[1:2], amax_ws)
            if L.kind == "conv":
                B.fpq_quantize_nhwc(xs, FX, 0.0, st2[1:2], cb)
            else:
                B.fpq_quantize(xs, FX, 0.0, st2[1:2], cb)
            yb = torch.empty(L.M * L.N, dtype=torch.float32, device=dev)
            wsb = torch.empty(max(256, wsz), dtype=torch.uint8, device=dev)
            pk = torch.empty(B.fpq_packed_size(L.N, L.Cin, kk, kk, FW4), dtype=torch.uint8, device=dev)
            pks = torch.empty(B.fpq_packed_sparse_size(L.N, L.Cin, kk, kk, FW4), dtype=torch.uint8, device=dev)
            sw = torch.empty(L.N, dtype=torch.float32, device=dev)
            dropped = torch.zeros(1, dtype=torch.int64, device=dev)
            B.fpq_pack_weights(w, FW4, None, None, pk, sw, None)
            B.fpq_pack_weights_sparse(w, FW4, None, None, pks, sw, None, dropped)

            def dense():
                if L.kind == "conv":
                    B.fpq_conv2d(cb, 0, FX, 0.0, st2[1:2], pk, FW4, sw, None, yb, L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k,
                                 L.stride, L.pad, B.FPQ_ACC_FP32, wsb)
                else:
                    B.fpq_gemm(cb, 0, FX, 0.0, st2[1:2], pk, FW4, sw, None, yb, L.M, L.N, L.K, B.FPQ_ACC_FP32, wsb)

            def sparse():
                if L.kind == "conv":
                    B.fpq_conv2d_sparse(cb, 0, FX, 0.0, st2[1:2], pks, FW4, sw, None, yb, L.B, L.Cin, L.H, L.W, L.Cout, L.k, L.k,
                                        L.stride, L.pad, wsb)
                else:
                    B.fpq_gemm_sparse(cb, 0, FX, 0.0, st2[1:2], pks, FW4, sw, None, yb, L.M, L.N, L.K, wsb)
            ent = {}
            for name, fn in (("dense", dense), ("sparse", sparse)):
                fn()
                torch.cuda.synchronize()
                gs = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gs):
                    for _ in range(16):
                        fn()
                gs.replay()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(4):
                    gs.replay()
                e1.record()
                e1.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 64
                ent[name] = {"us": round(us, 2), "TFLOP/s_of_2MNK": round(synth.flops(L) / us / 1e6, 1)}
            groups4 = L.N * kk * kk * ((L.Cin + 3) // 4)
            ent["weight_bytes_dense"] = pk.numel()
            ent["weight_bytes_sparse"] = pks.numel()
            ent["groups_that_lost_a_nonzero"] = round(int(dropped.item()) / groups4, 4)
            sp[cname] = ent
            del xs, w, cb, yb, wsb, pk, pks
        out["sparse_weights_e2m1"] = sp
        # the same-bitwidth integer baseline of Eq. (4) on two linear layers of the set (integer matrix instruction, exact
        # sums; peak 5.0 POP/s), next to the floating-point layer on the same shapes: layer kernel alone on prepared codes
        ib = {}
        for cname, (iM, iK, iN) in (("linear_2048x1280x10240", (2048, 1280, 10240)), ("linear_32768x320x2560", (32768, 320, 2560))):
            xs = synth.activations_torch((iM, iK), 1, dev)
            w = synth.weights_torch((iN, iK), 2, dev)
            ipar = torch.zeros(16, dtype=torch.uint8, device=dev)
            iws = torch.empty(8192, dtype=torch.uint8, device=dev)
            B.fpq_int_calibrate(xs, 8, ipar, iws)
            xc = torch.empty(iM * iK, dtype=torch.uint8, device=dev)
            B.fpq_int_quantize(xs, 8, 0.0, 0, ipar, xc)
            yb = torch.empty(iM * iN, dtype=torch.float32, device=dev)
            gws = torch.empty(max(256, B.fpq_int_gemm_workspace_size(iM)), dtype=torch.uint8, device=dev)
            ent = {}
            for wbits in (8, 4):
                ipk = torch.empty(B.fpq_int_packed_size(iN, iK, wbits), dtype=torch.uint8, device=dev)
                isw = torch.empty(iN, dtype=torch.float32, device=dev)
                izw = torch.empty(iN, dtype=torch.int32, device=dev)
                B.fpq_int_pack_weights(w, wbits, ipk, isw, izw, None)

                def ione():
                    B.fpq_int_gemm(xc, 0.0, 0, ipar, ipk, wbits, isw, izw, None, yb, iM, iN, iK, gws)
                ione()
                torch.cuda.synchronize()
                gi = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gi):
                    for _ in range(16):
                        ione()
                gi.replay()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(4):
                    gi.replay()
                e1.record()
                e1.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 64
                tops = 2.0 * iM * iN * iK / us / 1e6
                ent["w%da8" % wbits] = {"us": round(us, 2), "TOP/s": round(tops, 1), "frac_of_int8_peak": round(tops / 5000.0, 4)}
            ib[cname] = ent
            del xs, w, xc, yb
        out["integer_baseline"] = ib
        # encoding / bias search of Section V-A on one activation tensor (8 x 320 x 64 x 64): 4 FP8 encodings x 111
        # bias candidates; bound by vector ALU work: 11 vector instructions per element and candidate (SEARCH_OPS) against the lane-instruction rate of the chip
        xs = synth.activations_torch((8, 320, 64, 64), 3, dev).reshape(-1)
        encs = [(2, 5), (3, 4), (4, 3), (5, 2)]
        s_mse = torch.empty(4 * 111, dtype=torch.float32, device=dev)
        s_res = torch.zeros(40, dtype=torch.uint8, device=dev)
        s_ws = torch.empty(B.fpq_search_workspace_size(xs.numel(), 4, 111), dtype=torch.uint8, device=dev)
        B.fpq_search_format(xs, encs, 111, s_mse, s_res, s_ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            B.fpq_search_format(xs, encs, 111, s_mse, s_res, s_ws)
        e1.record()
        e1.synchronize()
        s_ms = e0.elapsed_time(e1) / 5
        r = B.search_result(s_res)
        evals = xs.numel() * 444 / (s_ms * 1e-3)
        out["format_search"] = {"elements": xs.numel(), "candidates": 444, "ms": round(s_ms, 3),
                                "Gevals/s": round(evals / 1e9, 1), "alu_peak_Gevals/s": round(ALU_LANE_RATE / SEARCH_OPS / 1e9, 1),
                                "frac": round(evals / (ALU_LANE_RATE / SEARCH_OPS), 4),
                                "chosen": "E%dM%d, max value %.4g (bias %.3f), mse %.3e" % (r.ebits, r.mbits, r.maxval,
                                                                                          r.real_bias, r.mse)}
        del xs
        # activation-quantize bandwidth: 64 Mi elements per launch, rotating over 8 buffers (2.7 GB) so that the
        # last-level cache cannot serve the reads; algorithmic bytes = 5 per element (4 read + 1 written)
        n = 64 << 20
        bufs = [torch.randn(n, device=dev) for _ in range(8)]
        codes = [torch.empty(n, dtype=torch.uint8, device=dev) for _ in range(2)]
        sc = torch.tensor([0.01], device=dev)
        for i in range(4):
            B.fpq_quantize(bufs[i], FX, 0.0, sc, codes[i & 1])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        reps = 32
        for i in range(reps):
            B.fpq_quantize(bufs[i & 7], FX, 0.0, sc, codes[i & 1])
        e1.record()
        e1.synchronize()
        q_gbs = 5.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        am = torch.empty(2, device=dev)
        e0.record()
        for i in range(reps):
            B.fpq_absmax(bufs[i & 7], 448.0, am[0:1], am[1:2], amax_ws)
        e1.record()
        e1.synchronize()
        a_gbs = 4.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        out["quantize"] = {"elements": n, "GB/s": round(q_gbs, 1), "frac_of_hbm_peak": round(q_gbs / PEAK_HBM_GBS, 4),
                           "absmax_GB/s": round(a_gbs, 1), "absmax_frac": round(a_gbs / PEAK_HBM_GBS, 4)}
        # zero count (sparsity) on the code buffers of 64 Mi elements: one read, 1 B per element; the fp32 form on
        # the rotating fp32 buffers, 4 B per element
        zc = torch.zeros(1, dtype=torch.int64, device=dev)
        zws = torch.empty(B.fpq_count_zeros_workspace_size(n), dtype=torch.uint8, device=dev)
        cbig = [torch.randint(0, 256, (4 * n,), dtype=torch.uint8, device=dev) for _ in range(4)]   # 256 MiB each
        B.fpq_count_zeros(cbig[0], B.FPQ_X_CODES, 4 * n, FX, zc, zws)
        e0.record()
        for i in range(reps):
            B.fpq_count_zeros(cbig[i & 3], B.FPQ_X_CODES, 4 * n, FX, zc, zws)
        e1.record()
        e1.synchronize()
        zc_gbs = 4.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        e0.record()
        for i in range(reps):
            B.fpq_count_zeros(bufs[i & 7], B.FPQ_X_FP32, n, None, zc, zws)
        e1.record()
        e1.synchronize()
        zf_gbs = 4.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        out["zero_count"] = {"code_bytes": 4 * n, "codes_GB/s": round(zc_gbs, 1), "codes_frac": round(zc_gbs / PEAK_HBM_GBS, 4),
                             "fp32_GB/s": round(zf_gbs, 1), "fp32_frac": round(zf_gbs / PEAK_HBM_GBS, 4)}
        del bufs, codes, cbig
        # one step of rounding learning (Section V-B) on a 1280 x 1280 linear layer with 8192 calibration rows, E2M1
        # weights: two fp32 contractions of 2 M N K flops each, on the fp32 matrix instruction (peak 157.3 TFLOP/s)
        rN, rK, rM = 1280, 1280, 8192
        rw = synth.weights_torch((rN, rK), 5, dev)
        rsw = (rw.abs().amax(dim=1) / FW4[3]).contiguous()
        ra = synth.activations_torch((rM, rK), 6, dev)
        ral = torch.empty((rN, rK), device=dev)
        B.fpq_rl_init_alpha(rw, rsw, FW4, ral)
        rloss = torch.zeros(2, device=dev)
        rws = torch.empty(B.fpq_rl_workspace_size(rM, rN, rK), dtype=torch.uint8, device=dev)
        for _ in range(3):
            B.fpq_rl_step(rw, rsw, FW4, ral, ra, 1000.0, 0.01, rloss, None, rws)
        e0.record()
        for _ in range(20):
            B.fpq_rl_step(rw, rsw, FW4, ral, ra, 1000.0, 0.01, rloss, None, rws)
        e1.record()
        e1.synchronize()
        r_ms = e0.elapsed_time(e1) / 20
        r_tf = 4.0 * rM * rN * rK / (r_ms * 1e-3) / 1e12
        out["rounding_learning_step"] = {"N": rN, "K": rK, "M": rM, "ms": round(r_ms, 3), "TFLOP/s": round(r_tf, 1),
                                         "peak_fp32_mfma": 157.3, "frac": round(r_tf / 157.3, 4),
                                         "mse_and_regulariser_after_23_steps": ["%.4e" % float(v) for v in rloss.cpu().tolist()]}
        del rw, ra, ral, rws

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample of the same kind of work (~370 GFLOP, about 10 s on 16 cores), W8A8, through the oracle as it stands, on the host cores
        t_cpu, fl_cpu = 0.0, 0.0
        for (shape, wshape, npix) in (((1, 320, 64, 64), (320, 320, 3, 3), None), ((8, 1280, 16, 16), (1280, 1280, 3, 3), None),
                                      ((8, 640, 32, 32), (640, 640, 3, 3), None), ((8, 1280, 32, 32), (1280, 1280, 3, 3), None)):
            x = synth.activations(shape, 2000)
            w = synth.weights(wshape, 2500)
            t0 = time.perf_counter()
            sx = oracle.scale_from_absmax(oracle.absmax(x), FX[3])
            xq = oracle.quantize(x, FX, sx)
            wq, sw = oracle.pack_weights(w, FW8)
            M = shape[0] * shape[2] * shape[3]
            pix = None if npix is None else np.arange(0, M, M // npix)
            oracle.conv2d(xq, FX, sx, wq, FW8, sw, stride=1, pad=1, pix=pix)
            t_cpu += time.perf_counter() - t0
            fl_cpu += 2.0 * (M if pix is None else len(pix)) * wshape[0] * wshape[1] * 9
        if "format_search" in out:
            xs_h = synth.activations((1 << 20,), 3)
            t0 = time.perf_counter()
            oracle.search(xs_h, [(2, 5), (3, 4), (4, 3), (5, 2)], 111)
            t_s = time.perf_counter() - t0
            out["format_search"]["oracle_Gevals/s"] = round((1 << 20) * 444 / t_s / 1e9, 4)
            out["format_search"]["oracle_sample"] = "2^20 elements x 444 candidates on %d host cores, %.1f s" % (
                oracle.num_threads(), t_s)
        out["cpu_baseline"] = {"value": round(fl_cpu / t_cpu / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": "oracle absmax + quantize + pack + conv2d, W8A8: the config-2 and config-4 convs in "
                                         "full and a 640-channel and a 1280-channel 32x32 conv of config 5 "
                                         "(%.1f GFLOP, %.1f s)" % (fl_cpu / 1e9, t_cpu)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
