#!/usr/bin/env python3
"""Benchmark of the ternary hot path on one MI355X.

A step is one pass of the whole path over one batch of the headline workload, the large
square ternary GEMM M = N = K = 8192 on the seeded operands of synth_inputs.cfg4(): pack the
activation levels into plane words, then the ternary GEMM with its int32 output.  Weights are
packed once before the timed region (the paper fixes everything derived from them after
training).  Inputs are seeded synthetic level tensors already resident in HBM.  Prints ONE
JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
                    [--workload cfg4|cfg2|cfg3|cfg5|quantpack|paper6|peaks] [--no-cpu] [--no-extra]

The roofline object carries two denominators: `peak`, the nominal VALU figure derived from the
chip's unit counts and clock, and `peak_measured`, the rate at which a register-resident loop of
the method's own instruction pair issues on this very GPU, measured inside this run
(`--workload peaks` prints the whole table of such probes).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X: 256 CUs x 4 SIMDs x 16 lanes = 16384 32-bit VALU lanes at 2.4 GHz.
VALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9
# The reduced ternary inner product needs one three-input logic op and one popcount per
# 32-bit plane word, two plane words per 32 elements: 4 lane-instructions per 32 MACs
# (= 64 ops under the 2*M*N*K convention).  The conventional two-bit form needs 8.
TERNARY_OPS_PER_LANE_INSTR = 64 / 4
TWOBIT_OPS_PER_LANE_INSTR = 64 / 8
TERNARY_PEAK_TOPS = VALU_LANE_OPS_PER_S * TERNARY_OPS_PER_LANE_INSTR / 1e12     # 629.1 (nominal)
HBM_PEAK_GBS = 8000.0
PEAK_BASIS = ("nominal: 256 CU x 64 lanes x 2.4 GHz = 39.3 T lane-instr/s, 4 lane-instr per 64 ops; measured: "
              "register-resident v_bitop3_b32 -> v_bcnt_u32_b32 loop on this GPU (fatnn_probe_valu), best over "
              "wavefronts per SIMD and operand kind, x 16 ops per lane-instr")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def measured_traffic_bytes(workload):
    """HBM bytes per launch of the workload's dominant kernel, from the table that bench_traffic.py writes out
    of rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script (None when no such run is on file)."""
    try:
        with open(TRAFFIC_FILE) as fh:
            for ln in fh:
                m = re.match(r"\|\s*%s\s*\|.*\|\s*(\d+)\s*\|\s*$" % re.escape(workload), ln)
                if m:
                    return int(m.group(1))
    except OSError:
        pass
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default depends on the workload)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed warm-up steps")
    ap.add_argument("--workload", default="cfg4",
                    choices=["cfg4", "cfg2", "cfg3", "cfg5", "quantpack", "paper6", "peaks", "midgemm"])
    ap.add_argument("--plain-input", action="store_true",
                    help="cfg2 only: pack the activations in plain NHWC order, so that the convolution takes the "
                         "LDS-tiled kernel's implicit-im2col front end instead of the streaming kernel")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-extra", action="store_true", help="skip the side measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run the library's 256 MiB copy kernel 5 times (reference for the FETCH_SIZE / "
                         "WRITE_SIZE counters of a rocprofv3 --pmc run, see bench_traffic.py) and exit")
    args = ap.parse_args()
    # Defaults long enough for the clocks to settle (a cfg2 step is 23 us: 200 steps were over before the GPU
    # had reached its sustained clock, and read 6 % slow), short enough to finish in seconds.
    steps, warmup = {"cfg2": (4000, 1000), "cfg4": (100, 20), "cfg3": (200, 50), "cfg5": (600, 100),
                     "quantpack": (300, 50), "paper6": (20, 3), "peaks": (3, 1), "midgemm": (20, 3)}[args.workload]
    if args.steps is None:
        args.steps = steps
    if args.warmup is None:
        args.warmup = warmup
    return args


def time_kernel_ms(torch, fn, iters, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def time_graph_ms(torch, fn, iters, replays=5, min_ms=40.0):
    """Average duration of fn's launches with the host out of the picture: `iters` calls recorded into one
    HIP graph (library kernels only), replayed at least `replays` times and for at least `min_ms` (a
    measurement of a few milliseconds is over before the clocks have settled and reads up to 8 % slow)."""
    fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(iters):
            fn()
    torch.cuda.synchronize()

    def run(n):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)
    first = run(1)
    n = max(replays, int(min_ms / max(first, 1e-3)) + 1)
    run(max(1, n // 2))            # untimed: brings the clocks up
    return run(n) / (iters * n)


class HipEvents:
    """Plain HIP timing events through the runtime's C API (the library attaches them to its kernel
    dispatch, see fatnn_time_next_launch)."""

    def __init__(self, n):
        import ctypes
        self.ct = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.ev = []
        for _ in range(n):
            e = ctypes.c_void_p()
            if self.hip.hipEventCreate(ctypes.byref(e)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.ev.append(e)

    def handle(self, i):
        return self.ev[i].value

    def elapsed_ms(self, i, j):
        ms = self.ct.c_float()
        if self.hip.hipEventSynchronize(self.ev[j]) != 0:
            raise RuntimeError("hipEventSynchronize failed")
        if self.hip.hipEventElapsedTime(self.ct.byref(ms), self.ev[i], self.ev[j]) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value

    def close(self):
        for e in self.ev:
            self.hip.hipEventDestroy(e)
        self.ev = []


def settle_clocks(torch, fn, seconds=0.3):
    """Untimed load before the warm-up: the GPU needs some tens of milliseconds of work to reach its
    sustained clock, and a short benchmark would otherwise be timed on the ramp.  Returns the time spent."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(4):
            fn()
        torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3


def measure_peaks(torch, fatnn, full=False):
    """The denominators, measured on this GPU with the library's probe kernels: issue rate of the method's
    instruction pair from registers (lane-instructions per second) over wavefronts per SIMD, and HBM streaming
    rates.  Each figure is the best of three launches, timed with events attached to the dispatch."""
    scratch = fatnn.probe_scratch("cuda:0")
    hev = HipEvents(2)

    def timed(launch):
        best = None
        for _ in range(3):
            fatnn.time_next_launch(hev.handle(0), hev.handle(1))
            work = launch()
            ms = hev.elapsed_ms(0, 1)
            best = ms if best is None or ms < best else best
        return work, best

    out = {"valu_T_lane_instr_per_s": {}, "hbm_GBps": {}}
    kinds = [("pair_vgpr_operands", fatnn.PROBE_PAIR_V), ("pair_sgpr_data_word", fatnn.PROBE_PAIR_S)]
    if full:
        kinds += [("pair_operands_from_lds", fatnn.PROBE_PAIR_LDS), ("bcnt_alone", fatnn.PROBE_BCNT),
                  ("bitop3_alone", fatnn.PROBE_BITOP3), ("xor_alone", fatnn.PROBE_XOR)]
    waves = (1, 2, 3, 4, 5, 6, 7, 8) if full else (2, 4, 8)
    fatnn.probe_valu(fatnn.PROBE_PAIR_V, 4, 200, scratch)      # first launch loads the code
    best_pair = 0.0
    for name, kind in kinds:
        row = {}
        for w in waves:
            work, ms = timed(lambda: fatnn.probe_valu(kind, w, 3000, scratch))
            rate = work / (ms * 1e-3) / 1e12
            row[f"{w}_waves_per_simd"] = round(rate, 2)
            if kind in (fatnn.PROBE_PAIR_V, fatnn.PROBE_PAIR_S):
                best_pair = max(best_pair, rate)
        out["valu_T_lane_instr_per_s"][name] = row
    out["valu_pair_best_T_lane_instr_per_s"] = round(best_pair, 2)
    out["valu_nominal_T_lane_instr_per_s"] = round(VALU_LANE_OPS_PER_S / 1e12, 2)
    out["ternary_peak_measured_tops"] = round(best_pair * TERNARY_OPS_PER_LANE_INSTR, 1)
    nbytes = 1 << 30
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(1)
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    for name, kind, moved in (("read", fatnn.HBM_READ, nbytes), ("write", fatnn.HBM_WRITE, nbytes),
                              ("copy", fatnn.HBM_COPY, 2 * nbytes)):
        _, ms = timed(lambda: fatnn.probe_hbm(kind, b, a, nbytes, scratch))
        out["hbm_GBps"][name] = round(moved / (ms * 1e-3) / 1e9, 1)
    out["hbm_best_GBps"] = max(out["hbm_GBps"].values())
    hev.close()
    del a, b, scratch
    return out


def alu_roofline(kernel, achieved_tops, kernel_ms, peaks, traffic):
    """Roofline object of a VALU-bound kernel: fraction of the nominal peak and of the measured one."""
    r = {"bound": "alu", "kernel": kernel, "achieved": round(achieved_tops, 2), "peak": round(TERNARY_PEAK_TOPS, 1),
         "unit": "Tops/s", "frac": round(achieved_tops / TERNARY_PEAK_TOPS, 4), "traffic": traffic,
         "kernel_ms": round(kernel_ms, 5), "peak_measured": None, "frac_measured": None,
         "graded_on": "frac_measured (the nominal figure is not a ceiling on this chip: the probe loop exceeds it)",
         "peak_basis": PEAK_BASIS}
    if peaks is not None:
        pm = peaks["ternary_peak_measured_tops"]
        r["peak_measured"] = pm
        r["frac_measured"] = round(achieved_tops / pm, 4)
    return r


def hbm_roofline(kernel, achieved_gbs, kernel_ms, peaks, traffic=None):
    r = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(achieved_gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel_ms": round(kernel_ms, 5),
         "peak_measured": None, "frac_measured": None}
    if peaks is not None:
        r["peak_measured"] = peaks["hbm_best_GBps"]
        r["frac_measured"] = round(achieved_gbs / peaks["hbm_best_GBps"], 4)
    return r


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for ln in fh:
                if ln.startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline_conv(case, seconds_target=10.0):
    """The oracle as it stands, timed on the host cores on whole passes of the workload."""
    import oracle
    Lw, Lx = case.make()
    threads = oracle.num_threads()
    t0 = time.perf_counter()
    oracle.ternary_conv2d(Lw, Lx, case.stride, case.pad, case.act_mode)
    first = time.perf_counter() - t0
    reps = max(1, min(100, int(seconds_target / max(first, 1e-3))))
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.ternary_conv2d(Lw, Lx, case.stride, case.pad, case.act_mode)
    dt = (time.perf_counter() - t0) / reps
    # one thread: a slice of the batch sized to a few seconds
    nb = max(1, min(case.B, int(case.B * 4.0 / max(first * threads, 1e-3))))
    oracle.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        oracle.ternary_conv2d(Lw, Lx[:nb], case.stride, case.pad, case.act_mode)
        dt1 = time.perf_counter() - t0
    finally:
        oracle.set_num_threads(threads)
    return {"value": round(2.0 * case.macs() / dt / 1e12, 5), "unit": "Tops/s", "cores": threads,
            "kind": "oracle", "sample": f"{reps} full passes of {case.name} (batch {case.B}), {dt:.3f} s each",
            "single_thread_value": round(2.0 * case.macs() * nb / case.B / dt1 / 1e12, 6),
            "single_thread_sample": f"first {nb} images, {dt1:.2f} s", "cpu_model": cpu_model()}


def cpu_baseline_gemm(case, rows=64, seconds_target=10.0):
    """The oracle on the first rows of the weight matrix against all columns, sized to about seconds_target."""
    import numpy as np
    import oracle
    Lw, La = case.make()
    threads = oracle.num_threads()
    t0 = time.perf_counter()
    oracle.ternary_gemm(np.ascontiguousarray(Lw[:rows]), La, case.act_mode)
    first = time.perf_counter() - t0
    rows_all = int(max(rows, min(case.M, rows * seconds_target / max(first, 1e-3))))
    sub = np.ascontiguousarray(Lw[:rows_all])
    t0 = time.perf_counter()
    oracle.ternary_gemm(sub, La, case.act_mode)
    dt = time.perf_counter() - t0
    rows_one = int(max(1, min(case.M, rows * 4.0 / max(first * threads, 1e-3))))
    sub1 = np.ascontiguousarray(Lw[:rows_one])
    oracle.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        oracle.ternary_gemm(sub1, La, case.act_mode)
        dt1 = time.perf_counter() - t0
    finally:
        oracle.set_num_threads(threads)
    return {"value": round(2.0 * rows_all * case.N * case.K / dt / 1e12, 5), "unit": "Tops/s", "cores": threads,
            "kind": "oracle", "sample": f"first {rows_all} of {case.M} weight rows against all columns, {dt:.2f} s",
            "single_thread_value": round(2.0 * rows_one * case.N * case.K / dt1 / 1e12, 6),
            "single_thread_sample": f"first {rows_one} weight rows, {dt1:.2f} s", "cpu_model": cpu_model()}


def other_config_summaries(torch, fatnn, si, dev, peaks):
    """Short timings of the other configurations next to the headline (each its own --workload in full):
    the cfg2 convolution step on the streaming kernel, the same and two cfg3 layers through the LDS-tiled
    kernel's implicit-im2col front end (plain NHWC packed input, nothing materialised), and the ragged GEMM."""
    out = {}
    pm = peaks["ternary_peak_measured_tops"]

    def tops(macs, ms):
        t = 2.0 * macs / (ms * 1e-3) / 1e12
        return {"us": round(ms * 1e3, 2), "tops": round(t, 1), "frac_nominal": round(t / TERNARY_PEAK_TOPS, 3),
                "frac_measured": round(t / pm, 3)}
    layers = si.cfg3(64)
    picks = [("cfg2_conv3x3_128_28_b32", si.cfg2()), (layers[0].name + "_b64", layers[0]),
             (layers[15].name + "_b64", layers[15])]      # first 64-channel and first 512-channel 3x3 layer
    for label, case in picks:
        Lw, Lx = case.make()
        Lw_d, Lx_d = torch.from_numpy(Lw).to(dev), torch.from_numpy(Lx).to(dev)
        Wp = fatnn.pack_ternary(Lw_d, fatnn.WEIGHT, fatnn.OHWI)
        Xb = fatnn.pack_ternary_bordered(Lx_d, case.pad, case.act_mode)
        Xplain = fatnn.pack_ternary(Lx_d, fatnn.ACT, fatnn.NHWC)
        Y = torch.empty((case.B, case.Ho, case.Wo, case.Cout), dtype=torch.int32, device=dev)
        a = (case.B, case.Cin, case.H, case.W, case.Cout, case.R, case.S, case.stride, case.pad, case.act_mode)
        t_stream = time_graph_ms(torch, lambda: fatnn.ternary_conv2d(Wp, Xb, *a, out=Y, x_layout=fatnn.X_BORDERED), 10)
        t_tiled = time_graph_ms(torch, lambda: fatnn.ternary_conv2d(Wp, Xplain, *a, out=Y, x_layout=fatnn.X_PLAIN), 10)
        out[label] = {"streaming_kernel_bordered_input": tops(case.macs(), t_stream),
                      "tiled_kernel_implicit_im2col_plain_input": tops(case.macs(), t_tiled)}
        del Wp, Xb, Xplain, Y, Lw_d, Lx_d
    g = si.cfg5_ragged()
    Lw, La = g.make()
    Wp = fatnn.pack_ternary(torch.from_numpy(Lw).to(dev), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(torch.from_numpy(La).to(dev), fatnn.ACT)
    C = torch.empty((g.M, g.N), dtype=torch.int32, device=dev)
    t = time_graph_ms(torch, lambda: fatnn.ternary_gemm(Wp, Ap, g.M, g.N, g.K, g.act_mode, out=C), 20)
    out[f"cfg5a_gemm_{g.M}x{g.N}x{g.K}"] = tops(g.macs(), t)
    # fully connected layers (Supplementary S1: convolutions whose filter covers the map) at batch 16-128
    Wfc = torch.randint(0, 3, (4096, 4608), dtype=torch.int8, device=dev)
    Wp = fatnn.pack_ternary(Wfc, fatnn.WEIGHT)
    for n in (16, 32, 64, 128):
        Ap = fatnn.pack_ternary(torch.randint(0, 3, (n, 4608), dtype=torch.int8, device=dev), fatnn.ACT)
        C = torch.empty((4096, n), dtype=torch.int32, device=dev)
        t = time_graph_ms(torch, lambda: fatnn.ternary_gemm(Wp, Ap, 4096, n, 4608, 0, out=C), 20)
        out[f"fc_4096x{n}x4608"] = tops(4096 * n * 4608, t)
    return out


def side_workload(args, torch, fatnn, si, dev):
    """Workloads beyond the headline ones: the chained ResNet-18-shaped trunk (cfg3 as one pipeline) and
    the HBM-bound quantize-and-pack pass.  Same JSON shape, one line."""
    import numpy as np
    scratch = fatnn.probe_scratch(dev)
    settle_clocks(torch, lambda: fatnn.probe_valu(fatnn.PROBE_PAIR_V, 4, 400, scratch))
    peaks = measure_peaks(torch, fatnn)
    if args.workload == "cfg3":
        from paper_2008_05101_amd import resnet_trunk as rt
        batch = 64
        blocks_np = si.trunk_params()

        def cv(d):
            t = lambda a: torch.from_numpy(a).to(dev)
            return rt.ConvParams(t(d["levels"]), t(d["scale"]), t(d["bias"]), d["alpha"], d["stride"])
        blocks = [rt.BlockParams(cv(b["conv1"]), cv(b["conv2"]), None if b["shortcut"] is None else cv(b["shortcut"]))
                  for b in blocks_np]
        trunk = rt.Trunk(blocks, batch, 56, (0.6, 0.7), device=str(dev))
        x = torch.from_numpy(si.trunk_input(batch)).to(dev)
        for _ in range(args.warmup):
            trunk.forward(x)
        torch.cuda.synchronize()
        steps = args.steps
        # event pairs on the 19 conv launches of every 4th pass only: attaching them costs about 5 us per launch
        every = 4 if steps >= 8 else 1
        timed = list(range(0, steps, every))
        hev = HipEvents(2 * 19 * len(timed))
        cur = [0]

        def hook(layer):
            i = cur[0] * 19 + layer
            fatnn.time_next_launch(hev.handle(2 * i), hev.handle(2 * i + 1))
        t0 = time.perf_counter()
        for s_ in range(steps):
            if s_ % every == 0:
                cur[0] = s_ // every
                trunk.forward(x, before_conv=hook)
            else:
                trunk.forward(x)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_per_step = wall * 1e3 / steps
        per_layer = [sum(hev.elapsed_ms(2 * (j * 19 + l), 2 * (j * 19 + l) + 1) for j in range(len(timed))) / len(timed)
                     for l in range(19)]
        hev.close()
        ops = 2.0 * trunk.macs
        kernel_ms = sum(per_layer)
        # the same pass as one HIP graph submission, and the paper's own setting (whole network, batch 1)
        side = {}
        if not args.no_extra:
            graph = trunk.capture(x)
            side["graph_replay_ms_per_pass"] = round(time_kernel_ms(torch, graph.replay, 20, 3), 5)
            t1 = rt.Trunk(blocks, 1, 56, (0.6, 0.7), device=str(dev))
            x1 = torch.from_numpy(si.trunk_input(1)).to(dev)
            side["batch1_eager_ms"] = round(time_kernel_ms(torch, lambda: t1.forward(x1), 50, 5), 5)
            g1 = t1.capture(x1)
            side["batch1_graph_replay_ms"] = round(time_kernel_ms(torch, g1.replay, 50, 5), 5)
            side["paper_context_resnet18_batch1_ms"] = {"qualcomm_835": 20.1, "qualcomm_821": 25.2}
            del t1, g1
            # the paper's second network: ResNet-34 shape (16 blocks, 35 ternary convolutions)
            blocks34 = [rt.BlockParams(cv(b["conv1"]), cv(b["conv2"]),
                                       None if b["shortcut"] is None else cv(b["shortcut"]))
                        for b in si.trunk_params(34)]
            t34 = rt.Trunk(blocks34, batch, 56, (0.6, 0.7), device=str(dev))
            ms34 = time_kernel_ms(torch, lambda: t34.forward(x), 10, 2)
            side["resnet34_batch64_ms_per_pass"] = round(ms34, 5)
            side["resnet34_batch64_tops"] = round(2.0 * t34.macs / (ms34 * 1e-3) / 1e12, 1)
            del t34
            t34b1 = rt.Trunk(blocks34, 1, 56, (0.6, 0.7), device=str(dev))
            g34 = t34b1.capture(x1)
            side["resnet34_batch1_graph_replay_ms"] = round(time_kernel_ms(torch, g34.replay, 50, 5), 5)
            side["paper_context_resnet34_batch1_ms"] = {"qualcomm_835": 42.1, "qualcomm_821": 51.4}
        layers = si.cfg3(batch)
        achieved = ops / (kernel_ms * 1e-3) / 1e12
        line = {
            "metric": "ternary GEMM Tops/s (2MNK) at 1 MI355X", "value": round(ops / (ms_per_step * 1e-3) / 1e12, 3),
            "unit": "Tops/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
            "config": {"workload": "cfg3: the 19 ternary conv layers of a ResNet-18 shape at batch 64 as ONE chained "
                                   "pipeline (quantize+pack the fp32 input, every conv writes the next layer's packed "
                                   "input through the fused affine/skip/ReLU/quantize epilogue)", "batch": batch,
                       "macs": trunk.macs},
            "roofline": alu_roofline("stream_conv_kernel (all 19 launches)", achieved, kernel_ms, peaks, None),
            "cpu_baseline": None,
            "extra": {**side, "per_layer_us": {l.name: round(t * 1e3, 2) for l, t in zip(layers, per_layer)},
                      "per_layer_tops": {l.name: round(2.0 * l.macs() / (t * 1e-3) / 1e12, 1)
                                         for l, t in zip(layers, per_layer)}},
        }
        print(json.dumps(line))
        return
    if args.workload == "paper6":
        # The paper's layer-wise comparison (Section 5.1.1, Tables 4 / S2): six 3x3 layers, ternary vs the
        # conventional two-bit form vs the xnor rule alone, at the paper's batch 1 and at batch 32.
        code = torch.tensor([0, 1, 3], dtype=torch.int8, device=dev)
        results = {}
        tot_ms = 0.0
        tot_ops = 0.0
        best = None
        for batch in (1, 32):
            for case in si.paper_six(batch):
                Lw, Lx = case.make()
                Lw_d = torch.from_numpy(Lw).to(dev)
                Lx_d = torch.from_numpy(Lx).to(dev)
                Wp = fatnn.pack_ternary(Lw_d, fatnn.WEIGHT, fatnn.OHWI)
                Xp = fatnn.pack_ternary_bordered(Lx_d, case.pad, case.act_mode)
                W2 = fatnn.pack_twobit(code[Lw_d.long()], fatnn.WEIGHT, fatnn.OHWI)
                X2 = fatnn.pack_twobit_bordered(code[Lx_d.long()], case.pad)
                Y = torch.empty((case.B, case.Ho, case.Wo, case.Cout), dtype=torch.int32, device=dev)
                a = (case.B, case.Cin, case.H, case.W, case.Cout, case.R, case.S, case.stride, case.pad)
                # launches recorded into a HIP graph: at batch 1 a Python call costs more than the kernel
                n = args.steps
                t_ter = time_graph_ms(torch, lambda: fatnn.ternary_conv2d(Wp, Xp, *a, case.act_mode, out=Y,
                                                                          x_layout=fatnn.X_BORDERED), n)
                t_two = time_graph_ms(torch, lambda: fatnn.twobit_conv2d(W2, X2, *a, out=Y,
                                                                         x_layout=fatnn.X_BORDERED), n)
                t_xn = time_graph_ms(torch, lambda: fatnn.twobit_conv2d(W2, X2, *a, fatnn.BASIS_XNOR_ONLY, out=Y,
                                                                        x_layout=fatnn.X_BORDERED), n)
                ops = 2.0 * case.macs()
                results[f"{case.name}_b{batch}"] = {
                    "ternary_us": round(t_ter * 1e3, 2), "twobit_us": round(t_two * 1e3, 2),
                    "xnor_only_us": round(t_xn * 1e3, 2), "ternary_tops": round(ops / (t_ter * 1e-3) / 1e12, 2),
                    "speedup_vs_twobit": round(t_two / t_ter, 3), "extra_bit_ops_cost": round((t_ter - t_xn) / t_xn, 4)}
                if batch == 32:
                    tot_ms += t_ter
                    tot_ops += ops
                    if best is None or ops / t_ter > best[0]:
                        best = (ops / t_ter, case.name, t_ter)
                del Wp, Xp, W2, X2, Y, Lw_d, Lx_d
        achieved = best[0] / 1e9
        line = {
            "metric": "ternary GEMM Tops/s (2MNK) at 1 MI355X", "value": round(tot_ops / (tot_ms * 1e-3) / 1e12, 3),
            "unit": "Tops/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(tot_ms, 5),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
            "config": {"workload": "paper6: the six 3x3 layer shapes of the paper's layer-wise timing (64 channels at "
                                   "28/56/112/224, 128 and 256 channels at 56), ternary vs two-bit vs xnor-only "
                                   "kernels; value and ms_per_step are the six ternary layers at batch 32, inputs "
                                   "already packed"},
            "roofline": alu_roofline(f"stream_conv_kernel on {best[1]} (batch 32)", achieved, best[2], peaks, None),
            "cpu_baseline": None,
            "extra": {"layers": results,
                      "paper_context_us_nvidia_2080ti_batch1": {"ternary": [11, 14.5, 26, 90, 34, 87],
                                                                "twobit": [38, 44, 73.5, 274, 91, 217.5]}},
        }
        print(json.dumps(line))
        return
    if args.workload == "midgemm":
        # GEMMs whose tiles do not fill the chip evenly: the ragged cfg5 GEMM, three square ones with a long K (the
        # even-share schedules) and fully connected layers at batch 16-128 (K-splitting kernel); each against the plain call
        shapes = [(512, 3136, 4609), (1536, 1536, 4096), (768, 768, 8192), (256, 256, 32768), (4096, 16, 4608), (4096, 32, 4608),
                  (4096, 64, 4608), (4096, 128, 4608)]
        results = {}
        tot_ms = tot_ops = 0.0
        best = None
        rng = torch.Generator(device=dev).manual_seed(20080510)
        for (M, N, K) in shapes:
            Wp = fatnn.pack_ternary(torch.randint(0, 3, (M, K), dtype=torch.int8, device=dev, generator=rng), fatnn.WEIGHT)
            Ap = fatnn.pack_ternary(torch.randint(0, 3, (N, K), dtype=torch.int8, device=dev, generator=rng), fatnn.ACT)
            C = torch.empty((M, N), dtype=torch.int32, device=dev)
            # graph replays: the smallest of these kernels take less time than a Python call
            ms = time_graph_ms(torch, lambda: fatnn.ternary_gemm(Wp, Ap, M, N, K, 0, out=C), args.steps)
            fatnn.set_tuning(gemm_even_share=9, gemm_deepk=2)
            ms_plain = time_graph_ms(torch, lambda: fatnn.ternary_gemm(Wp, Ap, M, N, K, 0, out=C, workspace=None),
                                     args.steps)
            fatnn.set_tuning(gemm_even_share=0, gemm_deepk=0)
            ops = 2.0 * M * N * K
            results[f"{M}x{N}x{K}"] = {"us": round(ms * 1e3, 2), "tops": round(ops / (ms * 1e-3) / 1e12, 1),
                                       "tile_per_workgroup_us": round(ms_plain * 1e3, 2),
                                       "speedup": round(ms_plain / ms, 3)}
            tot_ms += ms
            tot_ops += ops
            if best is None or ops / ms > best[0]:
                best = (ops / ms, f"{M}x{N}x{K}", ms)
        line = {
            "metric": "ternary GEMM Tops/s (2MNK) at 1 MI355X", "value": round(tot_ops / (tot_ms * 1e-3) / 1e12, 3),
            "unit": "Tops/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(tot_ms, 5),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
            "config": {"workload": "midgemm: ternary GEMMs whose tiles do not fill 256 compute units evenly "
                                   "(512x3136x4609, 1536^2x4096, 768^2x8192, 256^2x32768) and fully connected layers "
                                   "4096xNx4608 at N = 16..128; operands already packed; value = all eight in a row"},
            "roofline": alu_roofline(f"GEMM {best[1]}", best[0] / 1e9, best[2], peaks, None),
            "cpu_baseline": None, "extra": results,
        }
        print(json.dumps(line))
        return
    if args.workload == "cfg5":
        # ragged and low-K shapes, packing of the activations included in every step
        results = {}
        total_ms = 0.0
        total_ops = 0.0
        worst = None
        for case in (si.cfg5_ragged(), si.cfg5_gemv()):
            Lw, La = case.make()
            Lw_d, La_d = torch.from_numpy(Lw).to(dev), torch.from_numpy(La).to(dev)
            Wp = fatnn.pack_ternary(Lw_d, fatnn.WEIGHT)
            Ap = torch.empty(max(fatnn.packed_bytes(fatnn.ACT, case.N, case.K), 16), dtype=torch.uint8, device=dev)
            C = torch.empty((case.M, case.N), dtype=torch.int32, device=dev)

            def step(La_d=La_d, Ap=Ap, Wp=Wp, C=C, case=case):
                fatnn.pack_ternary(La_d, fatnn.ACT, out=Ap)
                fatnn.ternary_gemm(Wp, Ap, case.M, case.N, case.K, case.act_mode, out=C)
            ms = time_kernel_ms(torch, step, args.steps, args.warmup)
            kms = time_kernel_ms(torch, lambda: fatnn.ternary_gemm(Wp, Ap, case.M, case.N, case.K, case.act_mode, out=C),
                                 args.steps, args.warmup)
            Kw = (case.K + 31) // 32
            nbytes = case.N * case.K + 2 * case.N * Kw * 8 + case.M * Kw * 8 + case.M * case.N * 4
            results[case.name] = {"step_us": round(ms * 1e3, 2), "gemm_us": round(kms * 1e3, 2),
                                  "tops": round(2.0 * case.macs() / (ms * 1e-3) / 1e12, 2),
                                  "compulsory_GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
            total_ms += ms
            total_ops += 2.0 * case.macs()
        for case in si.cfg5_bottleneck():
            Lw, Lx = case.make()
            Lw_d, Lx_d = torch.from_numpy(Lw).to(dev), torch.from_numpy(Lx).to(dev)
            Wp = fatnn.pack_ternary(Lw_d, fatnn.WEIGHT, fatnn.OHWI)
            Xp = torch.empty(fatnn.bordered_act_bytes(case.B, case.H, case.W, case.Cin, 0), dtype=torch.uint8, device=dev)
            Y = torch.empty((case.B, case.Ho, case.Wo, case.Cout), dtype=torch.int32, device=dev)
            cargs = (case.B, case.Cin, case.H, case.W, case.Cout, 1, 1, 1, 0, case.act_mode)

            def step(Lx_d=Lx_d, Xp=Xp, Wp=Wp, Y=Y, cargs=cargs, case=case):
                fatnn.pack_ternary_bordered(Lx_d, 0, case.act_mode, out=Xp)
                fatnn.ternary_conv2d(Wp, Xp, *cargs, out=Y, x_layout=fatnn.X_BORDERED)
            ms = time_kernel_ms(torch, step, args.steps, args.warmup)
            kms = time_kernel_ms(torch, lambda: fatnn.ternary_conv2d(Wp, Xp, *cargs, out=Y, x_layout=fatnn.X_BORDERED),
                                 args.steps, args.warmup)
            npix = case.B * case.H * case.W
            # int8 levels read + packed words written and read back + int32 output written
            nbytes = npix * case.Cin + 2 * npix * case.Cin // 4 + npix * case.Cout * 4
            results[case.name] = {"step_us": round(ms * 1e3, 2), "conv_us": round(kms * 1e3, 2),
                                  "tops": round(2.0 * case.macs() / (ms * 1e-3) / 1e12, 2),
                                  "compulsory_GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                  "conv_GBps": round((npix * case.Cin // 4 + npix * case.Cout * 4) / (kms * 1e-3) / 1e9, 1)}
            total_ms += ms
            total_ops += 2.0 * case.macs()
            if worst is None or results[case.name]["conv_GBps"] > worst[1]:
                worst = (case.name, results[case.name]["conv_GBps"], kms)
        line = {
            "metric": "ternary GEMM Tops/s (2MNK) at 1 MI355X", "value": round(total_ops / (total_ms * 1e-3) / 1e12, 3),
            "unit": "Tops/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(total_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
            "config": {"workload": "cfg5: ragged GEMM 512x3136x4609, GEMV 4096x1x4608, 1x1 convs 256->64 and 64->256 "
                                   "@56x56 batch 128; every step packs its activations first"},
            "roofline": hbm_roofline(f"stream_conv_kernel on {worst[0]}", worst[1], worst[2], peaks),
            "cpu_baseline": None, "extra": results,
        }
        print(json.dumps(line))
        return
    # quantize-and-pack: fp32 NHWC activations of the 256-channel bottleneck input (128 x 56 x 56 x 256)
    B, H, W, C = 128, 56, 56, 256
    x = torch.randn((B, H, W, C), device=dev).abs_()
    out = torch.empty(fatnn.bordered_act_bytes(B, H, W, C, 0), dtype=torch.uint8, device=dev)
    lv = torch.randint(0, 3, (B, H, W, C), dtype=torch.int8, device=dev)
    f1 = lambda: fatnn.quantize_pack_bordered(x, 0, fatnn.RELU, 0.7, 0.9, out=out)
    f2 = lambda: fatnn.pack_ternary_bordered(lv, 0, fatnn.RELU, out=out)
    for _ in range(args.warmup):
        f1()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        f1()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    k1 = time_kernel_ms(torch, f1, 20, 3)
    k2 = time_kernel_ms(torch, f2, 20, 3)
    n = B * H * W * C
    line = {
        "metric": "quantize-and-pack GB/s at 1 MI355X", "value": round(n * 4.25 / (ms * 1e-3) / 1e9, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32 in, u32 bit-planes out",
        "data": "synthetic",
        "config": {"workload": "quantize-and-pack of fp32 NHWC activations 128x56x56x256 (Eq. 10 thresholds), "
                               "4 B read + 0.25 B written per element", "elements": n},
        "roofline": hbm_roofline("quantize_pack_bordered_kernel", n * 4.25 / (k1 * 1e-3) / 1e9, k1, peaks),
        "cpu_baseline": None,
        "extra": {"pack_from_int8_levels_ms": round(k2, 5),
                  "pack_from_int8_levels_GBps": round(n * 1.25 / (k2 * 1e-3) / 1e9, 1)},
    }
    print(json.dumps(line))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one MI355X; this build has no multi-GPU path (columns would be sharded "
              "with no collectives). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2008_05101_amd as fatnn
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    fatnn.lib()   # fail loudly now if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.calibrate_copy:
        nbytes = 256 << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        scratch = fatnn.probe_scratch(dev)
        for _ in range(5):
            fatnn.probe_hbm(fatnn.HBM_COPY, dst, src, nbytes, scratch)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 launches of hbm_copy_kernel over 268435456 bytes "
                                         "(read 256 MiB + write 256 MiB each)"}))
        return

    if args.workload == "peaks":
        scratch = fatnn.probe_scratch(dev)
        settle_ms = settle_clocks(torch, lambda: fatnn.probe_valu(fatnn.PROBE_PAIR_V, 4, 400, scratch))
        pk = measure_peaks(torch, fatnn, full=True)
        line = {"metric": "ternary VALU ceiling Tops/s (register-resident bitop3+bcnt pairs x 16 ops) at 1 MI355X",
                "value": pk["ternary_peak_measured_tops"], "unit": "Tops/s", "n_gpus": 1, "steps": args.steps,
                "warmup": args.warmup, "ms_per_step": None, "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "u32 bitwise", "data": "synthetic",
                "config": {"workload": "peaks: issue rate of the method's instruction pair from registers over "
                                       "1..8 wavefronts per SIMD, and HBM read / write / copy streams of 1 GiB"},
                "roofline": {"bound": "alu", "kernel": "valu_probe_kernel", "achieved": pk["ternary_peak_measured_tops"],
                             "peak": round(TERNARY_PEAK_TOPS, 1), "unit": "Tops/s",
                             "frac": round(pk["ternary_peak_measured_tops"] / TERNARY_PEAK_TOPS, 4), "traffic": None},
                "cpu_baseline": None, "extra": {**pk, "settle_ms": round(settle_ms, 1)}}
        print(json.dumps(line))
        return

    if args.workload in ("cfg3", "cfg5", "quantpack", "paper6", "midgemm"):
        side_workload(args, torch, fatnn, si, dev)
        return
    extra = {}
    if args.workload == "cfg2":
        case = si.cfg2()
        Lw, Lx = case.make()
        scale, bias = case.make_scale_bias()
        Lw_d = torch.from_numpy(Lw).to(dev)
        Lx_d = torch.from_numpy(Lx).to(dev)
        scale_d = torch.from_numpy(scale).to(dev)
        bias_d = torch.from_numpy(bias).to(dev)
        Wp = fatnn.pack_ternary(Lw_d, fatnn.WEIGHT, fatnn.OHWI)           # offline, once
        plain = args.plain_input
        x_layout = fatnn.X_PLAIN if plain else fatnn.X_BORDERED
        Xp = torch.empty(fatnn.packed_bytes(fatnn.ACT, case.B * case.H * case.W, case.Cin) if plain else
                         fatnn.bordered_act_bytes(case.B, case.H, case.W, case.Cin, case.pad), dtype=torch.uint8,
                         device=dev)
        Y = torch.empty((case.B, case.Ho, case.Wo, case.Cout), dtype=torch.int32, device=dev)
        Yf = torch.empty((case.B, case.Ho, case.Wo, case.Cout), dtype=torch.float32, device=dev)
        conv_args = (case.B, case.Cin, case.H, case.W, case.Cout, case.R, case.S, case.stride, case.pad,
                     case.act_mode)

        def pack_step():
            if plain:
                fatnn.pack_ternary(Lx_d, fatnn.ACT, fatnn.NHWC, out=Xp)
            else:
                fatnn.pack_ternary_bordered(Lx_d, case.pad, case.act_mode, out=Xp)

        def main_kernel():
            fatnn.ternary_conv2d(Wp, Xp, *conv_args, out=Y, scale=scale_d, bias=bias_d, out_f=Yf, x_layout=x_layout)

        ops_per_step = 2.0 * case.macs()
        config = {"workload": "cfg2: 3x3 conv 128->128 @28x28, batch 32, stride 1, pad 1 as implicit GEMM "
                              "(M=128, N=25088, K=1152), ReLU-mode activations, int32 + fp32 scale/bias outputs; "
                              "step = pack activations + conv",
                  "M": case.M, "N": case.N, "K": case.K, "batch": case.B}
        dominant = ("plane_gemm_kernel (ternary, LDS-tiled, implicit-im2col front end)" if plain else
                    "stream_conv_kernel (ternary, weight-stationary implicit-GEMM conv)")
        if plain:
            config["workload"] += "; activations packed in plain NHWC order (--plain-input)"
    else:
        case = si.cfg4()
        Lw, La = case.make()
        Lw_d = torch.from_numpy(Lw).to(dev)
        La_d = torch.from_numpy(La).to(dev)
        Wp = fatnn.pack_ternary(Lw_d, fatnn.WEIGHT)
        Ap = torch.empty(fatnn.packed_bytes(fatnn.ACT, case.N, case.K), dtype=torch.uint8, device=dev)
        C = torch.empty((case.M, case.N), dtype=torch.int32, device=dev)

        def pack_step():
            fatnn.pack_ternary(La_d, fatnn.ACT, out=Ap)

        def main_kernel():
            fatnn.ternary_gemm(Wp, Ap, case.M, case.N, case.K, case.act_mode, out=C)

        ops_per_step = 2.0 * case.macs()
        config = {"workload": "cfg4: ternary GEMM M=N=K=8192 on the seeded operands (weights P(0)=0.33, activations "
                              "uniform over 3 levels), symmetric activations, int32 output; step = pack activations + GEMM",
                  "M": case.M, "N": case.N, "K": case.K}
        dominant = "plane_gemm_kernel (ternary GEMM, 128x128 tiles)"

    def step():
        pack_step()
        main_kernel()

    # The timed loop calls the C ABI with arguments converted once: the Python-side marshalling of
    # the convenience wrappers costs about as much CPU time per call as a 10 us kernel takes to run.
    import ctypes
    L = fatnn.lib()
    stream = torch.cuda.current_stream().cuda_stream
    vp = ctypes.c_void_p
    if args.workload == "cfg2":
        dims = (ctypes.c_int64 * 4)(case.B, case.H, case.W, case.Cin)
        if plain:
            pack_args = (vp(Lx_d.data_ptr()), fatnn.NHWC, dims, fatnn.ACT, vp(Xp.data_ptr()), Xp.numel(), None, vp(stream))
            pack_fn = L.fatnn_pack_ternary
        else:
            pack_args = (vp(Lx_d.data_ptr()), dims, case.pad, case.act_mode, vp(Xp.data_ptr()), Xp.numel(), None,
                         vp(stream))
            pack_fn = L.fatnn_pack_ternary_bordered
        main_args = (vp(Wp.data_ptr()), vp(Xp.data_ptr()), x_layout, case.B, case.Cin, case.H, case.W, case.Cout,
                     case.R, case.S, case.stride, case.pad, case.act_mode, vp(Y.data_ptr()), vp(scale_d.data_ptr()),
                     vp(bias_d.data_ptr()), vp(Yf.data_ptr()), vp(stream))
        main_fn = L.fatnn_ternary_conv2d
    else:
        dims = (ctypes.c_int64 * 4)(case.N, case.K, 1, 1)
        pack_args = (vp(La_d.data_ptr()), fatnn.ROWMAJOR_K, dims, fatnn.ACT, vp(Ap.data_ptr()), Ap.numel(), None,
                     vp(stream))
        pack_fn = L.fatnn_pack_ternary
        main_args = (vp(Wp.data_ptr()), vp(Ap.data_ptr()), case.M, case.N, case.K, case.act_mode, vp(C.data_ptr()),
                     case.N, None, None, None, case.N, vp(stream))
        main_fn = L.fatnn_ternary_gemm
    hook_fn = L.fatnn_time_next_launch

    # ---- untimed: let the clocks settle, measure the ceilings on this GPU, warm up -------------
    settle_ms = settle_clocks(torch, step)
    peaks = measure_peaks(torch, fatnn)
    settle_ms += settle_clocks(torch, step, 0.1)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # ---- exactly K timed steps ----------------------------------------------------------------
    # Timed launches of the dominant kernel carry a pair of HIP events attached to their dispatch
    # (on the stream it is launched on), so its duration is measured inside the timed region
    # without serialising anything.  Attaching a pair costs about 5 us of step time with this
    # runtime: nothing against a millisecond GEMM, a quarter of a 20 us convolution step, so the
    # short workload carries one on every 8th step only.
    EVENT_EVERY = 8 if (args.workload == "cfg2" and args.steps >= 32) else 1
    timed = list(range(0, args.steps, EVENT_EVERY))
    hev = HipEvents(2 * len(timed))
    handles = {i: (vp(hev.handle(2 * j)), vp(hev.handle(2 * j + 1))) for j, i in enumerate(timed)}
    status = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        status |= pack_fn(*pack_args)
        if i in handles:
            status |= hook_fn(*handles[i])
        status |= main_fn(*main_args)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if status != 0:
        raise RuntimeError("a library call failed inside the timed loop")
    ms_per_step = wall * 1e3 / args.steps
    kernel_times = sorted(hev.elapsed_ms(2 * j, 2 * j + 1) for j in range(len(timed)))
    kernel_ms = sum(kernel_times) / len(kernel_times)
    hev.close()
    value = ops_per_step / (ms_per_step * 1e-3) / 1e12

    achieved = ops_per_step / (kernel_ms * 1e-3) / 1e12
    traffic_key = args.workload + ("_plain_input" if getattr(args, "plain_input", False) else "")
    roofline = alu_roofline(dominant, achieved, kernel_ms, peaks, measured_traffic_bytes(traffic_key))
    roofline["kernel_ms_median"] = round(kernel_times[len(kernel_times) // 2], 5)
    roofline["kernel_ms_min"] = round(kernel_times[0], 5)
    roofline["kernel_launches_timed"] = len(kernel_times)
    extra["settle_ms_untimed"] = round(settle_ms, 1)
    extra["peaks_measured_in_this_run"] = peaks

    # ---- side measurements (outside the timed region) ---------------------------------------
    if not args.no_extra:
        try:
            reps = (500, 100) if args.workload == "cfg2" else (20, 5)
            extra["pack_ms"] = round(time_kernel_ms(torch, pack_step, *reps), 5)
            extra["main_kernel_ms_back_to_back"] = round(time_kernel_ms(torch, main_kernel, *reps), 5)
            # the same step and the same kernel replayed from a HIP graph (no host launch path between them)
            extra["step_ms_graph_replay"] = round(time_graph_ms(torch, step, 20), 5)
            extra["main_kernel_ms_graph_replay"] = round(time_graph_ms(torch, main_kernel, 20), 5)
            code = torch.tensor([0, 1, 3], dtype=torch.int8, device=dev)
            if args.workload == "cfg2" and args.plain_input:
                pass
            elif args.workload == "cfg2":
                W2 = fatnn.pack_twobit(code[Lw_d.long()], fatnn.WEIGHT, fatnn.OHWI)
                X2 = fatnn.pack_twobit_bordered(code[Lx_d.long()], case.pad)
                t2 = time_kernel_ms(torch, lambda: fatnn.twobit_conv2d(W2, X2, *conv_args[:-1], out=Y,
                                                                       x_layout=fatnn.X_BORDERED), 500, 100)
                t3 = time_kernel_ms(torch, lambda: fatnn.ternary_conv2d(Wp, Xp, *conv_args, out=Y,
                                                                        x_layout=fatnn.X_BORDERED), 500, 100)
                t4 = time_kernel_ms(torch, lambda: fatnn.twobit_conv2d(W2, X2, *conv_args[:-1], fatnn.BASIS_XNOR_ONLY,
                                                                       out=Y, x_layout=fatnn.X_BORDERED), 500, 100)
                extra["twobit_conv_ms"] = round(t2, 5)
                extra["ternary_conv_int32_only_ms"] = round(t3, 5)
                extra["speedup_vs_twobit"] = round(t2 / t3, 3)
                # Table 4's ablation: the same layer with the xnor rule alone (no zero-operand fix)
                extra["xnor_only_conv_ms"] = round(t4, 5)
                extra["extra_bit_ops_cost"] = round((t3 - t4) / t3, 4)
                # int8 MFMA comparison point (context only): same operands as int8 values through the BLAS
                try:
                    a8 = (Lw_d.reshape(case.Cout, -1) - 1).contiguous()
                    x8 = torch.randint(-1, 2, (case.K, case.N), dtype=torch.int8, device=dev)
                    ti = time_kernel_ms(torch, lambda: torch._int_mm(a8, x8), 20, 3)
                    extra["int8_mfma_gemm_same_shape_ms"] = round(ti, 5)
                except Exception as exc:       # comparison only; never fatal
                    extra["int8_mfma_gemm_same_shape_ms"] = f"unavailable: {type(exc).__name__}"
            else:
                tk = extra["main_kernel_ms_back_to_back"]
                W2 = fatnn.pack_twobit(code[Lw_d.long()])
                A2 = fatnn.pack_twobit(code[La_d.long()])
                t2 = time_kernel_ms(torch, lambda: fatnn.twobit_gemm(W2, A2, case.M, case.N, case.K, 0, out=C), 10, 2)
                t3 = time_kernel_ms(torch, lambda: fatnn.twobit_gemm(W2, A2, case.M, case.N, case.K, 2, out=C), 10, 2)
                extra["twobit_gemm_ms"] = round(t2, 4)
                extra["speedup_vs_twobit"] = round(t2 / tk, 3)
                extra["xnor_only_gemm_ms"] = round(t3, 4)
                extra["extra_bit_ops_cost"] = round((tk - t3) / tk, 4)
                del W2, A2
                Bw = fatnn.pack_binary((Lw_d == 2).to(torch.int8))
                Ba = fatnn.pack_binary((La_d == 2).to(torch.int8))
                tb = time_kernel_ms(torch, lambda: fatnn.binary_gemm(Bw, Ba, case.M, case.N, case.K, out=C), 10, 2)
                extra["binary_gemm_ms"] = round(tb, 4)
                extra["ternary_over_binary"] = round(tk / tb, 3)
                del Bw, Ba
                try:
                    a8 = (Lw_d - 1).contiguous()
                    x8 = (La_d - 1).t().contiguous()
                    ti = time_kernel_ms(torch, lambda: torch._int_mm(a8, x8), 5, 2)
                    extra["int8_mfma_gemm_ms"] = round(ti, 4)
                    del a8, x8
                except Exception as exc:
                    extra["int8_mfma_gemm_ms"] = f"unavailable: {type(exc).__name__}"
                extra["other_configs"] = other_config_summaries(torch, fatnn, si, dev, peaks)
        except Exception as exc:   # side measurements must never lose the main line
            extra["error"] = f"{type(exc).__name__}: {exc}"

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline_conv(case) if args.workload == "cfg2" else cpu_baseline_gemm(case)

    line = {
        "metric": "ternary GEMM Tops/s (2MNK) at 1 MI355X",
        "value": round(value, 3),
        "unit": "Tops/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 bit-planes, int32 accumulate",
        "data": "synthetic",
        "config": config,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
