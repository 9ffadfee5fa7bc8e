#!/usr/bin/env python3
"""Benchmark of the fused sliced-GEMM + reduce-scatter-reduction path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: one call of
t3_gemm_rs_fused (tile issue in ring order, MFMA main loop, reduction epilogue,
track & trigger, release into the forward buffer).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line: fused TFLOP/s (2*M*N*K / time), the roofline figure of
the fused kernel measured with events on the launch stream, the unfused GEMM-then-reduce
time measured in the same process, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # 256 CU x 2.4 GHz x 4096 flop/clk/CU, dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM-side bytes per launch of the fused kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# scaled by the same counters' reading of a plain copy (profiles/*_hbm_traffic.txt says how).
# Keyed by (workload, release); None = not measured since the kernel last changed.
MEASURED_TRAFFIC_BYTES = {("gpt3_outproj", "direct"): 630.7e6}


def algorithmic_bytes(w, direct, fwd_bf16=False):
    """Bytes the method must move: A and B once, incoming once, result once; the default
    release adds one read and one write of every forwarded chunk.  bfloat16 forward slots
    halve the bytes written to them."""
    fwd_part = w.M * w.N * (w.tp - 1) / w.tp          # elements that are forwarded
    base = 2.0 * w.M * w.K + 2.0 * w.K * w.N + 8.0 * w.M * w.N
    if not direct:
        base += 8.0 * fwd_part
    if fwd_bf16:
        base -= 2.0 * fwd_part
    return base


def cpu_baseline(w, a_bits, b_bits, inc, target_s=12.0):
    """The oracle as it stands, on the host cores, on the first rows of the same workload."""
    from oracle import t3_oracle as orc
    probe = min(w.M, 16)
    t0 = time.perf_counter()
    orc.reduce_rows(orc.gemm_rows(a_bits, b_bits, rows=np.arange(probe, dtype=np.int32)),
                    inc, w.tp, rows=np.arange(probe, dtype=np.int32))
    t_probe = time.perf_counter() - t0
    rows = int(min(w.M, max(probe, probe * target_s / max(t_probe, 1e-3))))
    sel = np.arange(rows, dtype=np.int32)
    t0 = time.perf_counter()
    S = orc.reduce_rows(orc.gemm_rows(a_bits, b_bits, rows=sel), inc, w.tp, rows=sel)
    dt = time.perf_counter() - t0
    tf = 2.0 * rows * w.N * w.K / dt / 1e12
    return {"value": tf, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {w.M} rows of {w.name} (all {w.N} columns, K={w.K}): "
                      f"fp64 GEMM + reduction in {dt:.2f} s"}, S, sel


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="gpt3_outproj")
    ap.add_argument("--release", choices=["direct", "copy"], default="direct",
                    help="direct: forwarded sums go straight to the forward buffer "
                         "(T3_FLAG_FWD_DIRECT); copy: sums are added in place and release "
                         "workgroups copy each triggered chunk to its forward slot")
    ap.add_argument("--fwd-bf16", action="store_true",
                    help="forward slots in bfloat16 (T3_FLAG_FWD_BF16); the default run keeps fp32")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--main-only", action="store_true",
                    help="skip the leg that times the other release mode (it launches the same "
                         "kernel, so a per-kernel profile of the run would mix the two)")
    ap.add_argument("--graph", action="store_true",
                    help="replay each step as a captured HIP graph instead of launching its kernels "
                         "one by one (a step here is one or two kernels: back-to-back launches keep "
                         "the queue full, a graph launch per step leaves a gap between steps)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for `rocprofv3 --pmc` runs (FETCH_SIZE, WRITE_SIZE, MFMA counters): launch "
                         "5 x [a plain device copy of the M x N fp32 buffer, the fused kernel, the "
                         "unfused GEMM and reduction] and exit")
    args = ap.parse_args()
    args.direct = args.release == "direct"
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path is one rank's kernel, with no "
                 "collective between GPUs; run with --gpus 1")

    import torch
    from paper_2401_16677_amd import binding as t3
    from paper_2401_16677_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    w = wl.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    a_bits, b_bits, inc = wl.make_inputs(w)
    A = torch.from_numpy(a_bits.view(np.int16)).to(dev)
    B = torch.from_numpy(b_bits.view(np.int16)).to(dev)
    inc_dev = torch.from_numpy(inc).to(dev)
    R = inc_dev.clone()
    fwd = torch.zeros((w.tp - 1, w.M, w.W), dtype=torch.float32, device=dev)
    C = torch.empty((w.M, w.N), dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(w.tp), dtype=torch.int32, device=dev)
    fmt = t3.T3_FLAG_FWD_BF16 if args.fwd_bf16 else 0
    flags = (t3.T3_FLAG_FWD_DIRECT if args.direct else 0) | fmt
    p = t3.problem(w.M, w.N, w.K, w.tp, w.rank, w.tile_m, w.tile_n, flags=flags)
    tile = (w.tile_m, w.tile_n) if w.tile_m else t3.t3_default_tile(p)

    t3.t3_track_reset(w.tp, track)       # once: every launch leaves a clean bank for the next

    def fused_step():
        t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)

    def unfused_step():
        t3.t3_gemm(p, A, B, C)
        t3.t3_rs_reduce(p, C, R, fwd, track)

    if args.traffic_probe:
        # the copy (a known number of bytes each way) calibrates the counters; see profiles/
        for _ in range(5):
            C.copy_(R)
            fused_step()
            unfused_step()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": w.name, "copy_bytes_each_way": 4 * w.M * w.N,
                          "launches": 5}))
        return

    def graphed(step):
        """Capture one step (its kernels are launched on the capturing stream) and return a
        function that replays it: one graph launch per step instead of one per kernel."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                      # warm the launch path outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        return g.replay

    if args.graph:
        fused_step = graphed(fused_step)
        unfused_step = graphed(unfused_step)

    def timed(step, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    # Bring the device to its sustained state first: from idle the clocks need tens of
    # milliseconds of load to settle (the first ~100 launches run 20-25 % slower), which the W
    # warm-up steps alone do not cover.  Untimed.
    t_end = time.perf_counter() + 0.5
    while time.perf_counter() < t_end:
        for _ in range(20):
            fused_step()
        torch.cuda.synchronize()

    # parity of this very launch configuration on sampled rows is checked by the GPU tests;
    # here only a cheap sanity check that the run completed every chunk
    for _ in range(args.warmup):
        fused_step()
    t_fused = timed(fused_step, args.steps)
    tr = t3.read_track(track, w.tp)
    assert int(tr["counter"].sum()) == w.tp * t3.t3_tiles_per_chunk(p) and tr["error"] == 0, \
        "tracker did not complete"

    # kernel-only duration of the fused kernel, events on the stream it is launched on
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    for e0, e1 in ev:
        e0.record()
        t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
        e1.record()
    torch.cuda.synchronize()
    k_ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    k_avg = sum(k_ms) / len(k_ms)

    R.copy_(inc_dev)
    t_end = time.perf_counter() + 0.3
    while time.perf_counter() < t_end:
        for _ in range(20):
            unfused_step()
        torch.cuda.synchronize()
    for _ in range(max(3, args.warmup // 2)):
        unfused_step()
    t_unfused = timed(unfused_step, args.steps)

    # The other release mode, fused and unfused, timed the same way (reported beside the main
    # figures: `copy` is the literal add-in-place-then-release path, `direct` writes forwarded
    # sums straight to their forward slots).
    o_flags = (0 if args.direct else t3.T3_FLAG_FWD_DIRECT) | fmt
    po = t3.problem(w.M, w.N, w.K, w.tp, w.rank, w.tile_m, w.tile_n, flags=o_flags)

    def o_fused():
        t3.t3_gemm_rs_fused(po, A, B, R, fwd, track)

    def o_unfused():
        t3.t3_gemm(po, A, B, C)
        t3.t3_rs_reduce(po, C, R, fwd, track)

    other = {}
    for key, step in (() if args.main_only else
                      (("ms_per_step", o_fused), ("unfused_ms_per_step", o_unfused))):
        R.copy_(inc_dev)
        t_end = time.perf_counter() + 0.2
        while time.perf_counter() < t_end:
            for _ in range(20):
                step()
            torch.cuda.synchronize()
        other[key] = timed(step, args.steps) * 1e3
    if other:
        other["tflops"] = w.flop / (other["ms_per_step"] * 1e-3) / 1e12
        other["speedup_vs_unfused"] = other["unfused_ms_per_step"] / other["ms_per_step"]
        tr = t3.read_track(track, w.tp)
        assert tr["error"] == 0, "tracker error in the other release mode"

    tflops = w.flop / t_fused / 1e12
    bytes_alg = algorithmic_bytes(w, args.direct, args.fwd_bf16)
    t_mfma = w.flop / (PEAK_BF16_TFLOPS * 1e12)
    t_hbm = bytes_alg / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        ach = w.flop / (k_avg * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS,
                "traffic": None if args.fwd_bf16 else MEASURED_TRAFFIC_BYTES.get((w.name, args.release))}
    else:
        ach = bytes_alg / (k_avg * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS,
                "traffic": None if args.fwd_bf16 else MEASURED_TRAFFIC_BYTES.get((w.name, args.release))}
    roof.update(kernel="gemm_tile_kernel<%d,%d,fused>" % tuple(tile),
                kernel_ms_avg=k_avg, kernel_ms_min=k_ms[0], kernel_ms_median=k_ms[len(k_ms) // 2],
                algorithmic_bytes=bytes_alg, flop=w.flop)

    out = {
        "metric": "fused GEMM+RS-reduction TFLOP/s, % bf16 MFMA peak, speedup vs unfused (1 GPU)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": t_fused * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "tp": w.tp, "rank": w.rank,
                   "tile": list(tile),
                   "release": "direct" if args.direct else "copy",
                   "fwd": "bf16" if args.fwd_bf16 else "fp32",
                   "launch": "hip_graph" if args.graph else "eager"},
        "pct_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
        "unfused_ms_per_step": t_unfused * 1e3,
        "speedup_vs_unfused": t_unfused / t_fused,
        "roofline": roof,
    }
    if other:
        out["release_copy" if args.direct else "release_direct"] = other
    if not args.no_cpu:
        out["cpu_baseline"], _, _ = cpu_baseline(w, a_bits, b_bits, inc)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
