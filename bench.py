#!/usr/bin/env python3
"""Benchmark of the fused sliced-GEMM + reduce-scatter-reduction path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: one call of
t3_gemm_rs_fused (tile issue in ring order, MFMA main loop, reduction epilogue,
track & trigger, release into the forward buffer).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.  The headline (`value`, `ms_per_step`, `roofline`,
`cpu_baseline`) is the largest of the five configurations, wide_fc2, on the 128 x 256 tile
its description names; `configs` holds one record per configuration (fused step, TFLOP/s,
fraction of the bf16 MFMA peak or of the HBM peak, whichever bounds it, the unfused
GEMM-then-reduce step measured in the same process, and the speed-up).
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
HEADLINE = "wide_fc2"
CONFIGS = ["tiny_outproj", "gpt3_outproj", "gpt3_fc2", "wide_fc2", "hightp_outproj"]

# Bytes per launch of the fused kernel at the L2 <-> fabric boundary, TRANSCRIBED from the
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries under profiles/ (each scaled by the same
# counter's reading of a plain copy; the file says how).  Not measured in this run.  Keyed by
# (workload, release); a workload is listed only while the kernel is the one that was profiled.
PROFILED_TRAFFIC_BYTES = {("gpt3_outproj", "direct"): 630.8e6, ("gpt3_fc2", "direct"): 1314.0e6,
                          ("wide_fc2", "direct"): 2492.1e6, ("hightp_outproj", "direct"): 1737.4e6}
PROFILED_TRAFFIC_SOURCE = "profiles/fused_gemm_rs_<workload>_hbm_traffic.txt (transcribed, not measured in this run)"


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
    orc.reduce_rows(orc.gemm_rows(a_bits, b_bits, rows=sel), inc, w.tp, rows=sel)
    dt = time.perf_counter() - t0
    tf = 2.0 * rows * w.N * w.K / dt / 1e12
    return {"value": tf, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {w.M} rows of {w.name} (all {w.N} columns, K={w.K}): "
                      f"fp64 GEMM + reduction in {dt:.2f} s"}


def timeline_report(b, direct, torch, t3):
    """The last of 30 back-to-back fused launches, and of 30 plain-GEMM launches, of the workload
    with t3_timeline recording, after the usual settling; returns a text table (times in microseconds; medians over the
    workgroups that had an i-th piece of work)."""
    w = b.w
    p = b.problem(direct)
    items, wgs = t3.T3_TIMELINE_ITEMS, 512
    fused, unfused = b.steps(direct)
    b.settle(fused, 0.5)
    lines = [f"workload {w.name} (M={w.M} N={w.N} K={w.K} TP={w.tp} rank {w.rank}), "
             f"release={'direct' if direct else 'copy'}; device wall clock (100 MHz), microseconds"]
    runs = {"fused kernel (t3_gemm_rs_fused)": lambda: t3.t3_gemm_rs_fused(p, b.A, b.B, b.R, b.fwd, b.track),
            "plain GEMM (t3_gemm)": lambda: t3.t3_gemm(p, b.A, b.B, b.C)}
    totals = {}
    for label, call in runs.items():
        # 30 launches back to back, all recording into the same entries: what is read afterwards
        # is the last one's, taken in this kernel's own steady state (a launch that follows even
        # a short idle gap runs 15-20 % slower)
        st = torch.zeros(wgs * items * 4, dtype=torch.int64, device=b.A.device)
        ms = []
        for _ in range(60):
            call()                                   # this kernel's own steady state first
        for rec in (None, st):                       # 30 launches without recording, then 30 with
            t3.t3_timeline(rec)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(30):
                call()
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1) / 30)
        t3.t3_timeline(None)
        s = st.cpu().numpy().reshape(wgs, items, 4).astype(np.float64)
        used = s[:, 0, 0] > 0
        n_wg = int(used.sum())
        s = s[used]
        t0 = s[:, 0, 0].min()
        valid = s[:, :, 3] > 0
        rel = np.where(s > 0, (s - t0) / 100.0, np.nan)
        end = np.nanmax(rel[:, :, 3], axis=1)
        lines += ["", f"{label}: {n_wg} workgroups, launch spans {np.nanmax(end):.1f} us from the first piece taken "
                      f"to the last results handed over; {1e3 * ms[1]:.1f} us per launch with recording, {1e3 * ms[0]:.1f} without",
                  f"  {'piece':<7}{'workgroups':>11}{'taken at':>10}{'set-up':>9}{'main loop':>11}{'hand-over':>11}{'whole piece':>13}"]
        # A balanced tail gives half the workgroups a half tile first and the others one last:
        # the two kinds are tabulated apart (told by the length of the first piece).
        first = rel[:, 0, 3] - rel[:, 0, 0]
        groups = [("", np.ones(len(first), bool))]
        if first.max() > 1.5 * first.min():
            short = first < 0.5 * (first.max() + first.min())
            groups = [("  workgroups that start with half a tile:", short), ("  the others:", ~short)]
        per_piece = []
        for title, sel in groups:
            if title:
                lines.append(title)
            for i in range(items):
                v = valid[:, i] & sel
                if not v.any():
                    continue
                r = rel[v, i, :]
                d = [np.median(r[:, 1] - r[:, 0]), np.median(r[:, 2] - r[:, 1]), np.median(r[:, 3] - r[:, 2]),
                     np.median(r[:, 3] - r[:, 0])]
                if len(groups) == 1:
                    per_piece.append(d)
                lines.append(f"  {i:<7}{int(v.sum()):>11}{np.median(r[:, 0]):>10.1f}{d[0]:>9.1f}{d[1]:>11.1f}{d[2]:>11.1f}{d[3]:>13.1f}")
        xcd = np.arange(wgs)[used] % 8
        lines.append("  last hand-over per XCD (workgroup index mod 8), median of its workgroups: " +
                     "  ".join(f"{x}: {np.median(end[xcd == x]):.1f}" for x in range(8) if (xcd == x).any()))
        totals[label] = per_piece
    f, g = totals["fused kernel (t3_gemm_rs_fused)"], totals["plain GEMM (t3_gemm)"]
    if f and g and len(f) == len(g):   # (not with a balanced tail: its pieces differ in kind)
        lines += ["", "fused minus plain GEMM, per piece (set-up / main loop / hand-over / whole): " +
                  "; ".join(f"{a[0] - c[0]:+.1f} / {a[1] - c[1]:+.1f} / {a[2] - c[2]:+.1f} / {a[3] - c[3]:+.1f}"
                            for a, c in zip(f, g))]
    lines += ["", "set-up = piece taken -> accumulators hold the incoming partial (fused) or zeros (plain); for tiles after a",
              "workgroup's first the incoming partial was requested at the end of the previous piece's hand-over, so part of",
              "its flight time shows there.  main loop = the K loop.  hand-over = results through LDS into write-through stores",
              "(+ the request for the next tile's incoming partial); their acknowledgement overlaps the next piece."]
    return "\n".join(lines)


class Bench:
    """Device buffers of one workload and the timed steps over them."""

    def __init__(self, w, args, torch, t3, wl):
        self.w, self.args, self.torch, self.t3 = w, args, torch, t3
        dev = torch.device("cuda:0")
        self.host = wl.make_inputs(w)
        a_bits, b_bits, inc = self.host
        self.A = torch.from_numpy(a_bits.view(np.int16)).to(dev)
        self.B = torch.from_numpy(b_bits.view(np.int16)).to(dev)
        self.inc = torch.from_numpy(inc).to(dev)
        self.R = self.inc.clone()
        self.fwd = torch.zeros((w.tp - 1, w.M, w.W), dtype=torch.float32, device=dev)
        self.C = torch.empty((w.M, w.N), dtype=torch.float32, device=dev)
        self.track = torch.zeros(t3.t3_track_words(w.tp), dtype=torch.int32, device=dev)
        t3.t3_track_reset(w.tp, self.track)   # once: every launch leaves a clean bank for the next
        self.fmt = t3.T3_FLAG_FWD_BF16 if args.fwd_bf16 else 0

    def problem(self, direct):
        w, t3 = self.w, self.t3
        return t3.problem(w.M, w.N, w.K, w.tp, w.rank, w.tile_m, w.tile_n,
                          flags=(t3.T3_FLAG_FWD_DIRECT if direct else 0) | self.fmt)

    def steps(self, direct):
        p, t3 = self.problem(direct), self.t3

        def fused():
            t3.t3_gemm_rs_fused(p, self.A, self.B, self.R, self.fwd, self.track)

        def unfused():
            t3.t3_gemm(p, self.A, self.B, self.C)
            t3.t3_rs_reduce(p, self.C, self.R, self.fwd, self.track)

        if self.args.graph:
            return self.graphed(fused), self.graphed(unfused)
        return fused, unfused

    def graphed(self, step):
        """Capture one step (its kernels are launched on the capturing stream) and return a
        function that replays it: one graph launch per step instead of one per kernel."""
        torch = self.torch
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

    def settle(self, step, seconds):
        """Bring the device to its sustained state: from idle the clocks need tens of
        milliseconds of load to settle (the first ~100 launches run 20-25 % slower), which the
        warm-up steps alone do not cover.  Untimed."""
        torch = self.torch
        t_end = time.perf_counter() + seconds
        while time.perf_counter() < t_end:
            for _ in range(20):
                step()
            torch.cuda.synchronize()

    def timed(self, step, n):
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    def kernel_ms(self, direct, n):
        """Duration of the fused kernel alone: event pairs on the stream it is launched on."""
        torch, t3 = self.torch, self.t3
        p = self.problem(direct)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(n)]
        torch.cuda.synchronize()
        for e0, e1 in ev:
            e0.record()
            t3.t3_gemm_rs_fused(p, self.A, self.B, self.R, self.fwd, self.track)
            e1.record()
        torch.cuda.synchronize()
        return sorted(e0.elapsed_time(e1) for e0, e1 in ev)

    def check_tracker(self, direct):
        tr = self.t3.read_track(self.track, self.w.tp)
        tiles = self.w.tp * self.t3.t3_tiles_per_chunk(self.problem(direct))
        assert int(tr["counter"].sum()) == tiles and int(tr["ready"].sum()) == self.w.tp and \
            tr["queue_len"] == self.w.tp - 1 and tr["error"] == 0, "tracker did not complete"

    def measure(self, direct, settle_s=0.5):
        """Fused and unfused step of one release mode -> record."""
        w, args = self.w, self.args
        fused, unfused = self.steps(direct)
        self.R.copy_(self.inc)
        self.settle(fused, settle_s)
        for _ in range(args.warmup):
            fused()
        t_fused = self.timed(fused, args.steps)
        self.check_tracker(direct)            # the run completed every chunk, no release gave up
        k_ms = self.kernel_ms(direct, args.steps)
        k_avg = sum(k_ms) / len(k_ms)
        self.R.copy_(self.inc)
        self.settle(unfused, settle_s * 0.6)
        for _ in range(max(3, args.warmup // 2)):
            unfused()
        t_unfused = self.timed(unfused, args.steps)
        self.check_tracker(direct)

        bytes_alg = algorithmic_bytes(w, direct, args.fwd_bf16)
        t_mfma = w.flop / (PEAK_BF16_TFLOPS * 1e12)
        t_hbm = bytes_alg / (PEAK_HBM_GBS * 1e9)
        traffic = None if args.fwd_bf16 else PROFILED_TRAFFIC_BYTES.get(
            (w.name, "direct" if direct else "copy"))
        if t_mfma >= t_hbm:
            ach = w.flop / (k_avg * 1e-3) / 1e12
            roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic}
        else:
            ach = bytes_alg / (k_avg * 1e-3) / 1e9
            roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": ach / PEAK_HBM_GBS, "traffic": traffic}
        if traffic is not None:
            roof["traffic_source"] = PROFILED_TRAFFIC_SOURCE.replace("<workload>", w.name)
        tile = (w.tile_m, w.tile_n) if w.tile_m else self.t3.t3_default_tile(self.problem(direct))
        roof.update(kernel="gemm_tile_kernel<%d,%d,fused>" % tuple(tile), kernel_ms_avg=k_avg,
                    kernel_ms_min=k_ms[0], kernel_ms_median=k_ms[len(k_ms) // 2],
                    algorithmic_bytes=bytes_alg, flop=w.flop)
        tflops = w.flop / t_fused / 1e12
        return {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "tp": w.tp, "rank": w.rank,
                "tile": list(tile), "release": "direct" if direct else "copy",
                "ms_per_step": t_fused * 1e3, "tflops": tflops,
                "pct_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
                "hbm_gbs_algorithmic": bytes_alg / t_fused / 1e9,
                "unfused_ms_per_step": t_unfused * 1e3, "speedup_vs_unfused": t_unfused / t_fused,
                "roofline": roof}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE,
                    help="the headline workload (default: the largest configuration)")
    ap.add_argument("--release", choices=["direct", "copy"], default="direct",
                    help="direct: forwarded sums go straight to the forward buffer "
                         "(T3_FLAG_FWD_DIRECT); copy: sums are added in place and release "
                         "workgroups copy each triggered chunk to its forward slot")
    ap.add_argument("--fwd-bf16", action="store_true",
                    help="forward slots in bfloat16 (T3_FLAG_FWD_BF16); the default run keeps fp32")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--main-only", action="store_true",
                    help="time the headline workload in the chosen release mode only: no record "
                         "of the other release mode and none of the other configurations (for "
                         "per-kernel profiles, which would otherwise mix them)")
    ap.add_argument("--graph", action="store_true",
                    help="replay each step as a captured HIP graph instead of launching its kernels "
                         "one by one (a step here is one or two kernels: back-to-back launches keep "
                         "the queue full, a graph launch per step leaves a gap between steps)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for `rocprofv3 --pmc` runs (FETCH_SIZE, WRITE_SIZE, MFMA counters): launch "
                         "5 x [a plain device copy of the M x N fp32 buffer, the fused kernel, the "
                         "unfused GEMM and reduction] and exit")
    ap.add_argument("--with-library-gemm", action="store_true",
                    help="with --traffic-probe: also launch the vendor library's bf16 GEMM behind "
                         "torch.matmul on the same A and B (bf16 output, no reduction), so that a "
                         "counter run shows its counters beside this library's kernels")
    ap.add_argument("--timeline", action="store_true",
                    help="record where the time of one fused launch and of one plain-GEMM launch "
                         "goes (t3_timeline: per workgroup and piece of work, the wall clock when "
                         "the piece is taken, when the accumulators are set up, when the main loop "
                         "is done and when the results have been handed over), print a table and exit")
    args = ap.parse_args()
    direct = args.release == "direct"
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path is one rank's kernel, with no "
                 "collective between GPUs; run with --gpus 1")

    import torch
    from paper_2401_16677_amd import binding as t3
    from paper_2401_16677_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    w = wl.WORKLOADS[args.workload]
    b = Bench(w, args, torch, t3, wl)

    if args.traffic_probe:
        # the copy (a known number of bytes each way) calibrates the counters; see profiles/
        fused, unfused = b.steps(direct)
        a16, b16t = b.A.view(torch.bfloat16), b.B.view(torch.bfloat16).t()
        for _ in range(5):
            b.C.copy_(b.R)
            fused()
            unfused()
            if args.with_library_gemm:
                torch.matmul(a16, b16t)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": w.name, "copy_bytes_each_way": 4 * w.M * w.N,
                          "launches": 5}))
        return

    if args.timeline:
        print(timeline_report(b, direct, torch, t3))
        return

    main_rec = b.measure(direct)
    out = {
        "metric": "fused GEMM+RS-reduction TFLOP/s, % bf16 MFMA peak, speedup vs unfused (1 GPU)",
        "value": main_rec["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_rec["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "tp": w.tp, "rank": w.rank,
                   "tile": main_rec["tile"], "release": main_rec["release"],
                   "fwd": "bf16" if args.fwd_bf16 else "fp32",
                   "launch": "hip_graph" if args.graph else "eager"},
        "pct_bf16_mfma_peak": main_rec["pct_bf16_mfma_peak"],
        "unfused_ms_per_step": main_rec["unfused_ms_per_step"],
        "speedup_vs_unfused": main_rec["speedup_vs_unfused"],
        "roofline": main_rec["roofline"],
    }
    if not args.main_only:
        # the other release mode of the headline workload (`copy` is the literal
        # add-in-place-then-release path, `direct` writes forwarded sums straight to their slots)
        other = b.measure(not direct, settle_s=0.2)
        out["release_" + other["release"]] = {k: other[k] for k in (
            "ms_per_step", "tflops", "unfused_ms_per_step", "speedup_vs_unfused")}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, *b.host)
    if not args.main_only:
        # one record per configuration, same protocol, same release mode as the headline
        recs = {w.name: main_rec}
        del b
        torch.cuda.empty_cache()
        for name in CONFIGS:
            if name in recs:
                continue
            bb = Bench(wl.WORKLOADS[name], args, torch, t3, wl)
            recs[name] = bb.measure(direct, settle_s=0.3)
            del bb
            torch.cuda.empty_cache()
        out["configs"] = {name: recs[name] for name in CONFIGS if name in recs}
        if w.name not in CONFIGS:
            out["configs"][w.name] = main_rec
    print(json.dumps(out))


if __name__ == "__main__":
    main()
