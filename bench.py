#!/usr/bin/env python3
"""Benchmark of the low-bit GEMM hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input of the headline workload
(cfg4: ternary x ternary, A 1024 x 4608, B 4608 x 50176 = batch 16 of 56x56 im2col):
    pack_ternary(A)  ->  pack_ternary(B)  ->  gemm_tnn  ->  int32 C
with the int8 inputs already resident in HBM.  value = 2*M*N*K / (step time), in TOPS.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel (gemm_tnn) against the rate the chip's vector ALU sustains for the kernel's own
                instruction mix, measured in the same run (and against the nominal 64 lanes per clock and compute unit)
  cpu_baseline  the CPU oracle (plain int32 triple loop) timed on a bounded row slice of the same workload
  extra         gemm-only and pack-only times, the int8 matrix-core comparator, the other configurations, the paper's
                shape grid; every timed quantity as median and minimum over >= 20 batches (extra.timing_us)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Nominal 32-bit VALU rate of MI355X: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
# (= the 157.3 TFLOP/s fp32 vector figure divided by 2 for FMA and by 2 for packed issue).  Context only: simple
# two-source logic issues faster than this, three-source forms and popcounts slightly slower; the ceiling used for
# roofline.frac is the measured rate of the kernel's own instruction mix (calibration chains of the library).
VALU_NOMINAL_TOPS = 256 * 64 * 2.4e9 / 1e12
HBM_PEAK_GBS = 8000.0
# lane-instructions per output and per 32 depth positions executed by the shipped kernels
LANE_INSTR = {"tnn": 4, "tbn": 2, "bnn": 2}
CALIB_MIX = {"bnn": 0, "tnn": 1, "tbn": 2}
BATCHES = 20


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


class Timing:
    """Event timing in batches; keeps median / min / mean of every named quantity (microseconds per launch)."""

    def __init__(self, torch, np):
        self.torch, self.np, self.table = torch, np, {}

    def _keep(self, name, samples_s, launches):
        a = self.np.asarray(samples_s, dtype=self.np.float64)
        if name:
            self.table[name] = {"median": float(self.np.median(a)) * 1e6, "min": float(a.min()) * 1e6,
                                "mean": float(a.mean()) * 1e6, "batches": int(a.size), "launches_per_batch": launches}
        return float(self.np.median(a))

    def dev(self, name, fn, iters, batches=BATCHES, warm=3):
        """`batches` event-bracketed groups of `iters` back-to-back launches on the current stream; median seconds."""
        torch = self.torch
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(batches)]
        for a, b in evs:
            a.record()
            for _ in range(iters):
                fn()
            b.record()
        torch.cuda.synchronize()
        return self._keep(name, [a.elapsed_time(b) * 1e-3 / iters for a, b in evs], iters)

    def graph(self, name, fn, per_graph, replays=BATCHES):
        """Kernel time without host launch gaps: capture per_graph launches into one HIP graph; every replay is a
        batch with its own event pair (all replays are queued before the first one is waited for)."""
        torch = self.torch
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            fn()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(per_graph):
                fn()
        g.replay()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
        for a, b in evs:
            a.record()
            g.replay()
            b.record()
        torch.cuda.synchronize()
        return self._keep(name, [a.elapsed_time(b) * 1e-3 / per_graph for a, b in evs], per_graph)


def calibrate_valu(T, torch, np, lb, mixes=("bnn", "tnn", "tbn"), waves=8, iters=8192):
    """Rate of each kernel's instruction mix on registers with `waves` waves per SIMD, and the engine clock it ran at."""
    sink = torch.empty(lb.lb_calib_sink_bytes() // 4, dtype=torch.int32, device="cuda")
    clk = torch.zeros(lb.lb_calib_clocks_bytes() // 8, dtype=torch.int64, device="cuda")
    khz = lb.lb_calib_wall_clock_khz()
    out = {}
    for kind in mixes:
        mix = CALIB_MIX[kind] if isinstance(kind, str) else kind
        name = f"calib_valu_{kind}_w{waves}"
        T.dev(name, lambda: lb.lb_calib_valu(mix, iters, sink, clk, waves), 1, BATCHES, warm=2)
        work = lb.lb_calib_valu_lane_instr(mix, iters, waves)
        st = T.table[name]
        c = clk.cpu().numpy().reshape(-1, 2)[:256 * waves].astype(np.float64)
        mhz = float(np.median(c[:, 0] / np.maximum(c[:, 1], 1.0)) * khz / 1e3) if khz else None
        out[kind] = {"tops_median": work / (st["median"] * 1e-6) / 1e12, "tops_best": work / (st["min"] * 1e-6) / 1e12,
                     "clock_mhz_under_load": mhz,
                     "lanes_per_clk_per_cu": None if not mhz else work / (st["median"] * 1e-6) / 256 / (mhz * 1e6)}
    return out, sink


def trace_scenario(args, torch, lb, synth) -> int:
    """Launch patterns meant to be run under `rocprofv3`; the trace or the counters, not this process, are the result.

    skinny: for cfg5 (TNN, TBN, BNN) two rounds over 384 MiB worth of copies of the packed large operand (24
            ternary / 48 binary copies: every launch streams it from HBM, cold), then 24 launches on one copy
            (warm), per skinny configuration.
    small:  for cfg1, cfg2, cfg3 30 launches per tile variant of the tiled kernel.
    """
    if args.scenario == "skinny":
        for name in ("cfg5_tnn_fc_n8", "cfg5_tbn_fc_n8", "cfg5_bnn_fc_n8"):
            w = synth.WORKLOADS[name]
            ncopy = 48 if w.kind == "bnn" else 24
            A, B = synth.make_inputs(w)
            Ap = lb.pack_a(w.kind, torch.from_numpy(A).cuda())
            Bp = lb.pack_b(w.kind, torch.from_numpy(B).cuda())
            copies = [Ap.clone() for _ in range(ncopy)]
            C = torch.empty((w.M, w.N), dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            for cfg in (range(lb.lb_num_variants(3)) if args.all_variants else [-1]):
                lb.lb_set_variant(3, cfg)
                for i in range(2 * ncopy):
                    lb.gemm(w.kind, w.M, w.N, w.K, copies[i % ncopy], Bp, C, w.N)
                torch.cuda.synchronize()
                for i in range(24):
                    lb.gemm(w.kind, w.M, w.N, w.K, copies[0], Bp, C, w.N)
                torch.cuda.synchronize()
            lb.lb_set_variant(3, -1)
            print(f"{name}: traced", flush=True)
    else:
        for name in ("cfg1_tnn_conv3x3x64_16x16", "cfg2_bnn_conv3x3x128_56x56", "cfg3_tbn_conv3x3x256_28x28"):
            w = synth.WORKLOADS[name]
            A, B = synth.make_inputs(w)
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            Ap, Bp = lb.pack_a(w.kind, dA), lb.pack_b(w.kind, dB)
            C = torch.empty((w.M, w.N), dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            for v in (list(range(lb.lb_num_variants(w.kind))) if args.all_variants else []) + [-1]:
                lb.lb_set_variant(w.kind, v)
                for _ in range(30):
                    lb.gemm(w.kind, w.M, w.N, w.K, Ap, Bp, C, w.N)
                torch.cuda.synchronize()
            for _ in range(30):
                lb.gemm_i8_mfma(w.M, w.N, w.K, dA, w.K, dB, w.N, C, w.N)
            torch.cuda.synchronize()
            print(f"{name}: traced", flush=True)
    return 0


def valu_rates_scenario(torch, np, lb) -> int:
    """Issue rate of the kernels' instruction mixes and of single instruction forms, 1 .. 8 waves per SIMD."""
    T = Timing(torch, np)
    names = {0: "bnn: v_xor_b32(s,v) + v_bcnt_u32_b32", 1: "tnn: v_and_b32(s,v) + v_bitop3_b32(s,v,v) + 2 x v_bcnt_u32_b32",
             2: "tbn: v_bitop3_b32(s,v,v) + v_bcnt_u32_b32", 3: "v_xor_b32(v,v)", 4: "v_and_b32(s,v)",
             5: "v_bitop3_b32(s,v,v)", 6: "v_bcnt_u32_b32"}
    rows = []
    for mix in range(7):
        for waves in (1, 2, 4, 5, 6, 8):
            r, _ = calibrate_valu(T, torch, np, lb, mixes=(mix,), waves=waves, iters=4096)
            rows.append({"mix": names[mix], "waves_per_simd": waves, **r[mix]})
    print(json.dumps({"scenario": "VALU issue rates (register-only chains, every SIMD busy)",
                      "nominal_tops_64_lanes_per_clk_per_cu_2p4ghz": VALU_NOMINAL_TOPS, "rows": rows}), flush=True)
    return 0


def grid_measure(T, torch, np, lb, synth, with_library=True):
    """The paper's timing experiment (Section IV-B) on this hardware: height x width x depth over
    {72,120,240,360} x {24,48,72,96} x {128,256,384,512}, operands pre-packed, one GEMM per launch (kernel time from
    HIP-graph replays) and the same 64 products as ONE grouped launch per algorithm.  Returns the matrix
    mean_over_shapes(T_row / T_col) like the paper's Table III, launch for launch and group for group."""
    algos = ["int8_mfma", "tnn", "tbn", "bnn"] + (["library_int8"] if with_library else [])
    times = {a: [] for a in algos}
    shapes = synth.paper_shape_grid()
    packed = {k: [] for k in ("tnn", "tbn", "bnn")}
    raw = []
    for idx, (H, W, D) in enumerate(shapes):
        for kind in ("tnn", "tbn", "bnn"):
            A, B = synth.make_custom(kind, H, W, D, seed=1000 + idx)
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            Ap, Bp = lb.pack_a(kind, dA), lb.pack_b(kind, dB)
            packed[kind].append((Ap, Bp))
            C = torch.empty((H, W), dtype=torch.int32, device="cuda")
            times[kind].append(T.graph(None, lambda: lb.gemm(kind, H, W, D, Ap, Bp, C, W), 10, 5))
            if kind == "tnn":
                raw.append((dA, dB))
                times["int8_mfma"].append(T.graph(None, lambda: lb.gemm_i8_mfma(H, W, D, dA, D, dB, W, C, W), 10, 5))
                if with_library:
                    try:
                        times["library_int8"].append(T.graph(None, lambda: torch._int_mm(dA, dB, out=C), 10, 5))
                    except Exception:
                        times["library_int8"].append(float("nan"))
    ratio = {b: {a: float(np.mean(np.array(times[b]) / np.array(times[a]))) for a in algos} for b in algos}
    grouped = {}
    total_ops = float(sum(2 * H * W * D for (H, W, D) in shapes))
    gt = {}
    for kind in ("tnn", "tbn", "bnn"):
        grp = lb.GemmGroup(kind, packed[kind], shapes)
        t = T.graph(f"grid_grouped_{kind}", grp.run, 10)
        gt[kind] = t
        grouped[kind] = {"all_64_shapes_us": t * 1e6, "workgroups": grp.workgroups, "tops": total_ops / t / 1e12,
                         "speedup_vs_one_launch_per_shape": float(np.sum(times[kind]) / t)}
    if hasattr(lb, "I8Group"):
        grp8 = lb.I8Group(raw, shapes)
        t = T.graph("grid_grouped_int8_mfma", grp8.run, 10)
        gt["int8_mfma"] = t
        grouped["int8_mfma"] = {"all_64_shapes_us": t * 1e6, "workgroups": grp8.workgroups, "tops": total_ops / t / 1e12,
                                "speedup_vs_one_launch_per_shape": float(np.sum(times["int8_mfma"]) / t)}
    return {"scenario": "paper shape grid (Section IV-B), 64 shapes, pre-packed operands",
            "mean_time_us_one_launch_per_shape": {a: float(np.mean(times[a]) * 1e6) for a in algos},
            "grouped_launch": grouped,
            "ratio_mean_Trow_over_Tcol_one_launch_per_shape": ratio,
            "ratio_Trow_over_Tcol_grouped_launches": {b: {a: gt[b] / gt[a] for a in gt} for b in gt},
            "paper_table3_on_cortex_a73": {"U8/TNN": 2.51, "U8/TBN": 2.60, "U8/BNN": 7.52, "TNN/BNN": 2.99,
                                           "TBN/BNN": 2.90, "TNN/TBN": 1.03}}


def random_packed(torch, rows, KW, ternary, seed):
    """A packed operand of legal codes drawn on the device (timing only: no int8 source is materialised)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    lim = 2 ** 62
    if not ternary:
        return torch.randint(-lim, lim, (rows * KW,), dtype=torch.int64, device="cuda", generator=g)
    r = torch.randint(-lim, lim, (rows * KW, 2), dtype=torch.int64, device="cuda", generator=g)
    plus = r[:, 0] & r[:, 1]
    minus = ~r[:, 0] & r[:, 1]          # disjoint from plus: the code (1,1) never occurs
    return torch.stack((plus, minus), dim=1).reshape(-1).contiguous()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary measurements")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scenario", choices=["headline", "skinny", "small", "grid", "valu-rates"], default="headline",
                    help="headline: the benchmark proper.  skinny / small: launch patterns for rocprofv3 "
                         "(cfg5 cold/warm per skinny configuration; cfg1-3 per tile variant); they print no metric.  "
                         "grid: the paper's 64-shape timing grid alone.  valu-rates: issue rates of the kernels' "
                         "instruction mixes per occupancy")
    ap.add_argument("--all-variants", action="store_true", help="with --scenario: loop over every kernel variant")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM bytes) so that profiler byte counters "
                         "collected over this command can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2205_09120_amd import binding as lb
    from paper_2205_09120_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    lb.lib()  # raises if the HIP library is missing
    T = Timing(torch, np)

    if args.scenario == "grid":
        print(json.dumps(grid_measure(T, torch, np, lb, synth)), flush=True)
        return 0
    if args.scenario == "valu-rates":
        return valu_rates_scenario(torch, np, lb)
    if args.scenario != "headline":
        return trace_scenario(args, torch, lb, synth)

    w = synth.WORKLOADS[synth.HEADLINE]
    A, B = synth.make_inputs(w)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    M, N, K = w.M, w.N, w.K
    Ap = torch.empty(lb.packed_ternary_bytes(M, K) // 8, dtype=torch.int64, device="cuda")
    Bp = torch.empty(lb.packed_ternary_bytes(N, K) // 8, dtype=torch.int64, device="cuda")
    C = torch.empty((M, N), dtype=torch.int32, device="cuda")

    def step(ev=None):
        if ev is not None:
            ev[0].record()
        lb.pack_ternary(dA, M, K, K, 1, Ap)
        lb.pack_ternary(dB, N, K, 1, N, Bp)
        if ev is not None:
            ev[1].record()
        lb.gemm_tnn(M, N, K, Ap, Bp, C, N)
        if ev is not None:
            ev[2].record()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)      # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    step_s = wall / args.steps
    gemm_ms = np.array([b.elapsed_time(c) for a, b, c in evs])
    step_ms = np.array([a.elapsed_time(c) for a, b, c in evs])
    gemm_s = float(gemm_ms.mean()) * 1e-3

    # ceiling of the ternary kernel: the rate its own four instructions reach on registers with every wave slot busy
    calib, sink = calibrate_valu(T, torch, np, lb)
    peak = calib["tnn"]["tops_best"]
    lane_ops = M * N * (K / 32.0) * LANE_INSTR["tnn"]
    achieved = lane_ops / gemm_s / 1e12
    traffic, tsrc = None, None
    tf = os.path.join(ROOT, "profiles", "gemm_tnn_cfg4_hbm_traffic.txt")
    if os.path.exists(tf):
        for line in open(tf):
            if line.startswith("traffic_bytes_per_launch"):
                traffic, tsrc = float(line.split()[1]), "profiles/gemm_tnn_cfg4_hbm_traffic.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE)"
    out = {
        "metric": "effective TOPS (2*M*N*K/s), TNN GEMM incl. packing of both operands",
        "value": w.ops / step_s / 1e12,
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": step_s * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": w.name, "kind": "tnn", "M": M, "N": N, "K": K, "seed": w.seed,
                   "step": "pack_ternary(A) + pack_ternary(B) + gemm_tnn", "p_zero": w.p0_a},
        "roofline": {"bound": "alu", "kernel": "gemm_tnn (gemm_popc_kernel)", "achieved": achieved,
                     "peak": peak, "unit": "TOP/s (32-bit VALU lane-instructions)",
                     "frac": achieved / peak, "traffic": traffic, "traffic_source": tsrc,
                     "peak_basis": "measured in this run: register-only chains of the kernel's own four instructions "
                                   "(v_and_b32 and v_bitop3_b32 with a scalar source, 2 x v_bcnt_u32_b32), 8 waves on "
                                   "every SIMD, best of %d launches" % BATCHES,
                     "peak_nominal_64_lanes_per_clk_per_cu_at_2p4ghz": VALU_NOMINAL_TOPS,
                     "frac_of_nominal": achieved / VALU_NOMINAL_TOPS,
                     "clock_mhz_under_load": calib["tnn"]["clock_mhz_under_load"],
                     "lane_instr_per_output_per_32_depth": LANE_INSTR["tnn"], "kernel_ms": gemm_s * 1e3,
                     "kernel_ms_median": float(np.median(gemm_ms)), "kernel_ms_min": float(gemm_ms.min())},
    }

    extra = {"device_ms_per_step": {"median": float(np.median(step_ms)), "min": float(step_ms.min()),
                                    "mean": float(step_ms.mean())},
             "gemm_only_tops": w.ops / gemm_s / 1e12,
             "calibration": {"valu_mix_rates": calib, "valu_tops_nominal": VALU_NOMINAL_TOPS}}

    if not args.no_extra:
        big = 1 << 31
        s_buf = torch.empty(big, dtype=torch.uint8, device="cuda").fill_(3)
        d_buf = torch.empty(big, dtype=torch.uint8, device="cuda")
        tr = T.dev("calib_hbm_read_2GiB", lambda: lb.lb_calib_stream(0, s_buf, None, big, sink), 1)
        tw = T.dev("calib_hbm_write_2GiB", lambda: lb.lb_calib_stream(1, None, d_buf, big, sink), 1)
        tc = T.dev("calib_hbm_copy_2GiB", lambda: lb.lb_calib_stream(2, s_buf, d_buf, big, sink), 1)
        del s_buf, d_buf
        extra["calibration"].update({"hbm_read_gbs": big / tr / 1e9, "hbm_write_gbs": big / tw / 1e9,
                                     "hbm_copy_gbs_read_plus_write": 2 * big / tc / 1e9,
                                     "hbm_gbs_published": HBM_PEAK_GBS})
        # pack kernels: int8 bytes read + packed bytes written against the HBM peak
        packs = {}
        tpa = T.dev("pack_ternary_A", lambda: lb.pack_ternary(dA, M, K, K, 1, Ap), 10)
        tpb = T.dev("pack_ternary_B", lambda: lb.pack_ternary(dB, N, K, 1, N, Bp), 3)
        packs["ternary_A_depth_contiguous"] = {"us": tpa * 1e6, "gbs": (A.nbytes + Ap.numel() * 8) / tpa / 1e9}
        packs["ternary_B_depth_strided"] = {"us": tpb * 1e6, "gbs": (B.nbytes + Bp.numel() * 8) / tpb / 1e9}
        Bb = torch.empty(lb.packed_binary_bytes(N, K) // 8, dtype=torch.int64, device="cuda")
        tbb = T.dev("pack_binary_B", lambda: lb.pack_binary(dB, N, K, 1, N, Bb), 3)
        packs["binary_B_depth_strided"] = {"us": tbb * 1e6, "gbs": (B.nbytes + Bb.numel() * 8) / tbb / 1e9}
        # the same bytes as a depth-contiguous source (N x K row-major view of the buffer: timing only)
        tbc = T.dev("pack_ternary_B_as_contig", lambda: lb.pack_ternary(dB, N, K, K, 1, Bp), 3)
        tbcb = T.dev("pack_binary_B_as_contig", lambda: lb.pack_binary(dB, N, K, K, 1, Bb), 3)
        packs["ternary_50176x4608_depth_contiguous"] = {"us": tbc * 1e6, "gbs": (B.nbytes + Bp.numel() * 8) / tbc / 1e9}
        packs["binary_50176x4608_depth_contiguous"] = {"us": tbcb * 1e6, "gbs": (B.nbytes + Bb.numel() * 8) / tbcb / 1e9}
        del Bb
        # the cfg4 source (231 MB) fits the 256 MB last-level cache, so back-to-back calls on it are partly served from
        # there; a source of 461 MB (100000 strings of the same depth) shows the rate from HBM proper
        big_rows = 100000
        big_src = torch.randint(-1, 2, (K, big_rows), dtype=torch.int8, device="cuda")
        big_dst = torch.empty(lb.packed_ternary_bytes(big_rows, K) // 8, dtype=torch.int64, device="cuda")
        tbig = T.dev("pack_ternary_100000x4608_strided", lambda: lb.pack_ternary(big_src, big_rows, K, 1, big_rows, big_dst), 2)
        packs["ternary_100000x4608_depth_strided_beyond_last_level_cache"] = {
            "us": tbig * 1e6, "gbs": (big_src.numel() + big_dst.numel() * 8) / tbig / 1e9}
        del big_src, big_dst
        for v in packs.values():
            v["frac_of_hbm_peak"] = v["gbs"] / HBM_PEAK_GBS
        lb.pack_ternary(dB, N, K, 1, N, Bp)  # restore the real operand
        extra["pack"] = packs
        extra["pack_a_us"], extra["pack_b_us"] = tpa * 1e6, tpb * 1e6
        extra["pack_b_gbs"] = packs["ternary_B_depth_strided"]["gbs"]
        # product with the activation threshold fused into the epilogue (packed ternary output instead of int32 C)
        qlo = torch.full((M,), -20, dtype=torch.int32, device="cuda")
        qhi = torch.full((M,), 20, dtype=torch.int32, device="cuda")
        qout = torch.empty(lb.packed_ternary_bytes(N, M) // 8, dtype=torch.int64, device="cuda")
        trq = T.dev("gemm_requant_ternary", lambda: lb.gemm_requant("tnn", 2, M, N, K, Ap, Bp, qlo, qhi, qout), 2)
        extra["gemm_requant_ternary_ms"] = trq * 1e3
        extra["gemm_requant_ternary_tops"] = w.ops / trq / 1e12
        del qout
        # convolution lowering on packed words: the same right operand built from a channel-packed 16x56x56x512
        # feature map (pack the map, gather words) instead of packing the unrolled 4608 x 50176 int8 matrix
        nb, FH, FW, FC = 16, 56, 56, 512
        fmap = torch.from_numpy(synth.draw_ternary(np.random.default_rng(w.seed), (nb * FH * FW, FC), w.p0_b)).cuda()
        Fp = torch.empty(lb.packed_ternary_bytes(nb * FH * FW, FC) // 8, dtype=torch.int64, device="cuda")

        def conv_step():
            lb.pack_ternary(dA, M, K, K, 1, Ap)
            lb.pack_ternary(fmap, nb * FH * FW, FC, FC, 1, Fp)
            lb.im2col_packed(Fp, 2, nb, FH, FW, FC, 3, 3, 1, 1, 1, 1, Bp)
            lb.gemm_tnn(M, N, K, Ap, Bp, C, N)

        tfm = T.dev("pack_feature_map", lambda: lb.pack_ternary(fmap, nb * FH * FW, FC, FC, 1, Fp), 10)
        tic = T.dev("im2col_packed", lambda: lb.im2col_packed(Fp, 2, nb, FH, FW, FC, 3, 3, 1, 1, 1, 1, Bp), 5)
        tcs = T.dev("conv_step", conv_step, 2)
        extra["conv_lowering_on_packed_words"] = {"pack_feature_map_us": tfm * 1e6, "im2col_packed_us": tic * 1e6,
                                                  "step_ms": tcs * 1e3, "step_tops": w.ops / tcs / 1e12}
        if hasattr(lb, "conv_gemm"):
            Cc = torch.empty((M, N), dtype=torch.int32, device="cuda")

            def conv_fused():
                lb.pack_ternary(dA, M, K, K, 1, Ap)
                lb.pack_ternary(fmap, nb * FH * FW, FC, FC, 1, Fp)
                lb.conv_gemm("tnn", M, Ap, Fp, nb, FH, FW, FC, 3, 3, 1, 1, 1, 1, Cc, N)

            tcg = T.dev("conv_gemm_only", lambda: lb.conv_gemm("tnn", M, Ap, Fp, nb, FH, FW, FC, 3, 3, 1, 1, 1, 1, Cc, N), 2)
            tcf = T.dev("conv_gemm_step", conv_fused, 2)
            extra["conv_implicit_gemm"] = {"gemm_ms": tcg * 1e3, "step_ms": tcf * 1e3, "step_tops": w.ops / tcf / 1e12,
                                           "gemm_only_ms_on_materialised_operand": gemm_s * 1e3}
            del Cc
        del fmap, Fp
        lb.pack_ternary(dB, N, K, 1, N, Bp)
        # matrix-core comparators last: the clock stays low for a while after MFMA-heavy kernels, which would
        # otherwise colour the VALU-bound measurements above
        ti8 = T.dev("gemm_i8_mfma_cfg4", lambda: lb.gemm_i8_mfma(M, N, K, dA, K, dB, N, C, N), 3)
        extra["int8_mfma_tops"] = w.ops / ti8 / 1e12
        extra["int8_mfma_frac_of_int8_mfma_peak"] = w.ops / ti8 / 5.0e15
        extra["gemm_tnn_speedup_vs_int8_mfma"] = ti8 / gemm_s
        # the same comparator with unsigned operands and zero points (eq. (3) corrections in the epilogue)
        uA, uB = (dA + 1).to(torch.uint8), (dB + 1).to(torch.uint8)      # {-1,0,1} -> {0,1,2}, zero point 1
        tu8 = T.dev("gemm_u8_mfma_cfg4", lambda: lb.gemm_u8_mfma(M, N, K, uA, K, uB, N, 1, 1, C, N), 3)
        extra["u8_zero_point_mfma_tops"] = w.ops / tu8 / 1e12
        # 4-bit stand-in for the paper's U4: the same values ({0,1,2}, zero point 1) packed as 6-bit floats in
        # matrix-core fragment order, multiplied on the scaled 6-bit float matrix instruction
        uAp, usA = lb.pack_u4(uA, M, K, K, 1)
        uBp, usB = lb.pack_u4(uB, N, K, 1, N)
        tu4 = T.dev("gemm_u4_mfma_cfg4", lambda: lb.gemm_u4_mfma(M, N, K, uAp, usA, uBp, usB, 1, 1, C, N), 3)
        tu4pb = T.dev("pack_u4_B", lambda: lb.pack_u4(uB, N, K, 1, N, uBp, usB), 2)
        extra["u4_fp6_mfma"] = {"gemm_tops": w.ops / tu4 / 1e12, "gemm_ms": tu4 * 1e3, "pack_b_ms": tu4pb * 1e3,
                                "frac_of_fp6_mfma_peak": w.ops / tu4 / 10.1e15,
                                "speedup_vs_int8_mfma": ti8 / tu4, "gemm_tnn_speed_relative": tu4 / gemm_s}
        del uA, uB, uAp, usA, uBp, usB
        # the same ternary operands as 4-bit floats on the matrix cores (not the paper's method: what this chip's
        # low-precision matrix instruction does with them); step = pack A + pack B + product, like `value`
        tAp, tBp = lb.pack_t4(dA, M, K, K, 1), lb.pack_t4(dB, N, K, 1, N)

        def t4_step():
            lb.pack_t4(dA, M, K, K, 1, tAp)
            lb.pack_t4(dB, N, K, 1, N, tBp)
            lb.gemm_t4_mfma(M, N, K, tAp, tBp, C, N)

        tt4 = T.dev("gemm_t4_mfma_cfg4", lambda: lb.gemm_t4_mfma(M, N, K, tAp, tBp, C, N), 3)
        tt4s = T.dev("t4_step", t4_step, 2)
        extra["fp4_mfma_same_operands"] = {"gemm_tops": w.ops / tt4 / 1e12, "gemm_ms": tt4 * 1e3,
                                           "step_incl_packing_tops": w.ops / tt4s / 1e12, "step_ms": tt4s * 1e3,
                                           "frac_of_fp4_mfma_peak": w.ops / tt4 / 10.1e15,
                                           "speedup_vs_gemm_tnn": gemm_s / tt4, "speedup_vs_int8_mfma": ti8 / tt4}
        del tAp, tBp
        # context only: the vendor library's int8 GEMM (hipBLASLt behind torch._int_mm) on the same matrices
        try:
            torch._int_mm(dA, dB)
            tlib = T.dev("library_int8_cfg4", lambda: torch._int_mm(dA, dB), 2)
            extra["library_int8_gemm_tops"] = w.ops / tlib / 1e12
            extra["gemm_tnn_speedup_vs_faster_int8_kernel"] = min(ti8, tlib) / gemm_s
        except Exception as e:  # not available on every build
            extra["library_int8_gemm_tops"] = None
            extra["library_int8_gemm_error"] = str(e)[:120]
        others = {}
        del dB, Bp, C
        for name, ww in synth.WORKLOADS.items():
            if name == w.name:
                continue
            a_, b_ = synth.make_inputs(ww)
            da, db = torch.from_numpy(a_).cuda(), torch.from_numpy(b_).cuda()
            ap_, bp_ = lb.pack_a(ww.kind, da), lb.pack_b(ww.kind, db)
            c_ = torch.empty((ww.M, ww.N), dtype=torch.int32, device="cuda")
            t = T.graph(f"{name}_gemm_warm", lambda: lb.gemm(ww.kind, ww.M, ww.N, ww.K, ap_, bp_, c_, ww.N), 20)
            t8 = T.graph(f"{name}_int8_mfma", lambda: lb.gemm_i8_mfma(ww.M, ww.N, ww.K, da, ww.K, db, ww.N, c_, ww.N), 20)
            # the vendor library's int8 GEMM on the same operands, timed the same way (None where it refuses the shape
            # or cannot be captured); the speed-up is quoted against the faster of the two 8-bit kernels
            try:
                tlib = T.graph(f"{name}_library_int8", lambda: torch._int_mm(da, db, out=c_), 20)
            except Exception:
                tlib = None
            # the same operands as 4-bit floats on the matrix cores (second comparison point)
            ta_, tb_ = lb.pack_t4(da, ww.M, ww.K, ww.K, 1), lb.pack_t4(db, ww.N, ww.K, 1, ww.N)
            t4 = T.graph(f"{name}_fp4_mfma", lambda: lb.gemm_t4_mfma(ww.M, ww.N, ww.K, ta_, tb_, c_, ww.N), 20)
            del ta_, tb_
            packed_bytes = (ap_.numel() + bp_.numel()) * 8 + c_.numel() * 4
            mixpeak = calib[ww.kind]["tops_best"]
            valu_t = ww.M * ww.N * (ww.K / 32.0) * LANE_INSTR[ww.kind] / t / 1e12
            others[name] = {"gemm_us": t * 1e6, "gemm_us_min": T.table[f"{name}_gemm_warm"]["min"],
                            "tops": ww.ops / t / 1e12, "int8_mfma_us": t8 * 1e6,
                            "speedup_vs_int8_mfma": t8 / t,
                            "library_int8_us": None if tlib is None else tlib * 1e6,
                            "speedup_vs_faster_int8_kernel": (t8 if tlib is None else min(t8, tlib)) / t,
                            "fp4_mfma_us": t4 * 1e6, "speedup_vs_fp4_mfma": t4 / t,
                            "valu_frac": valu_t / mixpeak, "valu_frac_of_nominal": valu_t / VALU_NOMINAL_TOPS,
                            "hbm_frac": packed_bytes / t / 1e9 / HBM_PEAK_GBS}
            if name.startswith("cfg5_"):
                # cold operand: rotate over enough copies of packed A to exceed the 256 MB last-level cache
                ncopy = 24 if ww.kind != "bnn" else 48
                copies = [ap_.clone() for _ in range(ncopy)]
                it = iter(range(10 ** 9))
                cold = T.graph(f"{name}_gemm_cold", lambda: lb.gemm(ww.kind, ww.M, ww.N, ww.K, copies[next(it) % ncopy],
                                                                     bp_, c_, ww.N), ncopy)
                # the floor for one launch at this size: kernels that only read the same cold bytes, several grids
                nbytes = copies[0].numel() * 8
                floors = {}
                for blocks in (256, 512, 1024, 2048, 4096):
                    floors[str(blocks)] = T.graph(f"{name}_read_only_{blocks}_blocks",
                                                  lambda: lb.lb_calib_stream(0, copies[next(it) % ncopy], None, nbytes,
                                                                             sink, blocks), ncopy) * 1e6
                del copies
                others[name]["gemm_us_cold_operand"] = cold * 1e6
                others[name]["gemm_us_cold_operand_min"] = T.table[f"{name}_gemm_cold"]["min"]
                others[name]["hbm_frac_cold_operand"] = packed_bytes / cold / 1e9 / HBM_PEAK_GBS
                others[name]["read_only_kernel_same_cold_bytes_us_by_grid"] = floors
                others[name]["read_only_kernel_same_cold_bytes_us"] = min(floors.values())
        extra["other_configs_gemm_only_warm"] = others
        # the skinny kernel on a stream long enough to show its rate: M = 131072 rows of depth 16384 against 8 columns
        # (512 MiB ternary / 256 MiB binary, beyond every cache; operands drawn on the device as legal packed codes)
        longs = {}
        for kind in ("tnn", "tbn", "bnn"):
            m_, n_, k_ = 131072, 8, 16384
            kw = k_ // 64
            xp = random_packed(torch, m_, kw, kind != "bnn", 5)
            yp = random_packed(torch, n_, kw, kind == "tnn", 6)
            c_ = torch.empty((m_, n_), dtype=torch.int32, device="cuda")
            t = T.dev(f"skinny_long_{kind}", lambda: lb.gemm(kind, m_, n_, k_, xp, yp, c_, n_), 2, BATCHES)
            nbytes = (xp.numel() + yp.numel()) * 8 + c_.numel() * 4
            longs[f"{kind}_{m_}x{n_}x{k_}"] = {"us": t * 1e6, "us_min": T.table[f"skinny_long_{kind}"]["min"],
                                              "gbs": nbytes / t / 1e9, "hbm_frac": nbytes / t / 1e9 / HBM_PEAK_GBS,
                                              "plan": lb.lb_describe_plan(kind, m_, n_, k_)}
            del xp, yp, c_
        extra["skinny_long_stream"] = longs
        # mid-size popcount products (10 - 250 us): the shapes where partial rounds of tiles cost most
        mids = {}
        for kind in ("tnn", "tbn", "bnn"):
            for (m_, n_, k_) in ((1024, 12544, 4608), (512, 12544, 2304), (2048, 6272, 1152)):
                kw = k_ // 64
                xp = random_packed(torch, m_, kw, kind != "bnn", 7)
                yp = random_packed(torch, n_, kw, kind == "tnn", 8)
                c_ = torch.empty((m_, n_), dtype=torch.int32, device="cuda")
                key = f"{kind}_{m_}x{n_}x{k_}"
                t = T.graph(f"mid_{key}", lambda: lb.gemm(kind, m_, n_, k_, xp, yp, c_, n_), 5)
                valu_t = m_ * n_ * (k_ / 32.0) * LANE_INSTR[kind] / t / 1e12
                mids[key] = {"gemm_us": t * 1e6, "tops": 2.0 * m_ * n_ * k_ / t / 1e12,
                             "valu_frac": valu_t / calib[kind]["tops_best"], "plan": lb.lb_describe_plan(kind, m_, n_, k_)}
                del xp, yp, c_
        extra["mid_size_products"] = mids
        # shapes outside the configurations that exercise the other dispatch paths (graph replay, operands warm)
        paths = {}
        for kind, (m_, n_, k_) in (("tnn", (100000, 16, 576)), ("tbn", (8, 50176, 4608)), ("tnn", (128, 128, 16384)),
                                   ("bnn", (64, 64, 65536)), ("tbn", (8, 4096, 16384))):
            a_, b_ = synth.make_custom(kind, m_, n_, k_, seed=77)
            ap_, bp_ = lb.pack_a(kind, torch.from_numpy(a_).cuda()), lb.pack_b(kind, torch.from_numpy(b_).cuda())
            c_ = torch.empty((m_, n_), dtype=torch.int32, device="cuda")
            t = T.graph(f"path_{kind}_{m_}x{n_}x{k_}", lambda: lb.gemm(kind, m_, n_, k_, ap_, bp_, c_, n_), 10)
            paths[f"{kind}_{m_}x{n_}x{k_}"] = {"gemm_us": t * 1e6, "tops": 2.0 * m_ * n_ * k_ / t / 1e12,
                                              "plan": lb.lb_describe_plan(kind, m_, n_, k_)}
        extra["dispatch_paths"] = paths
        # the paper's own 64-shape grid: TNN : TBN : BNN : int8 ratios in the manner of Table III
        extra["paper_shape_grid"] = grid_measure(T, torch, np, lb, synth, with_library=False)
    extra["timing_us"] = T.table
    out["extra"] = extra

    if not args.no_cpu_baseline:
        from oracle import oracle
        rows = 32
        t0 = time.perf_counter()
        _, used = oracle.gemm_threads(np.ascontiguousarray(A[:rows]), B)
        probe = time.perf_counter() - t0
        rows = int(min(M, max(32, rows * 12.0 / max(probe, 1e-3))))
        t0 = time.perf_counter()
        _, used = oracle.gemm_threads(np.ascontiguousarray(A[:rows]), B)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * rows * N * K / dt / 1e12, "unit": "TOPS", "cores": used,
                               "cpu_model": cpu_model(), "host_logical_cpus": os.cpu_count(), "kind": "oracle",
                               "sample": f"first {rows} of {M} rows of A against the full B ({dt:.1f} s of CPU time)"}
        # the same oracle on one thread (last: the thread count set here stays in force for later calls)
        rows1 = int(min(M, max(8, rows * 3 // max(used, 1))))
        t0 = time.perf_counter()
        oracle.gemm_threads(np.ascontiguousarray(A[:rows1]), B, threads=1)
        dt1 = time.perf_counter() - t0
        out["cpu_baseline"]["single_thread"] = {"value": 2.0 * rows1 * N * K / dt1 / 1e12, "unit": "TOPS",
                                                "sample": f"first {rows1} rows ({dt1:.1f} s)"}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
