#!/usr/bin/env python3
"""Benchmark of the hot path: single-stream time steps per second versus block
size T, and achieved HBM bandwidth against the 8 TB/s peak.

A "step" of this benchmark (--steps K) is one pass of the whole hot path over
one batch of synthetic input: the full L-step sequence through the whole layer
stack with one block size T, every layer's weights read once per block.  The
headline workload is the benchmark's HBM-roofline configuration (8-layer SRU,
d = 4096, fp32 weights, 1.6 GB, L = 2048) at T = 4.  Inputs and weights are
resident in HBM before the timed region starts.

Two schedules are timed.  `value` / `roofline`: the library's default for a call
that holds the whole sequence, in which the independent (block, layer) stages of
an anti-diagonal share a launch -- block b+1 enters layer 0 while block b is in
layer 1, so a block's output exists only once n_layers - 1 further blocks of
input have been taken in (`config.lookahead_blocks`).  `roofline_streaming`:
one launch per stage in streaming order, block b through all layers before block
b+1 starts (no look-ahead: the T-step latency of Section 3 of the paper).

Prints ONE JSON line.  `sweep` lists the other block sizes of the headline
workload (each row in the weight layout that is faster there -- row-major, or
re-tiled once by ssrnn_pack_weights -- with the other layout beside it), `c5_sweep` the bf16 matrix-core configuration (8-layer QRNN, d = 4096,
T = 16, 64, 256), `cache_resident_configs` the two configurations whose weights
fit the Infinity Cache, priced against a read probe on resident data,
`lstm_comparator` the paper's comparison network (Eq. 1, Section 3.1) on the same
harness: its speed-up with T levels off below 2;
`cpu_baseline` is the CPU oracle timed on this machine's host cores on a bounded
sample.  Counter figures (`traffic`, `mfma_busy_pct`) are read from the rocprofv3
summaries under profiles/ (profiles/INDEX.md), which were made with this file.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E peak
FP32_PEAK_TFLOPS = 157.3    # MI355X published fp32 (vector / matrix) peak
BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 MFMA peak (8-bit weights are multiplied as bf16)
SWEEP_PASSES = 5            # sweep rows: median of this many timed passes after one warm-up


def profile_index(path=None):
    """Rows of profiles/INDEX.md as dicts (column header -> cell text)."""
    path = path or os.path.join(ROOT, "profiles", "INDEX.md")
    rows, header = [], None
    if not os.path.exists(path):
        return rows
    for line in open(path):
        if not line.startswith("|"):
            continue
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if header is None:
            header = cells
        elif not set(cells[0]) <= set("-: "):
            rows.append(dict(zip(header, cells)))
    return rows


def profile_row(workload: str, T: int, weights: str, schedule: str, rows=None):
    """The INDEX.md row of (workload name prefix, T, weight layout, schedule), or None."""
    for r in (profile_index() if rows is None else rows):
        if r.get("workload", "").startswith(workload) and r.get("T") == str(T) and r.get("weights") == weights \
                and r.get("schedule") == schedule:
            return r
    return None


def _num(cell):
    try:
        return float(cell)
    except (TypeError, ValueError):
        return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C4", help="workload name prefix (C1..C5, X1..X3)")
    ap.add_argument("--T", type=int, default=4, help="block size of the headline number")
    ap.add_argument("--no-sweep", action="store_true", help="skip the other block sizes and the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--headline-only", action="store_true",
                    help="time nothing but the headline configuration (no sweep, no second schedule, no read probe, no CPU "
                         "baseline): the form the rocprofv3 summaries under profiles/ are made with, so that the kernel "
                         "statistics hold launches of one kind")
    ap.add_argument("--flags", type=int, default=0, help="ssrnn flags (schedule / kernel override)")
    ap.add_argument("--packed", action="store_true",
                    help="pre-pack the weights (ssrnn_pack_weights, outside the timed region) and run every block size on the matrix-core kernel")
    ap.add_argument("--cpu-sample-steps", type=int, default=0, help="time steps of the CPU sample (0 = auto)")
    ap.add_argument("--lstm-only", default="", metavar="NAME",
                    help="time only the comparison network NAME (L1, L2) at block size --T (for profiling)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB three times and exit: the reference "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    return ap.parse_args()


class Stack:
    """One workload on the device: weights (row-major and, where a packed form exists, packed), input,
    output buffers and a workspace for its largest block."""

    def __init__(self, ss, wl, torch, cfg, dev, want_packed=True, tmax=0):
        self.ss, self.cfg, self.torch = ss, cfg, torch
        inp = wl.make_inputs(cfg)
        self.W_host = inp["W"]
        self.wdt = {"f32": ss.F32, "bf16": ss.BF16, "fp8": ss.FP8}[cfg.wdtype]
        if self.wdt == ss.FP8:
            self.W = [ss.Fp8Weights(torch.from_numpy(w.blob()).to(dev), cfg.d, cfg.k) for w in self.W_host]
        else:
            self.W = [torch.from_numpy(w).to(dev) for w in self.W_host]
        # second copy of the weights in the matrix-core kernel's order: a model-load-time step, outside every timed region
        self.W_packed = [ss.pack_weights(w) for w in self.W] if want_packed and ss.packed_weight_bytes(cfg.d, cfg.k, self.wdt) > 0 else None
        if cfg.d_feat:
            self.x = ss.linear_forward(torch.from_numpy(inp["P"]).to(dev), torch.from_numpy(inp["feat"]).to(dev))
        else:
            self.x = torch.from_numpy(inp["x"]).to(dev)
        self.h = torch.empty((cfg.L, cfg.d), dtype=torch.float32, device=dev)
        self.c_final = torch.empty((cfg.n_layers, cfg.d), dtype=torch.float32, device=dev)
        self.ws = ss.Workspace.for_shape(cfg.n_layers, cfg.d, cfg.k, max(max(cfg.Ts), tmax), self.wdt, dev)
        torch.cuda.synchronize()

    def one_pass(self, T, flags=0, packed=False):
        ss, cfg = self.ss, self.cfg
        Wl = self.W_packed if packed else self.W
        fl = flags | (ss.WEIGHTS_PACKED if packed else 0)
        if cfg.cell == "sru":
            ss.sru_forward(Wl, None, self.x, None, T=T, flags=fl, h=self.h, c_final=self.c_final, workspace=self.ws)
        else:
            ss.qrnn_forward(Wl, None, self.x, None, None, T=T, k=cfg.k, flags=fl, h=self.h, c_final=self.c_final, workspace=self.ws)

    def time_block(self, T, steps, warmup, flags=0, packed=False):
        """`steps` passes timed as one region: (seconds per pass by the host clock, ms per pass by HIP
        events recorded on the stream the kernels are launched on)."""
        torch = self.torch
        for _ in range(warmup):
            self.one_pass(T, flags, packed)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            self.one_pass(T, flags, packed)
        e1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps, e0.elapsed_time(e1) / steps

    def time_median(self, T, flags=0, packed=False, passes=SWEEP_PASSES):
        """One warm-up, then `passes` passes timed one by one with HIP events: the median, in ms."""
        torch = self.torch
        self.one_pass(T, flags, packed)
        torch.cuda.synchronize()
        ms = []
        for _ in range(passes):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            self.one_pass(T, flags, packed)
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        return statistics.median(ms)

    def launches(self, T, flags=0):
        """(stages, launches of the stage kernel) of one pass at block size T."""
        cfg, ss = self.cfg, self.ss
        nblocks = (cfg.L + T - 1) // T
        nstage = cfg.n_layers * nblocks
        if (flags & 3) == ss.SCHED_STAGES or cfg.n_layers == 1 or nblocks == 1:
            return nstage, nstage
        # wavefront: one launch per anti-diagonal of the (block, layer) grid, at most 8 stages per launch
        n = 0
        for step in range(nblocks + cfg.n_layers - 1):
            active = min(step, cfg.n_layers - 1) - max(0, step - (nblocks - 1)) + 1
            n += (active + 7) // 8
        return nstage, n

    def row(self, T, ms):
        cfg = self.cfg
        nstage = cfg.n_layers * ((cfg.L + T - 1) // T)
        steps_s = cfg.L / (ms * 1e-3)
        gbs = cfg.algorithmic_bytes_per_step(T) * steps_s / 1e9
        tflops = cfg.flops_per_step() * steps_s / 1e12
        r = {"T": T, "steps_per_s": round(steps_s, 1), "ms_per_pass": round(ms, 3),
             "us_per_stage": round(ms * 1e3 / nstage, 2), "algorithmic_GBps": round(gbs, 1),
             "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "TFLOPps": round(tflops, 2)}
        if cfg.wdtype == "f32" and T >= 32:        # near and past the fp32 ridge (T = 39) the matrix cores are the bound
            r["frac_fp32_mfma_peak"] = round(tflops / FP32_PEAK_TFLOPS, 4)
        return r


def roofline_block(stack, T, ev_ms, flags, packed, index_rows):
    """Prices the stage kernel of one timed configuration: algorithmic bytes (or flops) of a launch over its
    average duration (HIP events over the timed region / launches in it)."""
    cfg, ss = stack.cfg, stack.ss
    nstage, nlaunch = stack.launches(T, flags)
    per_launch = nstage / nlaunch
    stage_bytes = (cfg.weight_bytes_per_layer() + 2 * cfg.d * 4 * T) * per_launch
    stage_flops = 2.0 * 3 * cfg.d * cfg.ncol * T * per_launch
    launch_s = ev_ms * 1e-3 / nlaunch
    schedule = "per-stage" if nlaunch == nstage else "wavefront"
    prow = profile_row(cfg.name[:2], T, "packed" if packed else "row-major", schedule, index_rows) \
        if (flags & ~(3 | ss.WEIGHTS_PACKED)) == 0 else None
    common = {"traffic": int(_num(prow["traffic bytes per launch"])) if prow and _num(prow.get("traffic bytes per launch")) else None,
              "traffic_source": ("profiles/" + prow["file"]) if prow else None,
              "kernel": (prow["kernel"] if prow and prow.get("kernel") else "stage kernel"),
              "schedule": schedule, "lookahead_blocks": (cfg.n_layers - 1) if schedule == "wavefront" else 0,
              "launches_per_pass": nlaunch, "stages_per_launch": round(per_launch, 3),
              "avg_launch_us": round(launch_s * 1e6, 2), "us_per_stage": round(ev_ms * 1e3 / nstage, 2),
              "steps_per_s": round(cfg.L / (ev_ms * 1e-3), 1),
              "algorithmic_bytes_per_launch": round(stage_bytes), "flops_per_launch": stage_flops,
              "weights_vs_infinity_cache": round(cfg.n_layers * cfg.weight_bytes_per_layer() / 256e6, 2)}
    # fp32 weights cross the ridge (157.3 TFLOP/s against 8 TB/s) near T = 39; bf16 weights stay HBM-bound up to
    # T = 256 (ridge near T = 310 against 2.5 PFLOP/s); 8-bit weights (multiplied as bf16) cross near T = 156
    if (cfg.wdtype == "f32" and T >= 64) or (cfg.wdtype == "fp8" and T >= 160):
        peak = FP32_PEAK_TFLOPS if cfg.wdtype == "f32" else BF16_PEAK_TFLOPS
        achieved = stage_flops / launch_s / 1e12
        return {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), **common}
    achieved = stage_bytes / launch_s / 1e9
    return {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), **common}


def read_probe_rate(ss, torch, bufs, per_launch, reps_bytes=8e9):
    """GB/s of ssrnn_read_probe launches that hold `per_launch` of the equally long buffers each (the
    shape of a stage launch with that many stages), the best of a few workgroup counts."""
    dev = bufs[0].device
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    nbytes = bufs[0].numel() * bufs[0].element_size()
    groups_of = [bufs[i:i + per_launch] for i in range(0, len(bufs) - per_launch + 1, per_launch)]
    reps = max(1, int(reps_bytes / (nbytes * per_launch * len(groups_of))))
    best = None
    for groups in (64, 128, 256, 512, 1024, 2048):
        for g in groups_of:
            ss.read_probe(g, sink, groups=groups)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            for g in groups_of:
                ss.read_probe(g, sink, groups=groups)
        e1.record()
        torch.cuda.synchronize()
        sec = e0.elapsed_time(e1) * 1e-3 / (reps * len(groups_of))
        cand = {"GBps": round(nbytes * per_launch / sec / 1e9, 1), "us_per_launch": round(sec * 1e6, 2),
                "bytes_per_launch": nbytes * per_launch, "workgroups_per_buffer": groups}
        if best is None or cand["GBps"] > best["GBps"]:
            best = cand
    return best


def lstm_comparator_rows(ss, wl, torch, dev, configs, only_T=None):
    """The paper's comparison network (Eq. 1) timed like the stacks above.  An LSTM's feedback products
    cannot be blocked, so processing T steps at a time saves at most the input products' half of the weight
    traffic (Section 3.1): its speed-up over T = 1 levels off below 2 where the SRU's keeps growing."""
    rows = []
    lib = ss.load_library()
    for lc in configs:
        inp = wl.make_lstm_inputs(lc)
        Wd = [torch.from_numpy(w).to(dev) for w in inp["W"]]
        Ud = [torch.from_numpy(u).to(dev) for u in inp["U"]]
        xd = torch.from_numpy(inp["x"]).to(dev)
        del inp
        base = None
        for T_ in (lc.Ts if only_T is None else (only_T,)):
            ws = ss.Workspace(lib.lstm_workspace_bytes(lc.n_layers, lc.d, T_), dev)
            times = []
            for i in range(1 + 3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ss.lstm_forward(Wd, Ud, None, xd, T=T_, workspace=ws)
                torch.cuda.synchronize()
                if i:
                    times.append(time.perf_counter() - t0)
            sec = sorted(times)[len(times) // 2]
            sps = lc.L / sec
            base = base or sps
            gbps = lc.algorithmic_bytes_per_step(T_) * sps / 1e9
            resident = lc.n_layers * lc.weight_bytes_per_layer() < 256e6
            rows.append({"workload": lc.name, "T": T_, "steps_per_s": round(sps, 1), "ms_per_pass": round(sec * 1e3, 3),
                         "speedup_vs_T1": round(sps / base, 3) if only_T is None else None,
                         "us_per_step_and_layer": round(sec * 1e6 / lc.L / lc.n_layers, 2),
                         "algorithmic_bytes_per_step": int(lc.algorithmic_bytes_per_step(T_)),
                         "algorithmic_GBps": round(gbps, 1),
                         "frac_hbm_peak": None if resident else round(gbps / HBM_PEAK_GBS, 4),
                         "passes": "median of 3"})
        del Wd, Ud, xd
        torch.cuda.empty_cache()
    return rows


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this path is a single-stream, single-GPU kernel; run with --gpus 1 "
              "(sharding across GPUs is not built)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1803_11389_amd as ss
    import workloads as wl

    cfg = wl.by_name(args.config)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.copy_probe:
        n = args.copy_probe * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_MiB": args.copy_probe, "bytes_read_per_copy": n * 4, "bytes_written_per_copy": n * 4}))
        return
    ss.load_library()
    if args.lstm_only:
        lc = [c for c in wl.LSTM_CONFIGS if c.name.startswith(args.lstm_only)]
        assert lc, f"no LSTM workload named {args.lstm_only}"
        print(json.dumps({"lstm_comparator": lstm_comparator_rows(ss, wl, torch, dev, lc[:1], only_T=args.T)}))
        return
    index_rows = profile_index()
    if args.headline_only:
        args.no_sweep = args.no_cpu = True

    t_gen = time.perf_counter()
    wdt_is_fp8 = cfg.wdtype == "fp8"
    if wdt_is_fp8 and args.T > 8:
        args.packed = True      # 8-bit weights reach the matrix cores in packed form only
    sched = args.flags & 3
    stack = Stack(ss, wl, torch, cfg, dev, want_packed=args.packed or not args.no_sweep, tmax=args.T)
    if args.packed:
        assert stack.W_packed is not None, "this workload's weights cannot be packed"
    t_gen = time.perf_counter() - t_gen

    # ---- headline: exactly --steps passes timed as one region
    sec, ev_ms = stack.time_block(args.T, args.steps, args.warmup, args.flags, args.packed)
    head = stack.row(args.T, sec * 1e3)
    head["weights"] = "packed" if args.packed else "row-major"
    h_head = stack.h[: min(cfg.L, 1024)].clone()
    roofline = roofline_block(stack, args.T, ev_ms, args.flags, args.packed, index_rows)

    # ---- the same block size with one launch per stage in streaming order (no look-ahead)
    roofline_streaming = None
    if sched == 0 and roofline["schedule"] == "wavefront" and not args.headline_only:
        _, ev_s = stack.time_block(args.T, max(2, args.steps // 2), 1, args.flags | ss.SCHED_STAGES, args.packed)
        roofline_streaming = roofline_block(stack, args.T, ev_s, args.flags | ss.SCHED_STAGES, args.packed, index_rows)

    sweep = []
    if not args.no_sweep:
        for T in cfg.Ts:
            if wdt_is_fp8 and T > 8 and not args.packed:
                sweep.append({"T": T, "weights": "row-major", "note": "row-major 8-bit weights run 8 steps per weight pass beyond T = 8 (the T = 8 row); see packed"})
                continue
            r = stack.row(T, stack.time_median(T, args.flags, args.packed))
            r["weights"] = head["weights"]
            r["passes"] = f"median of {SWEEP_PASSES}"
            nstage, nlaunch = stack.launches(T, args.flags)
            if sched == 0 and nstage != nlaunch:
                ps = stack.row(T, stack.time_median(T, args.flags | ss.SCHED_STAGES, args.packed))
                r["per_stage_schedule"] = {key: ps[key] for key in ("steps_per_s", "us_per_stage", "frac_hbm_peak")}
                r["per_stage_schedule"]["weights"] = head["weights"]
            if stack.W_packed is not None and not args.packed:
                # the one-time weight pre-pack is part of the path: the row shows the layout that is faster at
                # this block size, the other one beside it
                pk = stack.row(T, stack.time_median(T, args.flags, True))
                keys = tuple(k for k in r if k in ("steps_per_s", "ms_per_pass", "us_per_stage", "algorithmic_GBps",
                                                   "frac_hbm_peak", "TFLOPps", "frac_fp32_mfma_peak"))
                if pk["steps_per_s"] > r["steps_per_s"]:
                    r["row_major"] = {key: r[key] for key in keys}
                    r.update({key: pk[key] for key in keys})
                    r["weights"] = "packed"
                else:
                    r["packed"] = {key: pk[key] for key in keys}
            sweep.append(r)

    # ---- what a kernel that only reads reaches, in launches of the stage launches' shape and size: eight
    # layers per launch (the wavefront schedule's launches) and one layer per launch (the per-stage schedule's)
    probe_bufs = [w.buf if wdt_is_fp8 else w for w in stack.W]
    probe = None if args.headline_only else {
        "wavefront_shaped": read_probe_rate(ss, torch, probe_bufs, min(8, len(probe_bufs))),
        "per_stage_shaped": read_probe_rate(ss, torch, probe_bufs, 1)}
    if probe and roofline["bound"] == "hbm":
        key = "wavefront_shaped" if roofline["schedule"] == "wavefront" else "per_stage_shaped"
        roofline["read_probe_GBps"] = probe[key]["GBps"]
        roofline["frac_of_read_probe"] = round(roofline["achieved"] / probe[key]["GBps"], 4)
    if roofline_streaming and roofline_streaming["bound"] == "hbm":
        roofline_streaming["read_probe_GBps"] = probe["per_stage_shaped"]["GBps"]
        roofline_streaming["frac_of_read_probe"] = round(roofline_streaming["achieved"] / probe["per_stage_shaped"]["GBps"], 4)

    # ---- configuration 5 (bf16 weights on the matrix cores) and the two cache-resident configurations
    c5_sweep, others = [], []
    if not args.no_sweep and cfg.name.startswith("C4") and args.flags == 0 and not args.packed:
        del stack.W_packed
        stack.W_packed = None
        torch.cuda.empty_cache()
        c5 = wl.by_name("C5")
        s5 = Stack(ss, wl, torch, c5, dev)
        for T in c5.Ts:
            r = s5.row(T, s5.time_median(T, 0, True))
            r["weights"] = "packed"
            r["frac_bf16_mfma_peak"] = round(r["TFLOPps"] / BF16_PEAK_TFLOPS, 4)
            ps = s5.row(T, s5.time_median(T, ss.SCHED_STAGES, True))
            r["per_stage_schedule"] = {key: ps[key] for key in ("steps_per_s", "us_per_stage", "frac_hbm_peak", "TFLOPps")}
            rm = s5.row(T, s5.time_median(T, 0, False))
            r["row_major"] = {key: rm[key] for key in ("steps_per_s", "us_per_stage", "frac_hbm_peak", "TFLOPps")}
            prow = profile_row("C5", T, "packed", "wavefront", index_rows)
            r["mfma_busy_pct"] = _num(prow.get("MFMA busy %")) if prow else None
            r["traffic"] = int(_num(prow["traffic bytes per launch"])) if prow and _num(prow.get("traffic bytes per launch")) else None
            r["profile"] = ("profiles/" + prow["file"]) if prow else None
            c5_sweep.append(r)
        # the longest block again on a stream four times as long: with 16 blocks in the sequence the launches
        # at its two ends (fewer than eight stages) weigh 38 rounds of workgroups for 32 rounds' worth of work
        import dataclasses
        long_cfg = dataclasses.replace(c5, L=4 * c5.L)
        s5.cfg = long_cfg
        s5.x = torch.from_numpy(wl.normal(c5.seed, wl.TID_X, (long_cfg.L * c5.d,)).reshape(long_cfg.L, c5.d)).to(dev)
        s5.h = torch.empty((long_cfg.L, c5.d), dtype=torch.float32, device=dev)
        T_long = max(c5.Ts)
        rl_ = s5.row(T_long, s5.time_median(T_long, 0, True, passes=3))
        c5_sweep[-1]["stream_four_times_as_long"] = {"L": long_cfg.L, **{key: rl_[key] for key in
                                                    ("steps_per_s", "us_per_stage", "frac_hbm_peak", "TFLOPps")}}
        del s5
        torch.cuda.empty_cache()
        for name in ("C2", "C3"):
            oc = wl.by_name(name)
            so = Stack(ss, wl, torch, oc, dev, want_packed=True)
            # the weights of the whole stack, read again and again: they stay in the Infinity Cache
            cache_probe = read_probe_rate(ss, torch, so.W, len(so.W), reps_bytes=2e9)
            for T_ in oc.Ts:
                r = so.row(T_, so.time_median(T_))
                weights = "row-major"
                if so.W_packed is not None:          # as in the sweep: the layout that is faster at this block size
                    pk = so.row(T_, so.time_median(T_, 0, True))
                    if pk["steps_per_s"] > r["steps_per_s"]:
                        r, weights = pk, "packed"
                others.append({"workload": oc.name, "T": T_, "weights": weights, "steps_per_s": r["steps_per_s"], "us_per_stage": r["us_per_stage"],
                               "algorithmic_GBps": r["algorithmic_GBps"],
                               "cache_read_probe_GBps": cache_probe["GBps"],
                               "frac_of_cache_read_probe": round(r["algorithmic_GBps"] / cache_probe["GBps"], 4),
                               "note": "weights fit the 256 MB Infinity Cache: priced against a read probe on the resident weights, not against the HBM peak"})
            del so
            torch.cuda.empty_cache()

    # ---- the paper's comparison network (Eq. 1) on the same harness
    lstm_rows = []
    if not args.no_sweep and cfg.name.startswith("C4") and args.flags == 0 and not args.packed:
        lstm_rows = lstm_comparator_rows(ss, wl, torch, dev, wl.LSTM_CONFIGS)

    cpu = None
    if not args.no_cpu:
        import oracle
        cores = oracle.num_threads()
        n = args.cpu_sample_steps or (1024 if cfg.d >= 4096 else 1000)   # about 15 s of CPU time on 16 cores at d = 4096
        n = min(n, cfg.L)
        xs = stack.x[:n].cpu().numpy()
        t0 = time.perf_counter()
        if cfg.cell == "sru":
            h_ref, _ = oracle.sru_forward(stack.W_host, None, xs, T=args.T)
        else:
            h_ref, _, _ = oracle.qrnn_forward(stack.W_host, None, xs, T=args.T, k=cfg.k)
        dt = time.perf_counter() - t0
        m = min(n, h_head.shape[0])
        err = float(np.abs(h_head[:m].cpu().numpy().astype(np.float64) - h_ref[:m]).max())
        # the same oracle on one thread, on a short prefix (a few seconds)
        n1 = max(4, min(n, int(4.0 * n / dt / max(cores, 1))))
        oracle.set_num_threads(1)
        try:
            t1 = time.perf_counter()
            if cfg.cell == "sru":
                oracle.sru_forward(stack.W_host, None, xs[:n1], T=args.T)
            else:
                oracle.qrnn_forward(stack.W_host, None, xs[:n1], T=args.T, k=cfg.k)
            dt1 = time.perf_counter() - t1
        finally:
            oracle.set_num_threads(cores)
        cpu = {"value": round(n / dt, 2), "unit": "time steps/s", "cores": cores, "kind": "oracle",
               "single_thread_value": round(n1 / dt1, 2), "single_thread_sample": f"first {n1} time steps, {dt1:.1f} s",
               "sample": f"first {n} of {cfg.L} time steps, all {cfg.n_layers} layers, T={args.T}, "
                         f"{dt:.1f} s of CPU time",
               "gpu_vs_oracle_max_abs_err_on_sample": err}

    lookahead = roofline["lookahead_blocks"]
    schedule_text = (f"wavefront: the independent (block, layer) stages of an anti-diagonal share a launch; a block's output "
                     f"needs {lookahead} further blocks ({lookahead * args.T} time steps) of input" if roofline["schedule"] == "wavefront"
                     else "one launch per stage, streaming order (no look-ahead)")
    out = {
        "metric": "single-stream time steps/sec vs block T; achieved HBM GB/s (% of peak)",
        "value": head["steps_per_s"], "unit": "time steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_pass"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16 weights, f32 accumulate", "fp8": "fp8 (E4M3, row-scaled) weights, f32 accumulate"}[cfg.wdtype],
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers}-layer {cfg.cell.upper()}, d={cfg.d}, k={cfg.k}, "
                               f"L={cfg.L}, batch 1, {cfg.wdtype} weights "
                               f"({cfg.n_layers * cfg.weight_bytes_per_layer() / 1e9:.2f} GB), block T={args.T}",
                   "T": args.T, "schedule": schedule_text, "lookahead_blocks": lookahead,
                   "weights": head["weights"], "flags": args.flags},
        "achieved_hbm_GBps": head["algorithmic_GBps"], "frac_hbm_peak": head["frac_hbm_peak"],
        "roofline": roofline, "roofline_streaming": roofline_streaming, "read_probe": probe,
        "sweep": sweep, "c5_sweep": c5_sweep, "cache_resident_configs": others, "lstm_comparator": lstm_rows,
        "cpu_baseline": cpu, "setup_s": round(t_gen, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
