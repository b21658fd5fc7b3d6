#!/usr/bin/env python3
"""Benchmark of the hot path: single-stream time steps per second versus block
size T, and achieved HBM bandwidth against the 8 TB/s peak.

A "step" of this benchmark (--steps K) is one pass of the whole hot path over
one batch of synthetic input: the full L-step sequence through the whole layer
stack with one block size T, every layer's weights read once per block, in the
library's default schedule (independent (block, layer) stages share a launch;
--flags 1 times the one-launch-per-stage schedule in streaming order).  The headline workload is the benchmark's HBM-roofline
configuration (8-layer SRU, d = 4096, fp32 weights, 1.6 GB, L = 2048) at T = 4.
Inputs and weights are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` = time steps per second of the headline (T given
by --T); `sweep` lists the other block sizes of the same workload; `roofline`
prices the dominant kernel against the HBM peak; `cpu_baseline` is the CPU
oracle timed on this machine's host cores on a bounded sample.
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

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E peak
FP32_PEAK_TFLOPS = 157.3    # MI355X published fp32 (vector / matrix) peak
BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 MFMA peak (8-bit weights are multiplied as bf16)

# HBM bytes per launch of the stage kernel (read + written) measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE and scaled by the copy probe; recorded from the summaries under profiles/ (same commands, same
# workloads, default schedule: a launch holds up to n_layers stages).
MEASURED_TRAFFIC_BYTES = {
    ("C4", 1, "row-major"): 1_608_320_000,    # profiles/stage_valu_kernel_C4_sru8_d4096_T1.txt
    ("C4", 4, "row-major"): 1_594_350_000,    # profiles/stage_valu_kernel_C4_sru8_d4096_T4.txt
    ("C4", 16, "row-major"): 1_555_170_000,    # profiles/stage_mfma_lds_kernel_f32_C4_sru8_d4096_T16.txt
    ("C4", 16, "packed"): 1_555_160_000,    # profiles/stage_mfma_packed_kernel_f32_C4_sru8_d4096_T16.txt
    ("C4", 64, "row-major"): 1_407_210_000,    # profiles/stage_mfma_lds_kernel_f32_C4_sru8_d4096_T64.txt
    ("C4", 64, "packed"): 1_407_300_000,    # profiles/stage_mfma_packed_kernel_f32_C4_sru8_d4096_T64.txt
    ("C4", 128, "packed"): 1_262_680_000,    # profiles/stage_mfma_packed_kernel_f32_C4_sru8_d4096_T128.txt
    ("C5", 16, "packed"): 1_583_890_000,    # profiles/stage_mfma_packed_kernel_bf16_C5_qrnn8_d4096_T16.txt
    ("C5", 64, "packed"): 1_497_710_000,    # profiles/stage_mfma_packed_kernel_bf16_C5_qrnn8_d4096_T64.txt
    # ("C5", 256, "packed"): two kernels share that pass (profiles/stage_mfma_wide_kernel_bf16_C5_qrnn8_d4096_T256.txt)
    ("C5", 256, "row-major"): 1_251_490_000,    # profiles/stage_mfma_lds_kernel_bf16_C5_qrnn8_d4096_T256.txt
    ("X1", 1, "row-major"): 805_270_000,    # profiles/stage_valu_kernel_bf16_X1_sru8_d4096_T1.txt
    ("X2", 1, "row-major"): 404_830_000,    # profiles/stage_valu_kernel_fp8_X2_sru8_d4096_T1.txt
    ("X2", 16, "packed"): 399_850_000,    # profiles/stage_mfma_packed_kernel_fp8_X2_sru8_d4096_T16.txt
    ("X3", 64, "packed"): 772_610_000,    # profiles/stage_mfma_packed_kernel_fp8_X3_qrnn8_d4096_T64.txt
    ("X3", 256, "packed"): 732_460_000,    # profiles/stage_mfma_packed_kernel_fp8_X3_qrnn8_d4096_T256.txt
    ("C2", 4, "row-major"): 50_660_000,    # profiles/stage_valu_kernel_C2_sru4_d1024_T4.txt
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C4", help="workload name prefix (C1..C5, X1..X3)")
    ap.add_argument("--T", type=int, default=4, help="block size of the headline number")
    ap.add_argument("--no-sweep", action="store_true", help="skip the other block sizes")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--flags", type=int, default=0, help="ssrnn flags (schedule / kernel override)")
    ap.add_argument("--packed", action="store_true",
                    help="pre-pack the weights (ssrnn_pack_weights, outside the timed region) and run every block size on the matrix-core kernel")
    ap.add_argument("--cpu-sample-steps", type=int, default=0, help="time steps of the CPU sample (0 = auto)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB three times and exit: the reference "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    return ap.parse_args()


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

    t_gen = time.perf_counter()
    inp = wl.make_inputs(cfg)
    W_host = inp["W"]
    wdt = {"f32": ss.F32, "bf16": ss.BF16, "fp8": ss.FP8}[cfg.wdtype]
    if wdt == ss.FP8:
        W = [ss.Fp8Weights(torch.from_numpy(w.blob()).to(dev), cfg.d, cfg.k) for w in W_host]
        if args.T > 8:
            args.packed = True      # 8-bit weights reach the matrix cores in packed form only
    else:
        W = [torch.from_numpy(w).to(dev) for w in W_host]
    # second copy of the weights in the matrix-core kernel's order (a model-load-time step, outside
    # every timed region); the sweep times both layouts
    W_packed = None
    if ss.packed_weight_bytes(cfg.d, cfg.k, wdt) > 0 and (args.packed or (not args.no_sweep and args.flags == 0)):
        W_packed = [ss.pack_weights(w) for w in W]
    if args.packed:
        assert W_packed is not None, "this workload's weights cannot be packed"
        W = W_packed
        args.flags |= ss.WEIGHTS_PACKED
    if cfg.d_feat:
        feat = torch.from_numpy(inp["feat"]).to(dev)
        P = torch.from_numpy(inp["P"]).to(dev)
        x = ss.linear_forward(P, feat)
    else:
        x = torch.from_numpy(inp["x"]).to(dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    h = torch.empty((cfg.L, cfg.d), dtype=torch.float32, device=dev)
    c_final = torch.empty((cfg.n_layers, cfg.d), dtype=torch.float32, device=dev)
    Tmax = max(max(cfg.Ts), args.T)
    ws = ss.Workspace.for_shape(cfg.n_layers, cfg.d, cfg.k, Tmax, wdt, dev)

    def one_pass(T, packed=False):
        Wl = W_packed if packed else W
        fl = args.flags | (ss.WEIGHTS_PACKED if packed else 0)
        if cfg.cell == "sru":
            ss.sru_forward(Wl, None, x, None, T=T, flags=fl, h=h, c_final=c_final, workspace=ws)
        else:
            ss.qrnn_forward(Wl, None, x, None, None, T=T, k=cfg.k, flags=fl, h=h, c_final=c_final, workspace=ws)

    def measure(T, steps, warmup, packed=False):
        """Returns (seconds per pass by the host clock, ms per pass by HIP events
        recorded on the stream the kernels are launched on)."""
        for _ in range(warmup):
            one_pass(T, packed)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            one_pass(T, packed)
        e1.record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dt / steps, e0.elapsed_time(e1) / steps

    def launches(T):
        """(stages, launches of the stage kernel) of one pass at block size T under args.flags."""
        nblocks = (cfg.L + T - 1) // T
        nstage = cfg.n_layers * nblocks
        sched = args.flags & 3
        if sched == ss.SCHED_PERSISTENT:
            return nstage, 1
        if sched == ss.SCHED_STAGES or cfg.n_layers == 1 or nblocks == 1:
            return nstage, nstage
        # wavefront: one launch per anti-diagonal of the (block, layer) grid, at most 8 stages per launch
        n = 0
        for step in range(nblocks + cfg.n_layers - 1):
            active = min(step, cfg.n_layers - 1) - max(0, step - (nblocks - 1)) + 1
            n += (active + 7) // 8
        return nstage, n

    def row(T, sec, ev_ms):
        nstage = cfg.n_layers * ((cfg.L + T - 1) // T)
        steps_s = cfg.L / sec
        gbs = cfg.algorithmic_bytes_per_step(T) * steps_s / 1e9
        tf = cfg.flops_per_step() * steps_s / 1e12
        return {"T": T, "steps_per_s": round(steps_s, 1), "ms_per_pass": round(sec * 1e3, 3),
                "us_per_stage": round(ev_ms * 1e3 / nstage, 2), "algorithmic_GBps": round(gbs, 1),
                "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "TFLOPps": round(tf, 2)}

    sec, ev_ms = measure(args.T, args.steps, args.warmup)
    head = row(args.T, sec, ev_ms)
    h_head = h[: min(cfg.L, 1024)].clone()

    head["weights"] = "packed" if args.packed else "row-major"
    sweep = []
    if not args.no_sweep:
        for T in cfg.Ts:
            if T == args.T:
                r = dict(head)
            elif wdt == ss.FP8 and T > 8 and not args.packed:
                r = {"T": T, "weights": "row-major", "note": "row-major 8-bit weights run 8 steps per weight pass beyond T = 8 (the T = 8 row); see packed"}
            else:
                s_, e_ = measure(T, max(1, min(args.steps, 2)), 1)
                r = row(T, s_, e_)
                r["weights"] = head["weights"]
            if (args.flags & 3) == 0 and launches(T)[0] != launches(T)[1] and "steps_per_s" in r:
                # the same block size with one launch per stage in streaming (block-major) order
                keep = args.flags
                args.flags |= ss.SCHED_STAGES
                s_, e_ = measure(T, max(1, min(args.steps, 2)), 1)
                args.flags = keep
                ps = row(T, s_, e_)
                r["per_stage_schedule"] = {key: ps[key] for key in ("steps_per_s", "us_per_stage", "frac_hbm_peak")}
            if W_packed is not None and not args.packed:
                # the same block size with pre-packed weights (matrix-core kernel at every T)
                s_, e_ = measure(T, max(1, min(args.steps, 2)), 1, packed=True)
                pk = row(T, s_, e_)
                r["packed"] = {key: pk[key] for key in ("steps_per_s", "us_per_stage", "algorithmic_GBps", "frac_hbm_peak", "TFLOPps")}
            sweep.append(r)

    # dominant kernel: the stage kernel.  Algorithmic bytes of one (block, layer)
    # stage = the layer's weights once + the input block read + the output block
    # written (fp32); a launch holds nstage / nlaunch stages on average.
    # Duration = event time of the timed region / launches in it.
    T = args.T
    nstage, nlaunch = launches(T)
    per_launch = nstage / nlaunch
    stage_bytes = (cfg.weight_bytes_per_layer() + 2 * cfg.d * 4 * T) * per_launch
    stage_flops = 2.0 * 3 * cfg.d * cfg.ncol * T * per_launch
    stage_s = ev_ms * 1e-3 / nlaunch
    traffic = MEASURED_TRAFFIC_BYTES.get((cfg.name[:2], T, "packed" if args.packed else "row-major")) \
        if (args.flags & ~ss.WEIGHTS_PACKED) == 0 else None
    per_stage_schedule = next((r_.get("per_stage_schedule") for r_ in sweep if r_["T"] == T), None)
    common = {"traffic": traffic, "kernel": "stage kernel (a launch holds the independent (block, layer) stages of one step)",
              "launches_per_pass": nlaunch, "stages_per_launch": round(per_launch, 3),
              "avg_launch_us": round(stage_s * 1e6, 2), "us_per_stage": head["us_per_stage"],
              "algorithmic_bytes_per_launch": round(stage_bytes),
              "flops_per_launch": stage_flops,
              "weights_vs_infinity_cache": round(cfg.n_layers * cfg.weight_bytes_per_layer() / 256e6, 2)}
    # fp32 weights cross the ridge (157.3 TFLOP/s against 8 TB/s) near T = 39; bf16 weights stay
    # HBM-bound up to T = 256 (ridge near T = 310 against 2.5 PFLOP/s)
    # 8-bit weights (multiplied as bf16) cross near T = 156
    if (cfg.wdtype == "f32" and T >= 64) or (cfg.wdtype == "fp8" and T >= 160):
        peak = FP32_PEAK_TFLOPS if cfg.wdtype == "f32" else BF16_PEAK_TFLOPS
        achieved = stage_flops / stage_s / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(achieved / peak, 4), **common}
    else:
        achieved = stage_bytes / stage_s / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), **common}

    # What a kernel that only reads reaches on this device, at the stage kernels' launch size: one probe
    # launch per layer's weight matrix, layers in turn so that nothing stays in cache between launches.
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    probe_bufs = [w.buf if wdt == ss.FP8 else w for w in W]
    for w in probe_bufs:
        ss.read_probe(w, sink)
    torch.cuda.synchronize()
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(1, 64 // len(W))
    p0.record()
    for _ in range(reps):
        for w in probe_bufs:
            ss.read_probe(w, sink)
    p1.record()
    torch.cuda.synchronize()
    probe_s = p0.elapsed_time(p1) * 1e-3 / (reps * len(W))
    probe_gbs = cfg.weight_bytes_per_layer() / probe_s / 1e9
    roofline["read_probe_GBps"] = round(probe_gbs, 1)
    roofline["read_probe_us_per_layer"] = round(probe_s * 1e6, 2)
    if roofline["bound"] == "hbm":
        roofline["frac_of_read_probe"] = round(roofline["achieved"] / probe_gbs, 4)

    # The two cache-resident configurations of the benchmark (4 layers of d = 1024, 50 / 101 MB of weights), every
    # block size of theirs in the default schedule: a few milliseconds each, reported next to the headline workload.
    others = []
    if not args.no_sweep and cfg.name.startswith("C4") and args.flags == 0:
        for name in ("C2", "C3"):
            oc = wl.by_name(name)
            oi = wl.make_inputs(oc)
            oW = [torch.from_numpy(w).to(dev) for w in oi["W"]]
            ox = ss.linear_forward(torch.from_numpy(oi["P"]).to(dev), torch.from_numpy(oi["feat"]).to(dev)) if oc.d_feat \
                else torch.from_numpy(oi["x"]).to(dev)
            oh = torch.empty((oc.L, oc.d), dtype=torch.float32, device=dev)
            occ = torch.empty((oc.n_layers, oc.d), dtype=torch.float32, device=dev)
            ows = ss.Workspace.for_shape(oc.n_layers, oc.d, oc.k, max(oc.Ts), ss.F32, dev)
            for T_ in oc.Ts:
                def go():
                    if oc.cell == "sru":
                        ss.sru_forward(oW, None, ox, None, T=T_, h=oh, c_final=occ, workspace=ows)
                    else:
                        ss.qrnn_forward(oW, None, ox, None, None, T=T_, k=oc.k, h=oh, c_final=occ, workspace=ows)
                go()
                torch.cuda.synchronize()
                q0, q1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                q0.record()
                for _ in range(5):
                    go()
                q1.record()
                torch.cuda.synchronize()
                sec_ = q0.elapsed_time(q1) * 1e-3 / 5
                others.append({"workload": oc.name, "T": T_, "steps_per_s": round(oc.L / sec_, 1),
                               "us_per_stage": round(sec_ * 1e6 / (oc.n_layers * ((oc.L + T_ - 1) // T_)), 2),
                               "note": "weights fit the 256 MB Infinity Cache: not priced against the HBM peak"})

    cpu = None
    if not args.no_cpu:
        import oracle
        cores = oracle.num_threads()
        n = args.cpu_sample_steps or (1024 if cfg.d >= 4096 else 1000)   # about 15 s of CPU time on 16 cores at d = 4096
        n = min(n, cfg.L)
        xs = x[:n].cpu().numpy()
        t0 = time.perf_counter()
        if cfg.cell == "sru":
            h_ref, _ = oracle.sru_forward(W_host, None, xs, T=args.T)
        else:
            h_ref, _, _ = oracle.qrnn_forward(W_host, None, xs, T=args.T, k=cfg.k)
        dt = time.perf_counter() - t0
        m = min(n, h_head.shape[0])
        err = float(np.abs(h_head[:m].cpu().numpy().astype(np.float64) - h_ref[:m]).max())
        # the same oracle on one thread, on a short prefix (a few seconds)
        n1 = max(4, min(n, int(4.0 * n / dt / max(cores, 1))))
        oracle.set_num_threads(1)
        try:
            t1 = time.perf_counter()
            if cfg.cell == "sru":
                oracle.sru_forward(W_host, None, xs[:n1], T=args.T)
            else:
                oracle.qrnn_forward(W_host, None, xs[:n1], T=args.T, k=cfg.k)
            dt1 = time.perf_counter() - t1
        finally:
            oracle.set_num_threads(cores)
        cpu = {"value": round(n / dt, 2), "unit": "time steps/s", "cores": cores, "kind": "oracle",
               "single_thread_value": round(n1 / dt1, 2), "single_thread_sample": f"first {n1} time steps, {dt1:.1f} s",
               "sample": f"first {n} of {cfg.L} time steps, all {cfg.n_layers} layers, T={args.T}, "
                         f"{dt:.1f} s of CPU time",
               "gpu_vs_oracle_max_abs_err_on_sample": err}

    out = {
        "metric": "single-stream time steps/sec vs block T; achieved HBM GB/s (% of peak)",
        "value": head["steps_per_s"], "unit": "time steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_pass"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": {"f32": "f32", "bf16": "bf16 weights, f32 accumulate", "fp8": "fp8 (E4M3, row-scaled) weights, f32 accumulate"}[cfg.wdtype],
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers}-layer {cfg.cell.upper()}, d={cfg.d}, k={cfg.k}, "
                               f"L={cfg.L}, batch 1, {cfg.wdtype} weights "
                               f"({cfg.n_layers * cfg.weight_bytes_per_layer() / 1e9:.2f} GB), block T={args.T}",
                   "T": args.T, "schedule": {0: "wavefront (independent stages share a launch)" if nlaunch != nstage else "one launch per stage",
                                             1: "one launch per stage, streaming order", 2: "persistent", 3: "wavefront"}[args.flags & 3],
                   "weights": head["weights"], "flags": args.flags},
        "achieved_hbm_GBps": head["algorithmic_GBps"], "frac_hbm_peak": head["frac_hbm_peak"],
        "per_stage_schedule": per_stage_schedule,
        "sweep": sweep, "roofline": roofline, "cpu_baseline": cpu,
        "cache_resident_configs": others,
        "setup_s": round(t_gen, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
