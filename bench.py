#!/usr/bin/env python3
"""Benchmark of the stacked-LSTM hot path on one MI355X.

A "step" is one full pass of the hot path over one synthetic batch: lstm_forward followed
by lstm_backward (full BPTT) at the headline shape L=4, I=H=512, B=64, T=100 (the paper's
Table 1 shape, Section 2.5), fp32, inputs resident in HBM before the timed region.

Prints ONE JSON line.  value = TFLOP/s with FLOPs = 3 passes x sum_l 2*4H*(I_l+H)*B*T
(forward, backward-data, backward-weights); the conservative two-pass figure, per-phase
times (HIP events recorded by the library on its launch streams), a roofline object for the
phase that takes the most time, the in-repo unfused baseline and the timed CPU oracle ride
along in the same line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # 256 CU x 256 FLOP/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the rocprofv3 counter passes whose summary is kept under profiles/
    (written by `python -m paper_1604_01946_amd.profile_summary traffic`), or None when no such file names this
    workload and this kernel: a figure recorded for other kernels is never reported."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic_pmc.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None
    k = rec.get("kernels", {}).get(kernel)
    if rec.get("workload") != workload or not k:
        return None
    return int(k["read_bytes"]) + int(k["write_bytes"])


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--path", type=int, default=0, help="LSTM_PATH_* value (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-naive", action="store_true")
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run one 1 GiB device-to-device copy first (reference point for rocprofv3 byte counters)")
    return ap.parse_args()


def phase_bytes(cfg, phase):
    """Algorithmic HBM bytes of the streaming phases (read once + write once)."""
    L, T, B, I, H = cfg.dims
    if phase == "bias_grad":
        return L * T * B * 4 * H * 4 + L * 4 * H * 4
    if phase in ("fwd_pack", "bwd_pack"):
        return 2 * L * 4 * H * H * 4
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no multi-GPU path); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1604_01946_amd import binding as B_
    from paper_1604_01946_amd.inputs import CONFIGS, make_inputs
    from paper_1604_01946_amd.runner import LstmRunner

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B_.library()  # fail loudly if the HIP library is not built

    cfg = CONFIGS[args.config]
    do_bwd = cfg.backward and not args.forward_only
    L, T, B, I, H = cfg.dims
    arrays = make_inputs(cfg, 0)
    r = LstmRunner(cfg.dims, arrays)
    flags = args.path
    path_f = flags or B_.lstm_auto_path(*cfg.dims, 0)
    path_b = flags or B_.lstm_auto_path(*cfg.dims, 1)

    def step():
        B_.check(r.forward(flags=flags), "lstm_forward")
        if do_bwd:
            B_.check(r.backward(flags=flags), "lstm_backward")

    if args.copy_calibration:
        src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # separate forward / backward times and per-phase times (events on the launch streams)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    B_.lstm_profile_enable(1)
    nprof = max(3, min(args.steps, 10))
    fwd_ms = bwd_ms = 0.0
    per_iter = []  # HIP-event time of each of these iterations, synchronised one by one (the paper's protocol, Section 2.1)
    phases = {}
    for _ in range(nprof):
        ev[0].record()
        B_.check(r.forward(flags=flags))
        ev[1].record()
        if do_bwd:
            B_.check(r.backward(flags=flags))
        ev[2].record()
        torch.cuda.synchronize()
        fwd_ms += ev[0].elapsed_time(ev[1]) / nprof
        bwd_ms += ev[1].elapsed_time(ev[2]) / nprof
        per_iter.append(ev[0].elapsed_time(ev[2]))
        st, ph = B_.lstm_profile_read()
        B_.check(st, "lstm_profile_read")
        for k, (m, c, fl, kern) in ph.items():
            a = phases.setdefault(k, [0.0, 0, 0.0, ""])
            a[0] += m / nprof
            a[1], a[2], a[3] = c, fl, kern   # FLOPs as the library counts them for the products the phase really carried
    B_.lstm_profile_enable(0)

    passes = 3 if do_bwd else 1
    flop1 = cfg.flops_per_pass()
    tflops = passes * flop1 / (ms * 1e-3) / 1e12
    tflops_2pass = (2 if do_bwd else 1) * flop1 / (ms * 1e-3) / 1e12

    # roofline of the phase that takes the most time
    dom = max(phases.items(), key=lambda kv: kv[1][0])[0] if phases else None
    if dom and phases[dom][0] <= 0.0:
        dom = None  # the unfused baseline paths record no phases
    roofline = {"bound": "mfma", "achieved": round(tflops, 3), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tflops / PEAK_FP32_MFMA_TFLOPS, 4), "traffic": None, "kernel_phase": "whole_step",
                "launch_intervals": 0, "avg_ms": round(ms, 4)}
    if dom:
        dom_ms, dom_n, fl, kern = phases[dom]
        traffic = recorded_traffic(cfg.name, kern) if flags == 0 else None
        # dependent steps of the recurrence: the layers of one persistent launch advance as a wavefront (T + L - 1
        # steps in a row), every other recurrence runs its L*T cells one after the other
        wave = kern.startswith("pers_") and "L_kernel" not in kern
        dep_steps = (T + L - 1) if wave else L * T
        mfma_us_per_step = fl / (PEAK_FP32_MFMA_TFLOPS * 1e12) * 1e6 / dep_steps if fl else 0.0
        if fl and not (dom.endswith("recurrence") and mfma_us_per_step < 0.5):
            ach = fl / (dom_ms * 1e-3) / 1e12
            roofline = {"bound": "mfma", "achieved": round(ach, 3), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(ach / PEAK_FP32_MFMA_TFLOPS, 4), "traffic": traffic, "kernel_phase": dom, "kernel": kern,
                        "launch_intervals": dom_n, "avg_ms": round(dom_ms, 4)}
        elif fl:
            # a chain of dependent steps whose matrix work takes well under a microsecond each: bound by the hop from
            # step to step, neither by the matrix cores nor by memory bandwidth -- reported as time per dependent step
            us = dom_ms * 1e3 / dep_steps
            roofline = {"bound": "latency", "achieved": round(us, 3), "peak": None, "unit": "us/step", "frac": None,
                        "traffic": traffic, "kernel_phase": dom, "kernel": kern, "dependent_steps": dep_steps,
                        "hbm_gbs": round(traffic / (dom_ms * 1e-3) / 1e9, 1) if traffic else None,
                        "launch_intervals": dom_n, "avg_ms": round(dom_ms, 4)}
        else:
            by = phase_bytes(cfg, dom)
            if by:
                ach = by / (dom_ms * 1e-3) / 1e9
                roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None, "kernel_phase": dom,
                            "launch_intervals": dom_n, "avg_ms": round(dom_ms, 4)}
    phase_report = {}
    for k, (m, c, fl, kern) in phases.items():
        if c == 0:
            continue
        phase_report[k] = {"ms": round(m, 4), "intervals": c}
        if fl:
            phase_report[k].update(kernel=kern, gflop=round(fl / 1e9, 2), tflops=round(fl / (m * 1e-3) / 1e12, 2))

    # in-repo unfused baseline: one kernel per operation, per-gate GEMMs (Section 2.1 starting point)
    naive = None
    if not args.no_naive and flags == 0:
        def nstep():
            B_.check(r.forward(flags=B_.LSTM_PATH_NAIVE))
            if do_bwd:
                B_.check(r.backward(flags=B_.LSTM_PATH_NAIVE))
        nstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            nstep()
        torch.cuda.synchronize()
        nms = (time.perf_counter() - t0) * 1e3 / 3
        naive = {"ms_per_step": round(nms, 3), "speedup_over_naive": round(nms / ms, 2)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lstm_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
        except Exception:
            cores = os.cpu_count()
        # repeat the oracle until about 10 s of wall time have been spent (at least once, at most 20 times)
        reps, cs = 0, 0.0
        while reps < 1 or (cs < 10.0 and reps < 20):
            t0 = time.perf_counter()
            y, hT, cT, res = O.lstm_forward(*cfg.dims, arrays["x"], arrays["h0"], arrays["c0"], arrays["W"],
                                            arrays["R"], arrays["b"])
            if do_bwd:
                O.lstm_backward(*cfg.dims, arrays["x"], arrays["h0"], arrays["c0"], arrays["W"], arrays["R"], res,
                                arrays["dy"], arrays["dhT"], arrays["dcT"])
            cs += time.perf_counter() - t0
            reps += 1
        per = cs / reps
        cpu = {"value": round(passes * flop1 / per / 1e12, 4), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{reps} full {'fwd+bwd' if do_bwd else 'fwd'} iterations of {cfg.name} "
                         f"(fp64 numpy oracle), {per:.2f} s each, {cs:.1f} s in all"}

    out = {
        "metric": "LSTM fwd+bwd fp32 TFLOPS at L=4 H=512 B=64 T=100 (1 GPU)" if args.config == "cfg3" and do_bwd
                  else f"LSTM {'fwd+bwd' if do_bwd else 'fwd'} fp32 TFLOPS ({cfg.name})",
        "value": round(tflops, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: L={L} I={I} H={H} B={B} T={T} {'forward+backward' if do_bwd else 'forward'}",
                   "path_forward": B_.PATH_NAMES[path_f], "path_backward": B_.PATH_NAMES[path_b] if do_bwd else None,
                   "flop_convention": f"{passes} passes x sum_l 2*4H*(I_l+H)*B*T"},
        "tflops_2pass": round(tflops_2pass, 3),
        "us_per_cell": round(ms * 1e3 / (L * T), 3),
        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4),
        "event_ms": {"iterations": len(per_iter), "median": round(sorted(per_iter)[len(per_iter) // 2], 4),
                     "min": round(min(per_iter), 4), "max": round(max(per_iter), 4)},
        "frac_of_fp32_mfma_peak": round(tflops / PEAK_FP32_MFMA_TFLOPS, 4),
        "phases": phase_report,
        "roofline": roofline,
        "unfused_baseline": naive,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    del r
    torch.cuda.synchronize()
    B_.lstm_shutdown()   # helper streams, events and the mapped watchdog page are released before the process ends


if __name__ == "__main__":
    main()
