#!/usr/bin/env python3
"""Throughput of the mixed-precision neural-ODE time stepper on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch: rampde_odeint_fwd
(paper Algorithm 1), the caller-side terminal-loss gradient, rampde_odeint_bwd (paper
Algorithm 2).  Metric: batch * RK-steps per second = B * N / (t_fwd + t_bwd).

Prints ONE JSON line (see the keys below).  `roofline` is measured in a second,
instrumented run of the same K steps (HIP events around every launch of the dominant
kernel class, on the stream the library launches on); `cpu_baseline` times the CPU oracle on
a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0}   # MI355X dense matrix peak
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--grad-t", action="store_true",
                    help="also form the time-grid gradient dL/dt in the backward pass (not part of the headline metric)")
    ap.add_argument("--cpu-steps", type=int, default=0,
                    help="RK steps of the oracle sample (0: the whole grid for the benchmark workload, "
                         "1-2 steps for the larger ones: about 10-30 s of CPU work)")
    ap.add_argument("--calibrate-mib", type=int, default=0,
                    help="before the timed region run ONE plain elementwise copy (read + write) of this many MiB: "
                         "under `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE` its counter value calibrates the HBM byte "
                         "counters of the other kernels")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_23498_amd import binding as rb
    from paper_2510_23498_amd import workloads as wl
    import parity as par

    cfg = wl.CONFIGS[args.config]
    rb.load_library()  # fails loudly when the HIP library is missing
    dev = torch.device("cuda:0")
    theta_np, y0_np, target_np = par.make_inputs(cfg)
    vel, tab, pol = par.gpu_descriptors(cfg)
    tgrid = cfg.tgrid()
    B, N = cfg.B, cfg.N

    theta = torch.from_numpy(theta_np).to(dev)
    y0 = torch.from_numpy(y0_np).to(dev)
    target = None if target_np is None else torch.from_numpy(target_np).to(dev)
    ckpt = torch.empty(vel.ckpt_shape(B, N), dtype=pol.torch_low, device=dev)
    yN = torch.empty_like(y0)
    grad_yN = torch.empty_like(y0)
    grad_y0 = torch.empty_like(y0)
    grad_theta = torch.zeros(rb.rampde_num_params(vel), dtype=torch.float32, device=dev)
    ws_f = rb.alloc_workspace(vel, B, N, tab, pol, False, dev)
    ws_b = rb.alloc_workspace(vel, B, N, tab, pol, True, dev)
    dynamic = wl.resolve_scaling(cfg) == "dynamic"
    grad_t = torch.zeros(N + 1, dtype=torch.float32, device=dev) if args.grad_t else None

    def loss_grad():
        # caller-side terminal loss gradient (outside the library), same formulas as the workload module
        if cfg.loss == "half_sse":
            torch.sub(yN, target, out=grad_yN)
        elif cfg.loss == "mse":
            torch.sub(yN, target, out=grad_yN)
            grad_yN.mul_(2.0 / grad_yN.numel())
        else:
            torch.mul(yN, 2.0 / yN.numel(), out=grad_yN)
        if cfg.grad_scale != 1.0:
            grad_yN.mul_(cfg.grad_scale)

    def one_pass():
        rb.rampde_odeint_fwd(vel, theta, y0, tgrid, tab, pol, ckpt=ckpt, yN=yN, workspace=ws_f)
        loss_grad()
        grad_theta.zero_()
        if grad_t is not None:
            grad_t.zero_()
        rb.rampde_odeint_bwd(vel, theta, tgrid, tab, pol, ckpt, grad_yN, grad_y0=grad_y0, grad_theta=grad_theta,
                             workspace=ws_b, want_info=dynamic, grad_t=grad_t)

    if args.calibrate_mib > 0:
        src = torch.ones(args.calibrate_mib * (1 << 18), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)  # one elementwise kernel: reads and writes calibrate_mib MiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_pass()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    value = B * N / (dt / args.steps)

    # ---- roofline of the dominant kernel class: instrumented repeat of the same K steps
    rb.rampde_timing_enable(True)
    for _ in range(args.steps):
        one_pass()
    torch.cuda.synchronize()
    classes = {"velocity_gemm": rb.K_VELOCITY_GEMM, "wgrad_gemm": rb.K_WGRAD_GEMM,
               "combine_store": rb.K_COMBINE_STORE, "adjoint_update": rb.K_ADJOINT_UPDATE,
               "fused_forward": rb.K_FUSED_FORWARD, "fused_adjoint_step": rb.K_FUSED_ADJOINT_STEP}
    timing = {}
    for name, cls in classes.items():
        ms, launches, work = rb.rampde_timing_read(cls)
        timing[name] = dict(ms=ms, launches=launches, work=work)
    rb.rampde_timing_enable(False)
    dom = max(("velocity_gemm", "wgrad_gemm", "fused_forward", "fused_adjoint_step"), key=lambda k: timing[k]["ms"])
    td = timing[dom]
    ach_tflops = td["work"] / (td["ms"] * 1e-3) / 1e12 if td["ms"] > 0 else 0.0
    roofline = {"bound": "mfma", "kernel": dom, "achieved": ach_tflops, "peak": PEAK_TFLOPS[cfg.low],
                "unit": "TFLOP/s", "frac": ach_tflops / PEAK_TFLOPS[cfg.low],
                "traffic": profiled_traffic(cfg.name, dom),
                "launches_per_step": td["launches"] / args.steps,
                "avg_launch_us": 1e3 * td["ms"] / max(1, td["launches"]),
                "flops_per_launch": td["work"] / max(1, td["launches"])}
    hbm = {}
    for k in ("combine_store", "adjoint_update"):
        t = timing[k]
        if t["ms"] > 0:
            gbs = t["work"] / (t["ms"] * 1e-3) / 1e9
            hbm[k] = {"achieved_GBs": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS,
                      "avg_launch_us": 1e3 * t["ms"] / max(1, t["launches"])}
    kernel_share = {k: timing[k]["ms"] / args.steps for k in timing}

    out = {
        "metric": "batch*RK-steps/sec (fwd+adjoint)", "value": value, "unit": "batch*RK-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.low, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.kind} B={B} widths={list(cfg.widths) or [cfg.C, cfg.H, cfg.W]} "
                               f"{cfg.tableau} N={N} t=[{cfg.t0},{cfg.t1}] low={cfg.low} "
                               f"scaling={wl.resolve_scaling(cfg)}" + (" +dL/dt" if args.grad_t else "")},
        "roofline": roofline, "hbm_kernels": hbm, "kernel_ms_per_step": kernel_share,
    }

    if not args.no_cpu:
        default_steps = {"cfg1": cfg.N, "cfg2": cfg.N, "cfg3": 1, "cfg4": 1, "cfg5": 16}.get(cfg.name, 1)
        out["cpu_baseline"] = cpu_baseline(cfg, theta_np, y0_np, target_np, args.cpu_steps or default_steps)
    print(json.dumps(out))


def profiled_traffic(workload, kernel_class):
    """HBM bytes per launch of a kernel class as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (calibrated against a plain copy) and recorded in the committed profile summary; None when the
    summary has no figure for this workload and kernel."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "bench_cfg2_kernels_and_hbm_traffic.md")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "traffic_bytes_per_launch" and f[1] == workload and f[2] == kernel_class:
                return int(f[3])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, theta, y0, target, n_steps):
    """The oracle as it stands (rounding-emulation mode), forward + adjoint, on the first
    `n_steps` RK steps of the workload's grid at the full batch size."""
    import parity as par
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    sub = cfg.with_(name=cfg.name, N=n_steps, t1=cfg.t0 + (cfg.t1 - cfg.t0) * n_steps / cfg.N)
    t0 = time.perf_counter()
    par.run_oracle(sub, theta, y0, target, "emul")
    dt = time.perf_counter() - t0
    return {"value": cfg.B * n_steps / dt, "unit": "batch*RK-steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n_steps} of {cfg.N} RK steps, full batch {cfg.B}, rounding-emulation mode, "
                      f"forward+adjoint, {dt:.1f} s"}


if __name__ == "__main__":
    main()
