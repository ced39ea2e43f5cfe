#!/usr/bin/env python3
"""Throughput of the mixed-precision neural-ODE time stepper on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch: rampde_odeint_fwd
(paper Algorithm 1), the caller-side terminal-loss gradient, rampde_odeint_bwd (paper
Algorithm 2).  Metric: batch * RK-steps per second = B * N / (t_fwd + t_bwd).

Prints ONE JSON line.  The headline (`value`, `roofline`, `cpu_baseline`) is the largest dense
workload, cfg3 (fp16, batch 16384, 512-wide, 64 RK4 steps, dynamic adjoint scaling); `all_configs`
holds one record per synthetic workload (cfg1, cfg2, cfg3, cfg4, cfg5 under RK4 / Heun / Euler, and
"parab": the parabolic convolution block of the paper's Sec. 6.3 at 256 channels, 64 x 64 pixels, batch 16)
measured the same way with fewer passes.

`roofline` is measured in a second, instrumented run of the same K passes (HIP events around
every launch of a kernel class, on the stream the library launches on).  Flops are ALGORITHMIC:
2 * rows * MACs per velocity evaluation with the unpadded layer shapes (time column included);
forward = s*N evaluations, adjoint kernels = 2*s*N (recomputation + input cotangents), parameter
gradients = s*N.  The flops of the padded contractions the kernels actually execute are reported
beside them.  `cpu_baseline` times the CPU oracle on a bounded sample of the headline workload.
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
HEADLINE = "cfg3"
ALL_CONFIGS = [("cfg1", None), ("cfg2", None), ("cfg3", None), ("cfg4", None),
               ("cfg5", "rk4"), ("cfg5", "heun"), ("cfg5", "euler"), ("parab", None), ("cnf", None)]
# evaluations of the velocity per forward evaluation that a kernel class performs
CLASS_EVALS = {"fused_forward": 1.0, "fused_adjoint_step": 2.0, "wgrad_gemm": 1.0, "velocity_gemm": 3.0}


def macs_per_row(cfg):
    """Multiply-accumulates of one velocity evaluation per batch row (MLP) or per pixel (conv),
    unpadded, time column / time channel included."""
    if cfg.kind in ("mlp", "cnf"):
        w = cfg.widths
        return sum((w[l] + (1 if l == 0 else 0)) * w[l + 1] for l in range(len(w) - 1))
    if cfg.kind == "parabolic":
        return 2 * cfg.C * 9 * cfg.C     # the convolution and its transpose
    return 2 * (cfg.C + 1) * 9 * cfg.C


def rows_of(cfg):
    return cfg.B if cfg.kind in ("mlp", "cnf") else cfg.B * cfg.H * cfg.W


def describe(cfg, wl, extra=""):
    shape = list(cfg.widths) if cfg.kind in ("mlp", "cnf") else [cfg.C, cfg.H, cfg.W]
    return (f"{cfg.name}: {cfg.kind} B={cfg.B} widths={shape} {cfg.tableau} N={cfg.N} t=[{cfg.t0},{cfg.t1}] "
            f"low={cfg.low} scaling={wl.resolve_scaling(cfg)}" + extra)


def measure(cfg, steps, warmup, grad_t=False, target_seconds=None):
    """Time `steps` forward+adjoint passes of one workload, then repeat them with per-kernel timing.
    target_seconds: choose the number of passes from a first timed pass instead."""
    import torch
    from paper_2510_23498_amd import binding as rb
    from paper_2510_23498_amd import workloads as wl
    import parity as par

    dev = torch.device("cuda:0")
    theta_np, y0_np, target_np = par.make_inputs(cfg)
    vel, tab, pol = par.gpu_descriptors(cfg)
    tgrid = cfg.tgrid()
    B, N, s = cfg.B, cfg.N, wl.TABLEAUX[cfg.tableau].s
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
    gt = torch.zeros(N + 1, dtype=torch.float32, device=dev) if grad_t else None
    retries = [0]

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
        if gt is not None:
            gt.zero_()
        _, _, info = rb.rampde_odeint_bwd(vel, theta, tgrid, tab, pol, ckpt, grad_yN, grad_y0=grad_y0,
                                          grad_theta=grad_theta, workspace=ws_b, want_info=dynamic, grad_t=gt)
        if info is not None:
            retries[0] = info.retries

    for _ in range(warmup):
        one_pass()
    torch.cuda.synchronize()
    if target_seconds is not None:
        t0 = time.perf_counter()
        one_pass()
        torch.cuda.synchronize()
        est = time.perf_counter() - t0
        steps = int(max(3, min(50, target_seconds / max(est, 1e-6))))
    t0 = time.perf_counter()
    for _ in range(steps):
        one_pass()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_pass = 1e3 * dt / steps

    # instrumented repeat of the same passes: HIP events around every launch of the kernel classes
    rb.rampde_timing_enable(True)
    for _ in range(steps):
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

    eval_flops = 2.0 * rows_of(cfg) * macs_per_row(cfg)      # one velocity evaluation of the batch
    peak = PEAK_TFLOPS[cfg.low]
    kernels = {}
    for name, evals in CLASS_EVALS.items():
        t = timing[name]
        if t["ms"] <= 0:
            continue
        alg = evals * s * N * eval_flops                      # per pass
        sec = t["ms"] * 1e-3 / steps                          # per pass
        kernels[name] = {
            "ms_per_pass": 1e3 * sec, "launches_per_pass": t["launches"] / steps,
            "avg_launch_us": 1e3 * t["ms"] / max(1, t["launches"]),
            "flops_per_pass": alg, "tflops": alg / sec / 1e12, "frac": alg / sec / 1e12 / peak,
            "padded_flops_per_pass": t["work"] / steps, "frac_padded": t["work"] / steps / sec / 1e12 / peak}
    hbm = {}
    for k in ("combine_store", "adjoint_update"):
        t = timing[k]
        if t["ms"] > 0:
            gbs = t["work"] / (t["ms"] * 1e-3) / 1e9
            hbm[k] = {"achieved_GBs": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS,
                      "avg_launch_us": 1e3 * t["ms"] / max(1, t["launches"]),
                      "ms_per_pass": t["ms"] / steps}
    n_state = cfg.B * cfg.d
    rec = {"workload": describe(cfg, wl, " +dL/dt" if grad_t else ""), "steps": steps, "ms_per_pass": ms_per_pass,
           "value": B * N / (dt / steps), "unit": "batch*RK-steps/s", "dtype": cfg.low,
           "flops_per_pass": 4.0 * s * N * eval_flops, "frac_overall": 4.0 * s * N * eval_flops / (dt / steps) / 1e12 / peak,
           "kernels": kernels, "hbm_kernels": hbm, "retries": retries[0],
           "ckpt_bytes_low": (N + 1) * n_state * 2, "ckpt_bytes_fp32": (N + 1) * n_state * 4}
    inputs = (theta_np, y0_np, target_np)
    del theta, y0, target, ckpt, yN, grad_yN, grad_y0, grad_theta, ws_f, ws_b
    torch.cuda.empty_cache()
    return rec, inputs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default=HEADLINE, help="headline workload (cfg1..cfg5; cfg5:heun selects a tableau)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-all", action="store_true", help="skip the per-workload records (all_configs)")
    ap.add_argument("--grad-t", action="store_true",
                    help="also form the time-grid gradient dL/dt in the backward pass (not part of the headline metric)")
    ap.add_argument("--cpu-steps", type=int, default=0,
                    help="RK steps of the oracle sample (0: the whole grid for the two small workloads, "
                         "1-16 steps for the larger ones: about 10-30 s of CPU work)")
    ap.add_argument("--calibrate-mib", type=int, default=0,
                    help="before the timed region run ONE plain elementwise copy (read + write) of this many MiB: "
                         "under `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE` its counter value calibrates the HBM byte "
                         "counters of the other kernels")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_23498_amd import binding as rb
    from paper_2510_23498_amd import workloads as wl

    rb.load_library()  # fails loudly when the HIP library is missing
    name, _, tabname = args.config.partition(":")
    cfg = wl.CONFIGS[name]
    if tabname:
        cfg = cfg.with_(tableau=tabname)

    if args.calibrate_mib > 0:
        dev = torch.device("cuda:0")
        src = torch.ones(args.calibrate_mib * (1 << 18), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)  # one elementwise kernel: reads and writes calibrate_mib MiB
        torch.cuda.synchronize()
        del src, dst

    head, inputs = measure(cfg, args.steps, args.warmup, grad_t=args.grad_t)
    dom = max(head["kernels"], key=lambda k: head["kernels"][k]["ms_per_pass"])
    kd = head["kernels"][dom]
    roofline = {"bound": "mfma", "kernel": dom, "achieved": kd["tflops"], "peak": PEAK_TFLOPS[cfg.low],
                "unit": "TFLOP/s", "frac": kd["frac"], "traffic": profiled_traffic(cfg.name, dom),
                "launches_per_step": kd["launches_per_pass"], "avg_launch_us": kd["avg_launch_us"],
                "flops_per_launch": kd["flops_per_pass"] / max(1.0, kd["launches_per_pass"]),
                "frac_padded": kd["frac_padded"]}
    out = {
        "metric": "batch*RK-steps/sec (fwd+adjoint)", "value": head["value"], "unit": "batch*RK-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_pass"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.low, "data": "synthetic",
        "config": {"workload": head["workload"]},
        "roofline": roofline, "hbm_kernels": head["hbm_kernels"],
        "kernel_ms_per_step": {k: v["ms_per_pass"] for k, v in head["kernels"].items()},
        "kernel_frac_of_mfma_peak": {k: v["frac"] for k, v in head["kernels"].items()},
        "ckpt_bytes_low": head["ckpt_bytes_low"], "ckpt_bytes_fp32": head["ckpt_bytes_fp32"],
    }

    if not args.no_cpu:
        default_steps = {"cfg1": cfg.N, "cfg2": cfg.N, "cfg3": 6, "cfg4": 1, "cfg5": 16}.get(cfg.name, 1)
        out["cpu_baseline"] = cpu_baseline(cfg, *inputs, args.cpu_steps or default_steps)
    del inputs

    if not args.no_all:
        recs = {}
        for nm, tb in ALL_CONFIGS:
            c = wl.CONFIGS[nm] if tb is None else wl.CONFIGS[nm].with_(tableau=tb)
            key = nm if tb is None else f"{nm}-{tb}"
            if c == cfg and not args.grad_t:
                recs[key] = head
                continue
            recs[key], _ = measure(c, 0, 2, target_seconds=1.0)
        out["all_configs"] = recs
    print(json.dumps(out))


def profiled_traffic(workload, kernel_class):
    """HBM bytes per launch of a kernel class as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (calibrated against a plain copy) and recorded in a committed profile summary; None when no
    summary has a figure for this workload and kernel."""
    pdir = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles")
    try:
        names = sorted(os.listdir(pdir))
    except OSError:
        return None
    for fn in names:
        try:
            for line in open(os.path.join(pdir, fn)):
                f = line.split()
                if len(f) == 4 and f[0] == "traffic_bytes_per_launch" and f[1] == workload and f[2] == kernel_class:
                    return int(f[3])
        except OSError:
            pass
    return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, theta, y0, target, n_steps):
    """The oracle as it stands (rounding-emulation mode, NumPy with its threaded BLAS), forward +
    adjoint, on the first `n_steps` RK steps of the workload's grid at the full batch size."""
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
            "cpu_model": cpu_model(),
            "sample": f"first {n_steps} of {cfg.N} RK steps, full batch {cfg.B}, rounding-emulation mode, "
                      f"forward+adjoint, {dt:.1f} s"}


if __name__ == "__main__":
    main()
