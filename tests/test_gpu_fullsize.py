"""GPU parity at the full sizes of the five workloads, in the launch configuration the benchmark
times (row-tile-persistent kernels for the dense networks, per-layer kernels for the convolution).

* the benchmark workload (bf16 MLP, batch 4096, 32 RK4 steps) is compared in full with both oracles;
* the larger workloads are compared in full over a few time steps at the full batch size (which is
  what fixes tile shapes, grids and workspace layout), and over ALL their time steps on sampled
  batch rows: samples are independent in the forward recursion and in the adjoint, so the oracle
  can compute those rows one by one.
Tolerances as in test_gpu_parity.py.
"""
import numpy as np
import pytest

from paper_2510_23498_amd import workloads as wl

import parity as par

pytestmark = pytest.mark.gpu


def _rows(cfg, k=6):
    # first and last rows, a tile boundary and a few in between
    cand = [0, 1, 15, 16, cfg.B // 2, cfg.B - 1]
    return sorted(set(min(max(int(r), 0), cfg.B - 1) for r in cand))[:k]


def test_benchmark_workload_full_size_both_oracles():
    cfg = wl.CONFIGS["cfg2"]
    theta, y0, target = par.make_inputs(cfg)
    print(f"[case] {cfg.name} full size B={cfg.B} N={cfg.N}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    e1 = par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    print("  vs emul:", {k: f"{v:.2e}" for k, v in e1.items()}, flush=True)
    f64 = par.run_oracle(cfg, theta, y0, target, "f64")
    e2 = par.compare(cfg, gpu, f64, par.TOL_F64[cfg.low], "fp64 oracle", check_ckpt=False)
    print("  vs f64 :", {k: f"{v:.2e}" for k, v in e2.items()}, flush=True)


@pytest.mark.parametrize("name,steps", [("cfg3", 2), ("cfg4", 1), ("cfg5", 4)])
def test_full_batch_few_steps(name, steps):
    full = wl.CONFIGS[name]
    cfg = full.with_(N=steps, t1=full.t0 + (full.t1 - full.t0) * steps / full.N)
    theta, y0, target = par.make_inputs(cfg)
    print(f"[case] {cfg.name} full batch B={cfg.B}, {steps} of {full.N} steps", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    errs = par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    print("  vs emul:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert gpu["status"] == 0 and emu["status"] == "ok"
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
    assert gpu["retries"] == emu["retries"]


@pytest.mark.parametrize("name,tab", [("cfg3", "rk4"), ("cfg4", "rk4"), ("cfg5", "rk4"), ("cfg5", "heun"),
                                       ("cfg5", "euler")])
def test_full_size_sampled_rows(name, tab):
    cfg = wl.CONFIGS[name].with_(tableau=tab)
    theta, y0, target = par.make_inputs(cfg)
    rows = _rows(cfg)
    print(f"[case] {cfg.name} {tab} full size B={cfg.B} N={cfg.N}, oracle on rows {rows}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target)
    assert gpu["status"] == 0
    assert np.all(np.isfinite(gpu["grad_theta"])) and np.all(np.isfinite(gpu["grad_y0"]))
    emu = par.run_oracle_rows(cfg, theta, y0, target, rows, "emul")
    f64 = par.run_oracle_rows(cfg, theta, y0, target, rows, "f64")
    ck_gpu = gpu["ckpt"].reshape(cfg.N + 1, cfg.B, -1)[:, rows]
    errs = {
        "yN": par.rel_err(gpu["yN"][rows], emu["yN"]),
        "ckpt": par.rel_err(ck_gpu, emu["ckpt"].reshape(ck_gpu.shape)),
        "yN_f64": par.rel_err(gpu["yN"][rows], f64["yN"]),
        "grad_y0_f64": par.rel_err(gpu["grad_y0"][rows], f64["grad_y0"]),
    }
    print("  ", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert errs["yN"] <= par.TOL_EMUL and errs["ckpt"] <= par.TOL_EMUL
    assert errs["yN_f64"] <= par.TOL_F64[cfg.low] and errs["grad_y0_f64"] <= par.TOL_F64[cfg.low]
    # stored trajectory = (N+1) low-precision states, half the bytes of an fp32 trajectory
    assert gpu["ckpt"].size == (cfg.N + 1) * cfg.B * cfg.d


@pytest.mark.parametrize("name,steps", [("cfg2", 32), ("cfg3", 2), ("cfg4", 1), ("cfg5", 4)])
def test_time_grid_gradient_full_batch(name, steps):
    # dL/dt is a sum over the whole batch, so it is compared at the full batch size (the benchmark
    # workload over all its steps, the larger ones over a few), beside the other outputs of that call
    full = wl.CONFIGS[name]
    cfg = full.with_(N=steps, t1=full.t0 + (full.t1 - full.t0) * steps / full.N)
    theta, y0, target = par.make_inputs(cfg)
    print(f"[case] dL/dt {cfg.name} full batch B={cfg.B}, {steps} of {full.N} steps", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, want_grad_t=True)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    e = par.rel_err(gpu["grad_t"], emu["grad_t"])
    print(f"  dL/dt vs emul {e:.2e}", flush=True)
    assert e <= par.TOL_EMUL, (e, gpu["grad_t"], emu["grad_t"])
    par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
