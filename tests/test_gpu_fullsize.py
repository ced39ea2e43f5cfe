"""GPU parity at the full sizes of the five workloads, in the launch configuration the benchmark
times (row-tile-persistent kernels for the dense networks, per-layer kernels for the convolution).

* the benchmark workload (bf16 MLP, batch 4096, 32 RK4 steps) is compared in full with both oracles;
* the larger workloads are compared in full over a few time steps at the full batch size (which is
  what fixes tile shapes, grids and workspace layout), and over ALL their time steps on sampled
  batch rows: samples are independent in the forward recursion and in the adjoint, so the oracle
  can compute those rows one by one.
Tolerances as in test_gpu_parity.py.
"""
import os

import numpy as np
import pytest

from paper_2510_23498_amd import workloads as wl

import parity as par

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


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


def _golden(name, tab):
    tag = name if tab == wl.CONFIGS[name].tableau else f"{name}_{tab}"
    path = os.path.join(GOLDEN, f"fullsize_{tag}.npz")
    assert os.path.exists(path), f"{path} is missing: run tests/golden/make_fullsize_golden.py {name}:{tab}"
    return np.load(path)


def _block_sums(g, nblocks):
    edges = np.linspace(0, g.size, nblocks + 1).astype(np.int64)
    return np.array([g[edges[i]:edges[i + 1]].sum(dtype=np.float64) for i in range(nblocks)])


@pytest.mark.parametrize("name,tab", [("cfg3", "rk4"), ("cfg4", "rk4"), ("cfg5", "rk4"), ("cfg5", "heun"),
                                       ("cfg5", "euler")])
def test_full_size_all_steps_parameter_gradient(name, tab):
    """Full batch x ALL time steps against the emulation oracle's stored digest (written by
    tests/golden/make_fullsize_golden.py from oracle/ alone): the parameter gradient is an fp32 sum
    over B * s * N rows, whose accumulation error a few-step run cannot show."""
    cfg = wl.CONFIGS[name].with_(tableau=tab)
    ref = _golden(name, tab)
    theta, y0, target = par.make_inputs(cfg)
    print(f"[case] {cfg.name} {tab} full size B={cfg.B} N={cfg.N} vs stored oracle digest", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target)
    assert gpu["status"] == 0
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), ref["scale_hist"])
    assert gpu["retries"] == int(ref["retries"])
    g = gpu["grad_theta"].astype(np.float64)
    rows = np.ix_(ref["rows"], ref["cols"] if "cols" in ref.files else np.arange(cfg.d))
    tol, tol_max = par.TOL_EMUL, par.TOL_EMUL_MAX[cfg.low]
    norms = np.array([np.linalg.norm(g[sl]) for _, sl in par.layer_slices(cfg)])
    errs = {
        "grad_theta_samples": par.rel_err(g[ref["theta_idx"]], ref["grad_theta_at_idx"]),
        "grad_theta_block_sums": par.rel_err(_block_sums(g, ref["grad_theta_block_sums"].size),
                                             ref["grad_theta_block_sums"]),
        "grad_theta_norm": abs(np.linalg.norm(g) / float(ref["grad_theta_norm"]) - 1.0),
        "grad_theta_tensor_norms": float(np.max(np.abs(norms / np.maximum(ref["grad_theta_tensor_norms"], 1e-300) - 1.0)
                                                * (ref["grad_theta_tensor_norms"] > 0))),
        "yN_rows": par.rel_err(gpu["yN"].reshape(cfg.B, -1)[rows], ref["yN_rows"]),
        "grad_y0_rows": par.rel_err(gpu["grad_y0"].reshape(cfg.B, -1)[rows], ref["grad_y0_rows"]),
        "yN_norm": abs(np.linalg.norm(gpu["yN"].astype(np.float64)) / float(ref["yN_norm"]) - 1.0),
        "grad_y0_norm": abs(np.linalg.norm(gpu["grad_y0"].astype(np.float64)) / float(ref["grad_y0_norm"]) - 1.0),
    }
    emax = {
        "max_grad_theta_samples": par.max_err(g[ref["theta_idx"]], ref["grad_theta_at_idx"]),
        "max_grad_y0_rows": par.max_err(gpu["grad_y0"].reshape(cfg.B, -1)[rows], ref["grad_y0_rows"]),
        "max_yN_rows": par.max_err(gpu["yN"].reshape(cfg.B, -1)[rows], ref["yN_rows"]),
    }
    print("  ", {k: f"{v:.2e}" for k, v in {**errs, **emax}.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    bad.update({k: v for k, v in emax.items() if not v <= tol_max})
    assert not bad, bad


@pytest.mark.parametrize("name", ["cfg3", "cfg5"])
def test_full_size_two_kernel_paths_agree(name):
    """The row-tile-persistent kernels and the per-layer kernels are independent implementations:
    at full size they must take the same scale decisions and agree on every output."""
    cfg = wl.CONFIGS[name]
    theta, y0, target = par.make_inputs(cfg)
    print(f"[case] {cfg.name} full size, both kernel paths", flush=True)
    a = par.run_gpu(cfg, theta, y0, target)
    b = par.run_gpu(cfg, theta, y0, target, flags=4)
    np.testing.assert_array_equal(a["scale_hist"], b["scale_hist"])
    assert a["retries"] == b["retries"] and a["status"] == b["status"] == 0
    errs = {k: par.rel_err(a[k], b[k]) for k in ("yN", "ckpt", "grad_y0", "grad_theta")}
    print("  ", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert max(errs.values()) <= par.TOL_EMUL, errs
