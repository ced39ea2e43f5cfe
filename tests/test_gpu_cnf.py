"""GPU parity of the normalising-flow state [z; l] with the exact trace row dl/dt = -tr(dv/dz)
(paper Sec. 6.1), one-hidden-layer velocity: the HIP library through its C ABI against the CPU oracle.
Bounds as for the other smooth networks: 1e-3 (2-norm, and the max-norm companion) against the
rounding-emulation oracle, 2e-2 (fp16) / 5e-2 (bf16) against fp64; scale history and retries exactly.
"""
import numpy as np
import pytest

from paper_2510_23498_amd import workloads as wl

import parity as par

pytestmark = pytest.mark.gpu

BASE = wl.CONFIGS["cnf"]


def _case(cfg, bias_std=0.1, want_grad_t=False):
    theta, y0, target = par.make_inputs(cfg, bias_std=bias_std)
    print(f"[case] {cfg.name} widths={cfg.widths} B={cfg.B} N={cfg.N} low={cfg.low} tab={cfg.tableau}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, want_grad_t=want_grad_t)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    f64 = par.run_oracle(cfg, theta, y0, target, "f64")
    e1 = par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle", tol_max=par.TOL_EMUL_MAX[cfg.low])
    e2 = par.compare(cfg, gpu, f64, par.TOL_F64[cfg.low], "fp64 oracle", check_ckpt=False)
    print("  vs emul:", {k: f"{v:.2e}" for k, v in e1.items()}, flush=True)
    print("  vs f64 :", {k: f"{v:.2e}" for k, v in e2.items()}, flush=True)
    # the l column on its own (one column among d + 1: a wrong trace row would hide in the whole-state norm)
    assert par.rel_err(gpu["yN"][:, -1], emu["yN"][:, -1]) <= par.TOL_EMUL
    assert par.rel_err(gpu["grad_y0"][:, -1], emu["grad_y0"][:, -1]) <= par.TOL_EMUL
    assert gpu["status"] == 0 and emu["status"] == "ok"
    np.testing.assert_array_equal(np.asarray(gpu["scale_hist"], dtype=np.float64), emu["scale_hist"])
    assert gpu["retries"] == emu["retries"]
    if want_grad_t:
        e = par.rel_err(gpu["grad_t"], emu["grad_t"])
        print(f"  dL/dt vs emul: {e:.2e}", flush=True)
        assert e <= 2e-3
    return gpu, emu


@pytest.mark.parametrize("low", ["f16", "bf16"])
def test_cnf_paper_shape_reduced_batch(low):
    # 63 features + time = 64 network inputs, width 1024; the state has 64 columns (16-byte vector kernels)
    _case(BASE.with_(name=f"cnfs{low}", B=70, N=3, low=low))


@pytest.mark.parametrize("tab", ["euler", "heun", "kutta3"])
def test_cnf_small_odd_shapes_and_tableaux(tab):
    # d + 1 = 4 state columns (scalar streaming kernels), hidden width padded 40 -> 64, ragged batch
    _case(BASE.with_(name=f"cnf{tab}", B=37, N=4, widths=(3, 40, 3), tableau=tab, grad_scale=1.0))


def test_cnf_state_wider_than_one_padding_block():
    # d = 64: the l column is column 64, the first of a second block of 64 padded state columns
    _case(BASE.with_(name="cnf65", B=40, N=2, widths=(64, 128, 64), grad_scale=1.0))


def test_cnf_time_grid_gradient():
    _case(BASE.with_(name="cnft", B=48, N=3, widths=(7, 64, 7), grad_scale=1.0), want_grad_t=True)
