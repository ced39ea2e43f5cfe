"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element
in the norm-wise sense, on seeded inputs with the shapes of the five workloads.

Tolerances: relative 2-norm error <= 1e-3 against the rounding-emulation oracle and
<= 2e-2 (fp16) / 5e-2 (bf16) against the fp64 oracle, for y_N, the stored trajectory,
dL/dy_0 and dL/dtheta (overall and per parameter tensor).  The adjoint scale history and
the retry count are compared exactly: they are powers of two and integers.
"""
import numpy as np
import pytest

from paper_2510_23498_amd import workloads as wl

import parity as par

pytestmark = pytest.mark.gpu


PER_LAYER = 4  # policy flag: one kernel per layer instead of the row-tile-persistent kernels
PATHS = pytest.mark.parametrize("flags", [0, PER_LAYER], ids=["tile", "layer"])


def _both(cfg, bias_std=0.0, scaling=None, tol_emul=par.TOL_EMUL, flags=0, row_tile=0, grad_ys=None, wgrad_tile=0):
    theta, y0, target = par.make_inputs(cfg, bias_std=bias_std)
    print(f"[case] {cfg.name} kind={cfg.kind} B={cfg.B} N={cfg.N} low={cfg.low} tab={cfg.tableau} flags={flags} "
          f"row_tile={row_tile} wgrad_tile={wgrad_tile}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling=scaling, flags=flags, row_tile=row_tile, grad_ys=grad_ys,
                      wgrad_tile=wgrad_tile)
    if grad_ys is not None:
        emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling=scaling, grad_ys=grad_ys.astype(np.float64))
        par.compare(cfg, gpu, emu, tol_emul, "emulation oracle")
        return gpu, emu, None
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling=scaling)
    f64 = par.run_oracle(cfg, theta, y0, target, "f64")
    e1 = par.compare(cfg, gpu, emu, tol_emul, "emulation oracle", tol_max=par.TOL_EMUL_MAX[cfg.low])
    e2 = par.compare(cfg, gpu, f64, par.TOL_F64[cfg.low], "fp64 oracle", check_ckpt=False)
    print("  vs emul:", {k: f"{v:.2e}" for k, v in e1.items()}, flush=True)
    print("  vs f64 :", {k: f"{v:.2e}" for k, v in e2.items()}, flush=True)
    assert gpu["status"] == 0 and emu["status"] == "ok"
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
    assert gpu["retries"] == emu["retries"]
    return gpu, emu, f64


@PATHS
def test_cfg1_tiny_mlp_full_size(flags):
    _both(wl.CONFIGS["cfg1"], flags=flags)


@PATHS
def test_cfg1_nonzero_bias_and_ragged_batch(flags):
    _both(wl.CONFIGS["cfg1"].with_(name="cfg1r", B=77, N=5), bias_std=0.3, flags=flags)


@PATHS
@pytest.mark.parametrize("tab", ["euler", "heun", "rk4", "kutta3"])
def test_small_mlp_all_tableaux(tab, flags):
    cfg = wl.CONFIGS["cfg1"].with_(name="tabs", B=130, N=6, widths=(5, 40, 24, 5), tableau=tab)
    _both(cfg, bias_std=0.2, flags=flags)


@PATHS
def test_mlp_odd_widths_many_layers(flags):
    # widths that pad to 64/128/192/320 columns: every column-group size of the tile kernels
    cfg = wl.CONFIGS["cfg1"].with_(name="odd", B=50, N=3, widths=(70, 130, 300, 190, 70), tableau="heun")
    _both(cfg, bias_std=0.1, flags=flags)


@PATHS
def test_cfg2_shape_reduced_batch(flags):
    # widths of the bf16 workload; batch spans several row tiles and a ragged tail
    _both(wl.CONFIGS["cfg2"].with_(name="cfg2s", B=300, N=6), bias_std=0.1, flags=flags)


@PATHS
def test_cfg3_shape_reduced_needs_dynamic_scaling(flags):
    cfg = wl.CONFIGS["cfg3"].with_(name="cfg3s", B=200, N=6)
    gpu, emu, f64 = _both(cfg, flags=flags)
    assert gpu["scale_hist"][cfg.N] > 2.0 ** 20  # the 1e-6 loss gradient needs a large scale
    # negative control: without scaling the fp16 cotangents underflow and the gradient is lost
    theta, y0, target = par.make_inputs(cfg)
    raw = par.run_gpu(cfg, theta, y0, target, scaling="none", flags=flags)
    e_raw = par.rel_err(raw["grad_theta"], f64["grad_theta"])
    e_dyn = par.rel_err(gpu["grad_theta"], f64["grad_theta"])
    assert e_raw > par.TOL_F64["f16"] and e_raw > 10 * e_dyn, (e_raw, e_dyn)


@PATHS
def test_unscaled_fp16_cotangents_in_the_subnormal_range_match_the_emulation(flags):
    # With the 1e-6 loss gradient and NO scaling most cotangents are a few units of the smallest fp16
    # subnormal (2^-24).  The oracle keeps gradual underflow; so must every conversion and matrix
    # instruction of the device path, or the two would differ by O(1) here (the fp64 comparison in
    # test_cfg3_shape_reduced_needs_dynamic_scaling only shows that the unscaled result is useless, not
    # that both sides agree on HOW it is useless).
    # ONE step of a network with ONE hidden layer: beyond that this regime is chaotic with respect to
    # rounding -- every cotangent is the rounding of a value of about one unit, so the first entry that
    # rounds the other way (the two sides sum their fp32 accumulators in different orders) moves a whole
    # row of the next layer by a sizeable fraction of a unit, and so on.  Measured on both kernel paths
    # alike: one RK4 step of 128-512-128 agrees to 7e-6 (one Euler step bit for bit); one step of the
    # four-layer cfg3 network to 3e-4 in dL/dy_0 but only 1e-2 in the first layer's gradient; 6 steps 5e-2.
    cfg = wl.CONFIGS["cfg3"].with_(name="cfg3sub", B=200, N=1, t1=2.0 / 64, widths=(128, 512, 128))
    theta, y0, target = par.make_inputs(cfg)
    print(f"[case] {cfg.name} scaling=none flags={flags}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling="none", flags=flags)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling="none")
    step = np.abs(emu["grad_y0"] - emu["grad_yN"])
    assert 0 < np.median(step[step > 0]) < 2.0 ** -20, "the case must exercise subnormal cotangents"
    # max-norm bound: a hidden cotangent here carries two or three significant bits, so ONE entry that
    # rounds the other way moves that sample's term of a first-layer gradient entry by up to half of
    # itself; the bound allows a handful of such entries (measured 4e-3), the 2-norm bound stays 1e-3.
    errs = par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle (unscaled)", tol_max=1e-2)
    print("  vs emul:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    # the adjoint increment itself (not hidden behind the much larger dL/dy_N), in units of 2^-24: it is
    # built from those two-or-three-bit cotangents alone, so the bound is 5 * TOL_EMUL (measured 1.2e-3);
    # flushing subnormals anywhere on the way would leave O(1) here
    inc_gpu = (gpu["grad_y0"].astype(np.float64) - gpu["grad_yN"]) * 2.0 ** 24
    inc_emu = (emu["grad_y0"] - emu["grad_yN"]) * 2.0 ** 24
    assert par.rel_err(inc_gpu, inc_emu) <= 5 * par.TOL_EMUL


# ------------------------------------------------------------------ 64-row-tile kernels of 512-wide networks
@pytest.mark.parametrize("B", [200, 64, 65, 1])
def test_wide_kernels_cfg3_shape(B):
    # the kernels the full-size cfg3 runs on, requested explicitly at a batch the oracle handles:
    # several tiles and a ragged tail, exactly one tile, one tile plus one row, a single row
    _both(wl.CONFIGS["cfg3"].with_(name=f"wide{B}", B=B, N=5), bias_std=0.1, row_tile=64)


@pytest.mark.parametrize("tab,low,widths", [("heun", "f16", (128, 512, 128)), ("kutta3", "f16", (128, 512, 512, 128)),
                                            ("euler", "f16", (128, 400, 512, 300, 500, 128)),
                                            ("rk4", "bf16", (128, 512, 512, 512, 128))])
def test_wide_kernels_depths_tableaux_precisions(tab, low, widths):
    # 2 to 5 layers (hidden widths that pad to 512), every tableau; bf16 under dynamic scaling so that
    # the adjoint also takes these kernels (with a fixed scale it runs groups of steps on the others)
    cfg = wl.CONFIGS["cfg3"].with_(name=f"wide{tab}{low}", B=150, N=4, tableau=tab, low=low, widths=widths,
                                   scaling="dynamic", grad_scale=1.0 if low == "bf16" else 1e-6)
    # bf16 at contraction length 512: the device sums 512 products in fp32, the oracle in fp64 with one
    # rounding; the two land on different sides of a bf16 rounding boundary (spacing 2^-8) often enough
    # that 16 stage evaluations of 4 layers accumulate to about 1e-3 in the 2-norm.  The 16-, 32- and
    # 64-row kernels give bit-identical results on this case, so it is not a property of one kernel.
    _both(cfg, bias_std=0.1, row_tile=64, tol_emul=2e-3 if low == "bf16" else par.TOL_EMUL)


# ------------------------------------------------------------------ parameter gradients: 128 x 128 block per wavefront
@pytest.mark.parametrize("B", [200, 65, 1])
def test_slab_parameter_gradient_kernel_cfg3_shape(B):
    # the kernel that the full-size cfg3 takes by its contraction length, requested at batches the oracle
    # handles: K-chunks shorter than its ring of k-steps, a ragged tail, a single row
    _both(wl.CONFIGS["cfg3"].with_(name=f"slab{B}", B=B, N=3), bias_std=0.1, row_tile=64, wgrad_tile=256)


@pytest.mark.parametrize("tab,low,widths,row_tile", [
    ("heun", "f16", (128, 512, 128), 64), ("kutta3", "bf16", (128, 512, 512, 128), 64),
    ("euler", "f16", (128, 400, 512, 300, 500, 128), 64),      # hidden widths that are no multiple of 128
    ("rk4", "f16", (64, 1024, 1024, 64), 0), ("rk4", "f16", (38, 302, 700, 38), 0)])  # 8-wave row-tile kernels; widths that are no multiple of 4
def test_slab_parameter_gradient_kernel_shapes(tab, low, widths, row_tile):
    # every arrangement of the four wavefronts (2 x 2, 4 x 1, 1 x 4), masked feature groups, rows with
    # and without a time column, both precisions
    cfg = wl.CONFIGS["cfg3"].with_(name=f"slab{tab}{low}{len(widths)}", B=150, N=3, tableau=tab, low=low, widths=widths,
                                   scaling="dynamic", grad_scale=1.0 if low == "bf16" else 1e-6)
    _both(cfg, bias_std=0.1, row_tile=row_tile, wgrad_tile=256, tol_emul=2e-3 if low == "bf16" else par.TOL_EMUL)


def test_slab_parameter_gradient_kernel_by_contraction_length():
    # chosen without being asked for: 4 stages x 2048 rows = 8192 k
    cfg = wl.CONFIGS["cfg3"].with_(name="slabauto", B=2048, N=2)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    gpu = par.run_gpu(cfg, theta, y0, target, row_tile=64)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle", tol_max=par.TOL_EMUL_MAX[cfg.low])
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
    small = par.run_gpu(cfg, theta, y0, target, row_tile=64, wgrad_tile=128)
    assert par.rel_err(gpu["grad_theta"], small["grad_theta"]) < 1e-5


def test_wide_kernels_running_cost_and_literal_flags():
    cfg = wl.CONFIGS["cfg3"].with_(name="widerun", B=100, N=4)
    gys = wl.normals(3, "widerun.gys", (cfg.N + 1, cfg.B, 128), 1e-7)
    _both(cfg, bias_std=0.1, row_tile=64, grad_ys=gys)
    # rounded increment + naive low-precision state (the forward pass takes the 64-row kernels)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling="none", flags=1 | 8, row_tile=64)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling="none",
                         flags=dict(round_increment=True, naive_state=True))
    for k in ("yN", "ckpt"):
        assert par.rel_err(gpu[k].reshape(emu[k].shape), emu[k]) <= par.TOL_EMUL, k


def test_cfg4_conv_shape_reduced():
    _both(wl.CONFIGS["cfg4"].with_(name="cfg4s", B=3, N=3), bias_std=0.1)


@pytest.mark.parametrize("C,H,W,B", [(96, 4, 8, 4), (8, 8, 16, 2), (70, 2, 64, 1), (8, 16, 24, 1), (16, 8, 40, 2)])
def test_conv_weight_gradient_all_taps_kernel(C, H, W, B):
    # image lines of 8 k pixels: the convolution weight gradient runs in the kernel that handles all
    # nine taps per workgroup (several channel blocks, a halo wider than the k-step, one-line images,
    # lines of 24 and 40 pixels: a k-step of 128 pixels then starts at a different column each time)
    cfg = wl.CONFIGS["cfg4"].with_(name=f"convw{C}x{H}x{W}", B=B, N=2, C=C, H=H, W=W, tableau="kutta3")
    _both(cfg, bias_std=0.1)


@pytest.mark.parametrize("H,W,B,wgrad_tile", [(16, 16, 3, 0), (8, 64, 2, 0), (20, 32, 3, 0), (32, 32, 2, 64)])
def test_conv_weight_gradient_64_channels_transposing_reads(H, W, B, wgrad_tile):
    # 64 channels and 16 / 32 / 64 pixels per line: the weight gradient (with the bias and time-channel sums) takes
    # the kernel built on transposing LDS reads -- K-chunks that start and end inside images (20 lines per image),
    # stage boundaries inside a chunk; policy.wgrad_tile = 64 keeps the kernel that transposes in registers
    cfg = wl.CONFIGS["cfg4"].with_(name=f"convtr{H}x{W}", B=B, N=2, C=64, H=H, W=W, tableau="kutta3")
    _both(cfg, bias_std=0.1, wgrad_tile=wgrad_tile)


def test_conv_weight_gradient_64_channels_transposing_reads_bf16():
    cfg = wl.CONFIGS["cfg4"].with_(name="convtrbf16", B=3, N=2, C=64, H=16, W=32, tableau="kutta3", low="bf16")
    # bf16 at contraction length 9 * 65: the device sums the products in fp32, the oracle in fp64 with one rounding,
    # and the two land on different sides of a bf16 rounding boundary often enough for 1e-3 (grad_y0, which no
    # weight-gradient kernel touches, is the largest: 1.9e-3); same bound as for the 512-wide bf16 networks above
    gpu, _, _ = _both(cfg, bias_std=0.1, tol_emul=2e-3)
    # the two weight-gradient kernels contract the same rounded operands: they agree to fp32 summation order
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    old = par.run_gpu(cfg, theta, y0, target, wgrad_tile=64)
    assert par.rel_err(gpu["grad_theta"], old["grad_theta"]) <= 1e-5
    np.testing.assert_array_equal(gpu["grad_y0"], old["grad_y0"])


def test_conv_small_odd_geometry():
    cfg = wl.CONFIGS["cfg4"].with_(name="convodd", B=2, N=2, C=5, H=7, W=6, tableau="kutta3")
    _both(cfg, bias_std=0.1)


@PATHS
@pytest.mark.parametrize("tab", ["rk4", "heun", "euler"])
def test_cfg5_shape_reduced(tab, flags):
    _both(wl.CONFIGS["cfg5"].with_(name="cfg5s", B=96, N=5, tableau=tab), flags=flags)


@PATHS
def test_running_cost_cotangents(flags):
    cfg = wl.CONFIGS["cfg1"].with_(name="run", B=64, N=4, widths=(6, 32, 6))
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    gys = wl.normals(3, "run.gys", (cfg.N + 1, cfg.B, 6), 0.1)
    gpu = par.run_gpu(cfg, theta, y0, target, grad_ys=gys, flags=flags)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", grad_ys=gys.astype(np.float64))
    par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")


@pytest.mark.parametrize("group", [2, 3, 64])
@pytest.mark.parametrize("low", ["bf16", "f16"])
def test_fixed_scale_runs_groups_of_steps_per_launch(group, low):
    # Without overflow detection (scaling "none") the adjoint kernel runs several steps per launch and
    # their parameter gradients are one contraction; groups of 2 / 3 (ragged last group) / all steps, ragged batch (rows padded inside the contraction), running-cost cotangents.
    # (group 3 on a 7-step grid: groups of 3, 3 and 1 steps)
    cfg = wl.CONFIGS["cfg2"].with_(name=f"grp{group}{low}", B=200, N=7 if group == 3 else 8,
                                   widths=(24, 256, 256, 24), low=low,
                                   tableau="kutta3" if group == 3 else "rk4")
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    gys = wl.normals(5, "grp.gys", (cfg.N + 1, cfg.B, 24), 1e-3)
    print(f"[case] {cfg.name}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling="none", grad_ys=gys, step_group=group)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling="none", grad_ys=gys.astype(np.float64))
    e = par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    print("  vs emul:", {k: f"{v:.2e}" for k, v in e.items()}, flush=True)
    assert gpu["status"] == 0
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])


# ------------------------------------------------------------------ time-grid gradient dL/dt
def _time_grid_case(cfg, scaling=None, bias_std=0.1, grad_ys=None, flags=0, step_group=0):
    theta, y0, target = par.make_inputs(cfg, bias_std=bias_std)
    print(f"[case] dL/dt {cfg.name} B={cfg.B} N={cfg.N} low={cfg.low} tab={cfg.tableau} flags={flags}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling=scaling, grad_ys=grad_ys, want_grad_t=True, flags=flags,
                      step_group=step_group)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling=scaling,
                         grad_ys=None if grad_ys is None else grad_ys.astype(np.float64))
    f64 = par.run_oracle(cfg, theta, y0, target, "f64", grad_ys=None if grad_ys is None else grad_ys.astype(np.float64))
    e_emu = par.rel_err(gpu["grad_t"], emu["grad_t"])
    e_f64 = par.rel_err(gpu["grad_t"], f64["grad_t"])
    print(f"  dL/dt vs emul {e_emu:.2e}  vs f64 {e_f64:.2e}", flush=True)
    assert e_emu <= par.TOL_EMUL, (e_emu, gpu["grad_t"], emu["grad_t"])
    assert e_f64 <= par.TOL_F64[cfg.low], e_f64
    # the other outputs are those of the plain backward pass
    par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
    return gpu, emu


@PATHS
@pytest.mark.parametrize("tab", ["euler", "heun", "rk4", "kutta3"])
def test_time_grid_gradient_small_mlp_all_tableaux(tab, flags):
    cfg = wl.CONFIGS["cfg1"].with_(name="dt" + tab, B=130, N=6, widths=(5, 40, 24, 5), tableau=tab)
    _time_grid_case(cfg, flags=flags)


@pytest.mark.parametrize("C,H,W,B,tab", [(64, 32, 32, 2, "rk4"), (64, 16, 16, 3, "heun"), (64, 4, 64, 2, "kutta3"),
                                          (5, 7, 6, 2, "kutta3"), (70, 4, 8, 4, "heun"),
                                          (70, 4, 8, 3, "heun"), (8, 16, 24, 1, "kutta3")])
def test_time_grid_gradient_conv(C, H, W, B, tab):
    # both convolutions carry a time channel; all-taps weight-gradient kernel and the generic one (W = 6)
    cfg = wl.CONFIGS["cfg4"].with_(name=f"dtconv{C}x{H}x{W}", B=B, N=2, C=C, H=H, W=W, tableau=tab)
    _time_grid_case(cfg)


@pytest.mark.parametrize("kind", ["mlp", "mlp_per_layer", "conv"])
def test_time_grid_gradient_is_reproducible_bit_for_bit(kind):
    # the batch sums of dL/dt are folded from per-workgroup slots in a fixed order (no floating-point atomics): two
    # runs on the same inputs give the same bits, with hundreds of workgroups adding to every step's sums
    if kind == "conv":
        cfg = wl.CONFIGS["cfg4"].with_(name="dtrep_conv", B=4, N=3, C=64, H=32, W=32)
        flags = 0
    else:
        cfg = wl.CONFIGS["cfg2"].with_(name="dtrep_mlp", B=4000, N=4)
        flags = 4 if kind == "mlp_per_layer" else 0
    theta, y0, target = par.make_inputs(cfg)
    a = par.run_gpu(cfg, theta, y0, target, want_grad_t=True, flags=flags)
    b = par.run_gpu(cfg, theta, y0, target, want_grad_t=True, flags=flags)
    assert np.all(np.isfinite(a["grad_t"])) and np.linalg.norm(a["grad_t"]) > 0
    np.testing.assert_array_equal(a["grad_t"], b["grad_t"])


def test_time_grid_gradient_cfg1_and_running_cost():
    _time_grid_case(wl.CONFIGS["cfg1"])
    cfg = wl.CONFIGS["cfg1"].with_(name="dtrun", B=64, N=4, widths=(6, 32, 6))
    _time_grid_case(cfg, grad_ys=wl.normals(3, "dtrun.gys", (cfg.N + 1, cfg.B, 6), 0.1))


@pytest.mark.parametrize("group", [3, 64])
def test_time_grid_gradient_fixed_scale_step_groups(group):
    cfg = wl.CONFIGS["cfg2"].with_(name=f"dtgrp{group}", B=200, N=7, widths=(24, 256, 256, 24))
    _time_grid_case(cfg, scaling="none", step_group=group)


def test_time_grid_gradient_wide_and_single_layer_networks():
    _time_grid_case(wl.CONFIGS["cfg5"].with_(name="dt5", B=96, N=4))
    _time_grid_case(wl.CONFIGS["cfg3"].with_(name="dt3", B=300, N=3))
    _time_grid_case(wl.CONFIGS["cfg1"].with_(name="dtlin", B=40, N=5, widths=(12, 12)))


# ------------------------------------------------------------------ naive low-precision baseline (Table 5)
NAIVE = 8  # policy flag: state and adjoint kept in low precision (no fp32 accumulators)


@PATHS
@pytest.mark.parametrize("low", ["f16", "bf16"])
def test_naive_state_baseline_matches_oracle(low, flags):
    cfg = wl.CONFIGS["cfg1"].with_(name="naive" + low, B=70, N=12, widths=(6, 40, 6), low=low)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    print(f"[case] naive baseline {low} flags={flags}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling="none", flags=flags | NAIVE)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling="none", flags=dict(naive_state=True))
    tol = par.TOL_EMUL
    for k in ("yN", "ckpt", "grad_y0", "grad_theta"):
        e = par.rel_err(gpu[k].reshape(emu[k].shape), emu[k])
        print(f"  {k}: {e:.2e}", flush=True)
        assert e <= tol, (k, e)
    # and it is a different computation from the scheme's
    good = par.run_gpu(cfg, theta, y0, target, scaling="none", flags=flags)
    assert par.rel_err(good["yN"], gpu["yN"]) > 0


def test_fp32_accumulator_beats_naive_low_precision_state_on_the_gpu():
    # many small steps of a contractive linear problem: rounding the state after every step loses the
    # increments (paper Sec. 4 discussion of Table 5); the scheme's fp32 accumulator does not
    import torch
    from paper_2510_23498_amd import binding as rb
    from oracle import rampde_oracle as orc
    rng = np.random.default_rng(11)
    d, B, N = 8, 4, 1000
    M = rng.normal(size=(d, d))
    A = -(M @ M.T) / d
    theta = np.concatenate([A.ravel(), np.zeros(d)])
    y0 = rng.normal(size=(B, d))
    rho = np.max(np.abs(np.linalg.eigvalsh(A)))
    tg = np.arange(N + 1) * (0.5 * 2.0 / rho) * 0.05
    t = wl.TABLEAUX["euler"]
    ref = orc.odeint_fwd(orc.MLPVelocity((d, d), time_input=False, activation="identity"), theta, y0, tg, t,
                         orc.Policy(low="f64"))[0]
    dev = torch.device("cuda:0")
    vel = rb.Velocity.mlp((d, d), time_input=False)
    tab = rb.Tableau(t.A, t.b, t.c)
    th = torch.from_numpy(theta.astype(np.float32)).to(dev)
    y0d = torch.from_numpy(y0.astype(np.float32)).to(dev)
    for low in ("f16", "bf16"):
        errs = {}
        for name, fl in (("scheme", 0), ("naive", NAIVE)):
            yN, _ = rb.rampde_odeint_fwd(vel, th, y0d, tg, tab, rb.Policy(low=low, scaling="none", flags=fl))
            torch.cuda.synchronize()
            errs[name] = par.rel_err(yN.cpu().numpy(), ref)
        print(f"[case] naive vs scheme {low}: {errs}", flush=True)
        assert errs["naive"] > 10.0 * errs["scheme"], (low, errs)


# ------------------------------------------------------------------ non-uniform time grids
def _nonuniform_grid(N, t0=0.0, t1=1.0, seed=3):
    w = 0.25 + wl.normals(seed, "grid", (N,), 1.0) ** 2       # step lengths differing by up to ~20x
    return t0 + (t1 - t0) * np.concatenate([[0.0], np.cumsum(w) / np.sum(w)])


@PATHS
@pytest.mark.parametrize("low,scaling,group", [("f16", "dynamic", 0), ("bf16", "none", 64), ("bf16", "none", 3)])
def test_nonuniform_time_grid(low, scaling, group, flags):
    # every step has its own h (and, with fixed scale, the groups-of-steps contraction rescales its
    # running sums by h_i / h_{i+1} at the step boundaries); dL/dt rides along
    cfg = wl.CONFIGS["cfg2"].with_(name=f"nonuni{low}{group}", B=150, N=10, widths=(20, 256, 256, 20), low=low)
    tg = _nonuniform_grid(cfg.N)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    print(f"[case] non-uniform grid {low} {scaling} group={group} flags={flags} h in [{np.diff(tg).min():.3f}, "
          f"{np.diff(tg).max():.3f}]", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling=scaling, flags=flags, tgrid=tg, want_grad_t=True,
                      step_group=group)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling=scaling, tgrid=tg)
    e = par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    et = par.rel_err(gpu["grad_t"], emu["grad_t"])
    print("  vs emul:", {k: f"{v:.2e}" for k, v in e.items()}, f"dL/dt {et:.2e}", flush=True)
    assert et <= par.TOL_EMUL
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])


def test_nonuniform_time_grid_conv():
    cfg = wl.CONFIGS["cfg4"].with_(name="nonuniconv", B=2, N=4)
    tg = _nonuniform_grid(cfg.N, seed=4)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    gpu = par.run_gpu(cfg, theta, y0, target, tgrid=tg)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", tgrid=tg)
    par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])


def test_fixed_scale_many_steps_default_group_length():
    # 130 steps without an environment override: groups of 64, 64 and 2 steps
    cfg = wl.CONFIGS["cfg2"].with_(name="grp130", B=48, N=130, widths=(8, 256, 256, 8), tableau="heun")
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    print(f"[case] {cfg.name}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, scaling="none", want_grad_t=True)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling="none")
    e = par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")
    et = par.rel_err(gpu["grad_t"], emu["grad_t"])
    print("  vs emul:", {k: f"{v:.2e}" for k, v in e.items()}, f"dL/dt {et:.2e}", flush=True)
    assert et <= par.TOL_EMUL
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])


@pytest.mark.parametrize("group", [1, 2, 4])
def test_slab_parameter_gradient_groups_of_steps_nonuniform_grid(group):
    # 7 steps in groups of 1, 2 and 4 (the last group is cut short at step 0); on a non-uniform grid h_i / S_i
    # differs from step to step, so the rescaling of the running sums at step boundaries is exercised
    cfg = wl.CONFIGS["cfg3"].with_(name=f"slabgrp{group}", B=100, N=7)
    tg = _nonuniform_grid(cfg.N, t1=2.0, seed=5)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    gpu = par.run_gpu(cfg, theta, y0, target, row_tile=64, wgrad_tile=256, step_group=group, tgrid=tg, want_grad_t=True)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", tgrid=tg)
    par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle", tol_max=par.TOL_EMUL_MAX[cfg.low])
    assert par.rel_err(gpu["grad_t"], emu["grad_t"]) <= par.TOL_EMUL
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
