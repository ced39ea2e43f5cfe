"""GPU parity of the parabolic convolution block  f = -W^T N(relu(W y + b))  with piecewise-constant
weights (paper Sec. 6.3, eq. (NODE_STL10)): the HIP library through its C ABI against the CPU oracle.

Bounds.  The ReLU mask is a discontinuous factor of the state and of the gradient: a pre-activation that
a rounding-level difference moves across zero flips a mask bit, and one flipped bit is an O(1) error in
that element.  Two correct implementations that sum their fp32 accumulators in different orders
therefore agree to 1e-3 only where no pre-activation sits within rounding distance of zero.  What is
checked:
  * one Euler step (identical stage input on both sides): everything to 1e-3;
  * biases shifted so that every pre-activation is positive (the mask is all ones), one RK4 step: 1e-3;
  * general runs: per tensor, max(1e-3, 4 x the oracle's OWN response to a relative perturbation of theta
    by 2e-4 unit roundoffs of the low format (1e-7 for fp16: below one fp32 rounding), measured in the
    same test).  The GPU may deviate from the emulation oracle by what the oracle itself does under a
    change no implementation can resolve, and by no more.
Against fp64: the forward bound of the workload's precision and the gradient bounds of the oracle's own
emulation-vs-fp64 pin.  Scale history and retry count must agree exactly.
"""
import numpy as np
import pytest

from paper_2510_23498_amd import workloads as wl

import parity as par

pytestmark = pytest.mark.gpu

# (gradients against fp64: mask flips between low precision and fp64 are far more frequent than between two
# low-precision implementations; small images (few pixels per statistic) are the most sensitive)
GRAD_TOL_F64 = {"f16": 6e-2, "bf16": 1.5e-1}


def _oracle_sensitivity(cfg, theta, y0, target, ref, scaling, flags):
    """Relative change of the oracle's outputs when theta moves by 2e-4 unit roundoffs of the low format,
    relative (seeded): a handful of the rounded weights then change by one unit in the last place, about as
    many low-precision roundings as separate two implementations that sum in different orders."""
    u_low = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8}[cfg.low]
    noise = wl.normals(11, cfg.name + ".noise", theta.shape).astype(np.float64)
    th2 = (theta.astype(np.float64) * (1.0 + 2e-4 * u_low * noise)).astype(np.float32)
    alt = par.run_oracle(cfg, th2, y0, target, "emul", scaling=scaling, flags=flags)
    return {k: par.rel_err(alt[k], ref[k]) for k in ("yN", "ckpt", "grad_y0", "grad_theta")}


def _all_positive(cfg, theta):
    """Biases shifted by +8: every pre-activation is positive, the ReLU passes everything, and only
    rounding separates the two sides (used by the cases that exist for a code path, not for the mask)."""
    theta = theta.copy()
    blk = cfg.C * cfg.C * 9 + cfg.C
    for q in range(cfg.n_intervals):
        theta[q * blk + cfg.C * cfg.C * 9:(q + 1) * blk] += 8.0
    return theta


def _case(cfg, bias_std=0.1, scaling=None, scale_group=0, positive=False, strict=False, wgrad_tile=0):
    theta, y0, target = par.make_inputs(cfg, bias_std=bias_std)
    if positive:
        theta = _all_positive(cfg, theta)
    print(f"[case] {cfg.name} C={cfg.C} {cfg.H}x{cfg.W} B={cfg.B} N={cfg.N} pieces={cfg.n_intervals} low={cfg.low} "
          f"tab={cfg.tableau}", flush=True)
    flags = dict(scale_group=scale_group) if scale_group else None
    gpu = par.run_gpu(cfg, theta, y0, target, scaling=scaling, scale_group=scale_group, wgrad_tile=wgrad_tile)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling=scaling, flags=flags)
    f64 = par.run_oracle(cfg, theta, y0, target, "f64")
    sens = {k: 0.0 for k in ("yN", "ckpt", "grad_y0", "grad_theta")} if strict else \
        _oracle_sensitivity(cfg, theta, y0, target, emu, scaling, flags)
    errs = {k: par.rel_err(np.asarray(gpu[k]).reshape(np.shape(emu[k])), emu[k]) for k in sens}
    print("  vs emul:", {k: f"{v:.2e}" for k, v in errs.items()}, " oracle sensitivity:",
          {k: f"{v:.2e}" for k, v in sens.items()}, flush=True)
    for k, e in errs.items():
        assert e <= max(par.TOL_EMUL, 4.0 * sens[k]), (k, e, sens[k])
    assert par.rel_err(gpu["yN"], f64["yN"]) <= par.TOL_F64[cfg.low]
    for k in ("grad_y0", "grad_theta"):
        e = par.rel_err(gpu[k], f64[k])
        print(f"  vs f64 {k}: {e:.2e}", flush=True)
        assert e <= GRAD_TOL_F64[cfg.low], (k, e)
    assert gpu["status"] == 0 and emu["status"] == "ok"
    np.testing.assert_array_equal(np.asarray(gpu["scale_hist"], dtype=np.float64).reshape(emu["scale_hist"].shape),
                                  emu["scale_hist"])
    assert gpu["retries"] == emu["retries"]
    # every piece of the piecewise-constant parameters received a gradient
    blk = cfg.C * cfg.C * 9 + cfg.C
    for q in range(cfg.n_intervals):
        assert np.linalg.norm(gpu["grad_theta"][q * blk:(q + 1) * blk]) > 0
    return gpu, emu


BASE = wl.CONFIGS["parab"]


@pytest.mark.parametrize("low", ["f16", "bf16"])
def test_parabolic_single_euler_step_is_tight(low):
    _case(BASE.with_(name=f"pbeuler{low}", B=3, C=64, H=16, W=16, N=1, n_intervals=1, tableau="euler", t1=0.25, low=low),
          strict=True)


@pytest.mark.parametrize("low,B,H,W", [("f16", 65, 8, 8), ("bf16", 16, 16, 16)])
def test_parabolic_wide_convolution_kernel_single_euler_step_is_tight(low, B, H, W):
    # 256 channels and >= 4096 pixels: the convolutions take the kernel with 256 x 256 workgroup tiles; image
    # borders inside a tile (four 8 x 8 images per tile), a last tile that is cut short (65 images)
    _case(BASE.with_(name=f"pbwide{low}", B=B, C=256, H=H, W=W, N=1, n_intervals=1, tableau="euler", t1=0.25, low=low),
          strict=True)


@pytest.mark.parametrize("B,H,W,wgrad_tile", [(4, 32, 32, 0), (1, 64, 64, 0), (2, 32, 64, 0), (8, 32, 16, 0), (4, 32, 32, 64)])
def test_parabolic_line_staged_convolution_kernel_single_euler_step_is_tight(B, H, W, wgrad_tile):
    # 256 channels, >= 4096 pixels, 16 / 32 / 64 pixels per line and image heights that are multiples of 512 / W: the
    # convolutions take the kernel that stages the input by image lines (several tiles per image: tiles at the top, in
    # the middle and at the bottom of an image); policy.wgrad_tile = 64 keeps the kernel that fetches a slab per tap
    _case(BASE.with_(name=f"pblines{H}x{W}", B=B, C=256, H=H, W=W, N=1, n_intervals=1, tableau="euler", t1=0.25),
          strict=True, wgrad_tile=wgrad_tile)


@pytest.mark.parametrize("C,B,H,W", [(128, 4, 32, 32), (384, 4, 32, 32)])
def test_parabolic_line_staged_and_transposing_kernels_other_channel_counts(C, B, H, W):
    # 128 channels: one block of output channels in both kernels; 384: three blocks each way (nine weight-gradient
    # workgroups per K-chunk and output-channel block, fewer whole groups per XCD than compute units)
    _case(BASE.with_(name=f"pbch{C}", B=B, C=C, H=H, W=W, N=1, n_intervals=1, tableau="euler", t1=0.25), strict=True)


def test_parabolic_line_staged_and_transposing_kernels_bf16():
    # the bf16 instantiations of the line-staged convolution and of the transposing-read weight gradient
    _case(BASE.with_(name="pblinesbf16", B=4, C=256, H=32, W=32, N=1, n_intervals=1, tableau="euler", t1=0.25, low="bf16"),
          strict=True)


def test_parabolic_benchmark_shape_single_euler_step_is_tight():
    # the shape the benchmark times (256 channels, 64 x 64 images, batch 16: 128 convolution tiles on each half of the
    # output channels, 20 K-chunks of 205 image lines in the weight gradient), one Euler step, everything to 1e-3
    _case(BASE.with_(name="pbfull", N=1, n_intervals=1, tableau="euler", t1=0.25), strict=True)


def test_parabolic_wide_convolution_kernel_rk4_two_pieces():
    _case(BASE.with_(name="pbwiderk4", B=16, C=256, H=16, W=16, N=2, n_intervals=2, t1=0.25))


# Weight gradients with channel counts in multiples of 128 and 16, 32 or 64 pixels per image line take the kernel built on
# transposing LDS reads (the cases above with 256 channels and 16 x 16 images among them); policy.wgrad_tile = 64 keeps
# the kernel with 64 x 64 channel blocks.  One Euler step: the same stage input on both sides, everything to 1e-3.
@pytest.mark.parametrize("C,B,H,W,wgrad_tile", [(256, 4, 16, 16, 64), (128, 3, 8, 32, 0), (128, 1, 24, 64, 0),
                                                (128, 5, 16, 16, 0)])
def test_parabolic_weight_gradient_kernels_single_euler_step_is_tight(C, B, H, W, wgrad_tile):
    # (128 channels: one channel block, three workgroups per K-chunk, so that chunks of a few image lines occur,
    # which start and end inside images; 5 images of 16 lines: a last chunk that is cut short)
    _case(BASE.with_(name=f"pbwg{C}x{H}x{W}", B=B, C=C, H=H, W=W, N=1, n_intervals=1, tableau="euler", t1=0.25),
          strict=True, wgrad_tile=wgrad_tile)


def test_parabolic_all_positive_preactivations_one_rk4_step_is_tight():
    _case(BASE.with_(name="pbpos", B=3, C=64, H=16, W=16, N=1, n_intervals=1, t1=0.25), positive=True, strict=True)


@pytest.mark.parametrize("low", ["f16", "bf16"])
def test_parabolic_one_channel_block_two_pieces(low):
    _case(BASE.with_(name=f"pb64{low}", B=3, C=64, H=16, W=16, N=4, n_intervals=2, low=low))


def test_parabolic_several_channel_blocks_and_padding():
    # 160 channels: padded to 192, three 64-channel blocks in the convolutions, weight gradients and statistics
    _case(BASE.with_(name="pb160", B=2, C=160, H=8, W=16, N=2, n_intervals=1))


@pytest.mark.parametrize("tab,n_int,N", [("heun", 3, 3), ("euler", 2, 4), ("kutta3", 1, 2)])
def test_parabolic_tableaux_and_pieces(tab, n_int, N):
    _case(BASE.with_(name=f"pb{tab}", B=2, C=24, H=8, W=8, N=N, n_intervals=n_int, tableau=tab, t1=0.1), positive=True)


def test_parabolic_odd_geometry_takes_the_generic_weight_gradient():
    # image lines of 6 pixels: the weight gradient runs in the tap-by-tap kernel, biases by column sums
    _case(BASE.with_(name="pbodd", B=2, C=10, H=5, W=6, N=2, n_intervals=2, tableau="rk4", t1=0.1), positive=True)


def test_parabolic_many_pixel_chunks_in_the_statistics():
    # 64 x 64 pixels, one sample: the statistics sums are split over pixel chunks and folded in fixed order
    _case(BASE.with_(name="pbhw", B=1, C=64, H=64, W=64, N=1, n_intervals=1, tableau="heun"))


@pytest.mark.parametrize("C,H,W", [(64, 8, 8), (128, 16, 16)])
def test_parabolic_retry_inside_a_piece_keeps_the_pieces_gradient(C, H, W):
    # a terminal gradient large enough that the first scale overflows in the chain: S is halved, the step is
    # redone, and the gradient of the piece that was being accumulated is continued, not lost
    # (128 channels, 16 pixels per line: the weight-gradient kernel built on transposing LDS reads)
    cfg = BASE.with_(name="pbretry" if C == 64 else f"pbretry{C}", B=2, C=C, H=H, W=W, N=4, n_intervals=2, grad_scale=1.0)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    theta = (theta * np.float32(12.0)).astype(np.float32)      # cotangents grow backward through W^T W
    gpu = par.run_gpu(cfg, theta, y0, target, scaling="dynamic")
    emu = par.run_oracle(cfg, theta, y0, target, "emul", scaling="dynamic")
    print(f"  retries gpu {gpu['retries']} oracle {emu['retries']}; scale history {emu['scale_hist']}", flush=True)
    assert emu["retries"] > 0, "the case is meant to overflow at least once"
    assert gpu["retries"] == emu["retries"]
    np.testing.assert_array_equal(np.asarray(gpu["scale_hist"], dtype=np.float64), emu["scale_hist"])
    sens = _oracle_sensitivity(cfg, theta, y0, target, emu, "dynamic", None)
    for k, sk in sens.items():
        e = par.rel_err(np.asarray(gpu[k]).reshape(np.shape(emu[k])), emu[k])
        assert e <= max(par.TOL_EMUL, 4.0 * sk), (k, e, sk)


def test_parabolic_scale_groups():
    _case(BASE.with_(name="pbgrp", B=4, C=64, H=8, W=8, N=2, n_intervals=2), scale_group=2)


def test_parabolic_time_grid_gradient_is_refused():
    import torch
    from paper_2510_23498_amd import binding as rb
    cfg = BASE.with_(name="pbt", B=1, C=8, H=8, W=8, N=2, n_intervals=1)
    theta, y0, target = par.make_inputs(cfg)
    out = par.run_gpu(cfg, theta, y0, target, want_grad_t=True, expect_error=True)
    assert out.get("error") == rb.EUNSUPPORTED
