"""GPU checks of the dynamic adjoint scaling state machine (paper Algorithm 2: initial scale,
halve-and-retry on overflow, failure after k_max attempts, growth) and of the unscaled-safe
variant, against the CPU oracle; plus degenerate inputs.  Scale histories and retry counts are
powers of two and integers: they must match exactly."""
import numpy as np
import pytest
import torch

from paper_2510_23498_amd import binding as rb
from paper_2510_23498_amd import workloads as wl
from oracle import rampde_oracle as orc

import parity as par

pytestmark = pytest.mark.gpu
PATHS = pytest.mark.parametrize("flags", [0, rb.PER_LAYER_KERNELS], ids=["tile", "layer"])


def _linear_case(N):
    """One linear layer with gain 128 and no time input: the cotangent W^T lambda overflows fp16
    at the initial scale (|lambda| ~ 2^11 times 2^7), so the scale has to be halved."""
    d = 4
    theta = np.concatenate([(np.eye(d) * 128.0).ravel(), np.zeros(d)]).astype(np.float32)
    y0 = np.full((2, d), 0.001, dtype=np.float32)
    tg = np.arange(N + 1, dtype=np.float64) * 2.0 ** -10
    aN = np.full((2, d), 1.5, dtype=np.float32)
    return d, theta, y0, tg, aN


def _gpu_linear(d, theta, y0, tg, aN, scaling, k_max, flags, tabname="euler", grad_t=None):
    dev = torch.device("cuda:0")
    vel = rb.Velocity.mlp((d, d), time_input=False)
    t = wl.TABLEAUX[tabname]
    tab = rb.Tableau(t.A, t.b, t.c)
    pol = rb.Policy(low="f16", scaling=scaling, k_max=k_max, flags=flags)
    th = torch.from_numpy(theta).to(dev)
    yN, ck = rb.rampde_odeint_fwd(vel, th, torch.from_numpy(y0).to(dev), tg, tab, pol)
    return rb.rampde_odeint_bwd(vel, th, tg, tab, pol, ck, torch.from_numpy(aN).to(dev), grad_t=grad_t), ck


def _oracle_linear(d, theta, y0, tg, aN, scaling, k_max, tabname="euler"):
    vel = orc.MLPVelocity((d, d), time_input=False, activation="identity")
    pol = orc.Policy(low="f16", scaling=scaling, k_max=k_max)
    tab = wl.TABLEAUX[tabname]
    yN, ck = orc.odeint_fwd(vel, theta.astype(np.float64), y0, tg, tab, pol)
    return orc.odeint_bwd(vel, theta.astype(np.float64), tg, tab, pol, ck, aN)


@PATHS
@pytest.mark.parametrize("N,tabname", [(1, "euler"), (5, "euler"), (4, "rk4")])
def test_overflow_halves_scale_and_retries(N, tabname, flags):
    case = _linear_case(N)
    print(f"[case] overflow retry N={N} {tabname} flags={flags}", flush=True)
    (gy0, gth, info), _ = _gpu_linear(*case, "dynamic", 16, flags, tabname)
    ref = _oracle_linear(*case, "dynamic", 16, tabname)
    assert ref.status == "ok" and ref.retries >= 1
    assert info.status == 0 and info.retries == ref.retries
    np.testing.assert_array_equal(info.scale_hist.astype(np.float64), ref.scale_hist)
    assert par.rel_err(gy0.cpu().numpy(), ref.grad_y0) <= par.TOL_EMUL
    assert par.rel_err(gth.cpu().numpy(), ref.grad_theta) <= par.TOL_EMUL
    assert info.s_min == ref.scale_hist.min() and info.s_max == ref.scale_hist.max()


@PATHS
def test_scaling_fails_after_k_max_attempts(flags):
    case = _linear_case(3)
    ref = _oracle_linear(*case, "dynamic", 1)
    assert ref.status == "scale_failed"
    with pytest.raises(rb.RampdeError) as ei:
        _gpu_linear(*case, "dynamic", 1, flags)
    assert ei.value.code == rb.ESCALE
    assert ei.value.stats.failed_step == ref.failed_step == 2
    assert ei.value.stats.status == 2


@PATHS
def test_unscaled_safe_returns_infinite_gradients(flags):
    d, theta, y0, tg, aN = _linear_case(2)
    ref = _oracle_linear(d, theta, y0, tg, aN * 1000.0, "none_safe", 1)
    assert ref.status == "overflow_inf"
    (gy0, gth, info), _ = _gpu_linear(d, theta, y0, tg, aN * 1000.0, "none_safe", 1, flags)
    assert info.status == 1 and info.failed_step == ref.failed_step
    assert torch.isinf(gth).all() and torch.isinf(gy0).all()
    # without an overflow the safe variant equals the unscaled one
    (gy0s, gths, infos), _ = _gpu_linear(d, theta, y0, tg, aN * 1e-3, "none_safe", 1, flags)
    (gy0n, gthn, _), _ = _gpu_linear(d, theta, y0, tg, aN * 1e-3, "none", 1, flags)
    assert infos.status == 0
    assert torch.equal(gy0s, gy0n) and par.rel_err(gths.cpu().numpy(), gthn.cpu().numpy()) < 1e-6


@PATHS
def test_nonfinite_terminal_gradient_is_reported_at_step_N(flags):
    d, theta, y0, tg, aN = _linear_case(3)
    aN = aN.copy()
    aN[1, 2] = np.inf
    with pytest.raises(rb.RampdeError) as ei:
        _gpu_linear(d, theta, y0, tg, aN, "dynamic", 16, flags)
    assert ei.value.code == rb.ESCALE and ei.value.stats.failed_step == 3


@PATHS
def test_zero_terminal_gradient_gives_unit_scale_and_zero_gradients(flags):
    d, theta, y0, tg, aN = _linear_case(3)
    (gy0, gth, info), _ = _gpu_linear(d, theta, y0, tg, np.zeros_like(aN), "dynamic", 16, flags)
    assert info.status == 0 and info.scale_hist[3] == 1.0
    assert not gy0.any() and not gth.any()


@PATHS
def test_scale_grows_when_the_adjoint_decays(flags):
    # contracting linear dynamics: |a| shrinks going backward, so the scale must double (growth rule)
    d = 4
    theta = np.concatenate([(-np.eye(d) * 64.0).ravel(), np.zeros(d)]).astype(np.float32)
    y0 = np.full((3, d), 0.25, dtype=np.float32)
    tg = np.linspace(0.0, 12 * 2.0 ** -8, 13)
    aN = np.full((3, d), 3.0, dtype=np.float32)
    (gy0, gth, info), _ = _gpu_linear(d, theta, y0, tg, aN, "dynamic", 16, flags)
    ref = _oracle_linear(d, theta, y0, tg, aN, "dynamic", 16)
    assert ref.scale_hist[0] > ref.scale_hist[-1]
    np.testing.assert_array_equal(info.scale_hist.astype(np.float64), ref.scale_hist)
    assert info.retries == ref.retries
    assert par.rel_err(gy0.cpu().numpy(), ref.grad_y0) <= par.TOL_EMUL
    assert par.rel_err(gth.cpu().numpy(), ref.grad_theta) <= par.TOL_EMUL


@PATHS
def test_literal_policy_flags(flags):
    cfg = wl.CONFIGS["cfg1"].with_(name="lit", B=40, N=6)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    for gflag, okw in ((rb.ROUND_INCREMENT, {"round_increment": True}), (rb.GROW_RAW_NORM, {"grow_raw_norm": True})):
        gpu = par.run_gpu(cfg, theta, y0, target, flags=flags | gflag)
        emu = par.run_oracle(cfg, theta, y0, target, "emul", flags=okw)
        par.compare(cfg, gpu, emu, par.TOL_EMUL, f"emulation oracle {okw}")
        np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])


@PATHS
def test_single_sample_single_step(flags):
    cfg = wl.CONFIGS["cfg1"].with_(name="one", B=1, N=1, widths=(3, 16, 3), tableau="euler")
    theta, y0, target = par.make_inputs(cfg, bias_std=0.2)
    gpu = par.run_gpu(cfg, theta, y0, target, flags=flags)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    par.compare(cfg, gpu, emu, par.TOL_EMUL, "emulation oracle")


def test_gradient_is_accumulated_into_the_callers_vector():
    # g starts at the caller's dL/dtheta (Algorithm 2, initialisation)
    cfg = wl.CONFIGS["cfg1"].with_(name="acc", B=32, N=3)
    theta, y0, target = par.make_inputs(cfg)
    vel, tab, pol = par.gpu_descriptors(cfg)
    dev = torch.device("cuda:0")
    th = torch.from_numpy(theta).to(dev)
    yN, ck = rb.rampde_odeint_fwd(vel, th, torch.from_numpy(y0).to(dev), cfg.tgrid(), tab, pol)
    gyN = (yN - torch.from_numpy(target).to(dev)).contiguous()
    _, g0, _ = rb.rampde_odeint_bwd(vel, th, cfg.tgrid(), tab, pol, ck, gyN)
    init = torch.full_like(g0, 0.5)
    _, g1, _ = rb.rampde_odeint_bwd(vel, th, cfg.tgrid(), tab, pol, ck, gyN, grad_theta=init.clone())
    assert par.rel_err((g1 - 0.5).cpu().numpy(), g0.cpu().numpy()) < 1e-5



@PATHS
@pytest.mark.parametrize("N,tabname", [(5, "euler"), (4, "rk4")])
def test_time_grid_gradient_counts_a_retried_step_once(N, tabname, flags):
    # the sums of a step whose cotangent chain overflowed are discarded before the step is redone
    case = _linear_case(N)
    print(f"[case] dL/dt with overflow retry N={N} {tabname}", flush=True)
    gt = torch.full((N + 1,), 0.25, dtype=torch.float32, device="cuda:0")   # accumulated into
    (gy0, gth, info), _ = _gpu_linear(*case, "dynamic", 16, flags, tabname, grad_t=gt)
    ref = _oracle_linear(*case, "dynamic", 16, tabname)
    assert ref.retries >= 1 and info.retries == ref.retries
    assert par.rel_err(gt.cpu().numpy() - 0.25, ref.grad_t) <= par.TOL_EMUL, (gt.cpu().numpy() - 0.25, ref.grad_t)
    assert par.rel_err(gy0.cpu().numpy(), ref.grad_y0) <= par.TOL_EMUL
