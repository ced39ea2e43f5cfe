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


# ------------------------------------------------------------------ the state machine at multi-workgroup sizes
def _gain_case(base, **kw):
    """A workload whose LAST weight tensor is multiplied by `gain`: the cotangent chain then amplifies
    the scaled adjoint beyond the fp16 range at the initial scale, and the adjoint itself grows from
    step to step going backward, so that the scale has to be halved again in the middle of the pass."""
    gain = kw.pop("gain")
    cfg = wl.CONFIGS[base].with_(low="f16", **kw)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    name, shp, off = [x for x in wl.theta_layout(cfg) if x[0].startswith("W")][-1]
    theta = theta.copy()
    theta[off:off + int(np.prod(shp))] *= gain
    return cfg, theta, y0, target


MULTI_WG = [
    # the 8-wavefront adjoint kernel (wide network), several row tiles and a ragged tail
    ("cfg3", dict(name="retry512", B=300, N=6, t1=0.09, gain=256.0, scaling="dynamic")),
    # the 4-wavefront adjoint kernel with the parameter gradients on the helper stream
    ("cfg2", dict(name="retry256", B=300, N=6, t1=0.09, gain=256.0, scaling="dynamic")),
    # the convolution path (per-layer kernels)
    ("cfg4", dict(name="retryconv", B=2, N=4, C=8, H=8, W=16, t1=0.02, gain=256.0, scaling="dynamic")),
]


@pytest.mark.parametrize("base,kw", MULTI_WG, ids=[k["name"] for _, k in MULTI_WG])
@pytest.mark.parametrize("flags,row_tile,wgrad_tile,step_group",
                         [(0, 0, 0, 0), (rb.PER_LAYER_KERNELS, 0, 0, 0), (0, 64, 0, 0), (0, 64, 256, 0), (0, 64, 256, 3),
                          (0, 64, 256, 1)],
                         ids=["tile", "layer", "wide", "wide-groups-of-4", "wide-groups-of-3", "wide-groups-of-1"])
def test_retry_in_the_middle_of_the_pass_many_workgroups(base, kw, flags, row_tile, wgrad_tile, step_group):
    # (wgrad_tile = 256: the parameter gradients of a group of accepted steps are one launch; a rejected
    # step cuts its group short and the next group starts with it)
    if base == "cfg4" and (flags or row_tile):
        pytest.skip("the convolution has one path")
    if base == "cfg2" and row_tile:
        pytest.skip("the 64-row-tile kernels are for 512-wide networks")
    cfg, theta, y0, target = _gain_case(base, **dict(kw))
    print(f"[case] mid-pass retry {cfg.name} B={cfg.B} flags={flags}", flush=True)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    hist = emu["scale_hist"]
    assert emu["status"] == "ok" and emu["retries"] >= 3
    assert np.sum(hist[:-1] < hist[1:]) >= 2, "the scale must drop at more than one step"
    gpu = par.run_gpu(cfg, theta, y0, target, flags=flags, row_tile=row_tile, wgrad_tile=wgrad_tile, step_group=step_group)
    assert gpu["status"] == 0
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), hist)
    assert gpu["retries"] == emu["retries"]
    # (the scale decisions above are exact; the values are compared at the fp64 tolerance: a last layer
    # with gain 256 magnifies every difference in fp32 summation order by that gain, here and in the
    # forward pass, so these deliberately ill-conditioned networks do not reach 1e-3)
    errs = par.compare(cfg, gpu, emu, par.TOL_F64[cfg.low], "emulation oracle (amplifying network)")
    print("  vs emul:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)


@pytest.mark.parametrize("base,kw", MULTI_WG, ids=[k["name"] for _, k in MULTI_WG])
def test_scaling_failure_many_workgroups(base, kw):
    cfg, theta, y0, target = _gain_case(base, **dict(kw))
    emu = par.run_oracle(cfg, theta, y0, target, "emul", k_max=1)
    assert emu["status"] == "scale_failed"
    print(f"[case] scaling failure {cfg.name}: oracle fails at step {emu['failed_step']}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target, k_max=1, expect_error=True)
    assert gpu.get("error") == rb.ESCALE
    assert gpu["info"].failed_step == emu["failed_step"] and gpu["info"].status == 2


@pytest.mark.parametrize("base,kw", MULTI_WG, ids=[k["name"] for _, k in MULTI_WG])
def test_unscaled_safe_many_workgroups(base, kw):
    # a loss gradient of order 1e3 overflows the unscaled fp16 chain of these amplifying networks
    kw = dict(kw)
    kw["scaling"] = "none_safe"
    cfg, theta, y0, target = _gain_case(base, **kw)
    cfg = cfg.with_(grad_scale=1e3 if cfg.loss == "half_sse" else 1e3 * cfg.B * cfg.d)
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    assert emu["status"] == "overflow_inf"
    print(f"[case] unscaled-safe overflow {cfg.name}: oracle overflows at step {emu['failed_step']}", flush=True)
    gpu = par.run_gpu(cfg, theta, y0, target)
    assert gpu["status"] == 1 and gpu["failed_step"] == emu["failed_step"]
    assert np.all(np.isinf(gpu["grad_theta"])) and np.all(np.isinf(gpu["grad_y0"]))


@PATHS
@pytest.mark.parametrize("want_info", [True, False])
def test_unscaled_variant_propagates_a_nonfinite_loss_gradient(flags, want_info):
    # the plain unscaled variant has no range checks (paper Sec. 5): an inf in dL/dy_N is not an
    # error and must come back as non-finite gradients, with or without the statistics block
    cfg = wl.CONFIGS["cfg1"].with_(name="infgrad", B=40, N=5, widths=(6, 32, 6))
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    vel, tab, pol = par.gpu_descriptors(cfg, scaling="none", flags=flags)
    dev = torch.device("cuda:0")
    th = torch.from_numpy(theta).to(dev)
    yN, ck = rb.rampde_odeint_fwd(vel, th, torch.from_numpy(y0).to(dev), cfg.tgrid(), tab, pol)
    gyN = torch.ones_like(yN)
    gyN[3, 2] = float("inf")
    gy0 = torch.zeros_like(yN)
    gth = torch.zeros(rb.rampde_num_params(vel), dtype=torch.float32, device=dev)
    _, _, info = rb.rampde_odeint_bwd(vel, th, cfg.tgrid(), tab, pol, ck, gyN, grad_y0=gy0, grad_theta=gth,
                                      want_info=want_info)
    torch.cuda.synchronize()
    assert not torch.isfinite(gy0).all() and not torch.isfinite(gth).all()
    if want_info:
        assert info.status == 0


def _constant_adjoint_case(N):
    """Zero velocity: the adjoint stays at 1.5 in every entry, nothing in the chain can overflow
    except lambda = Q(S a) itself.  S_N = 2^10 (S_N * 1.5 = 1536 lies in (1024, 2048])."""
    d = 4
    theta = np.zeros(d * d + d, dtype=np.float32)
    y0 = np.full((2, d), 0.5, dtype=np.float32)
    tg = np.arange(N + 1, dtype=np.float64) / N
    aN = np.full((2, d), 1.5, dtype=np.float32)
    return d, theta, y0, tg, aN


@PATHS
def test_raw_norm_growth_rule_differs_from_the_default(flags):
    # default rule: S ||a|| = 1536 > 1/(2 u) = 1024, the scale never grows: 2^10 throughout.
    # literal rule (||a|| = 1.5 <= 1024 at every clean step): the scale doubles after every clean
    # step, so step i is entered with 2^(10 + N-1-i), until lambda = 2^16 * 1.5 overflows fp16; that
    # step halves back to 2^15 (one retry, and no growth after a retried step), the next one is
    # entered with 2^15, is clean and doubles, the one after overflows again, and so on.
    N = 10
    d, theta, y0, tg, aN = _constant_adjoint_case(N)
    expect_default = np.full(N + 1, 2.0 ** 10)
    expect_raw = np.array([2.0 ** min(10 + (N - 1 - i), 15) for i in range(N)] + [2.0 ** 10])
    first_overflow = N - 1 - 6
    expect_retries = {0: 0, rb.GROW_RAW_NORM: (first_overflow + 2) // 2}
    for gflag, want in ((0, expect_default), (rb.GROW_RAW_NORM, expect_raw)):
        (gy0, gth, info), _ = _gpu_linear(d, theta, y0, tg, aN, "dynamic", 16, flags | gflag)
        np.testing.assert_array_equal(info.scale_hist.astype(np.float64), want)
        assert info.status == 0 and info.retries == expect_retries[gflag]
        assert torch.equal(gy0.cpu(), torch.from_numpy(aN))


# ------------------------------------------------------------------ scale groups (policy.scale_group)
def _group_inputs(cfg, spread):
    """Inputs whose loss gradient differs from sample to sample by powers of two up to 2^-spread, so that
    the groups start from different scales: the running-cost cotangents of sample b (added to the adjoint
    at every step) are scaled by 2^-(b * spread // B); the terminal-cost gradient, which weighs all
    samples alike, is made negligible beside them (the caller passes a cfg with a tiny grad_scale)."""
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    shape = (cfg.N + 1,) + tuple(np.shape(y0))
    u = wl.uniforms(cfg.seed + 29, f"{cfg.name}.scale_groups.gys", int(np.prod(shape))).reshape(shape)
    w = 2.0 ** -(np.arange(cfg.B) * spread // cfg.B)
    gys = (0.05 * (u - 0.5) * w.reshape((1, cfg.B) + (1,) * (len(shape) - 2))).astype(np.float32)
    return theta, y0, target, gys


GROUP_CASES = [
    # (workload, overrides, G, flags, row_tile): a group size that does not divide the batch; groups of one
    # 64-row tile of the wide kernels; the per-layer kernels; the convolution path with one sample per group
    ("cfg1", dict(name="groups_cfg1", B=70), 32, 0, 0),
    ("cfg3", dict(name="groups_cfg3", B=200, N=4), 64, 0, 64),
    ("cfg3", dict(name="groups_cfg3_tile", B=100, N=3), 48, 0, 16),
    ("cfg2", dict(name="groups_cfg2_layer", B=90, N=4, low="f16", scaling="dynamic"), 40, 4, 0),
    ("cfg4", dict(name="groups_conv", B=3, N=3, C=8, H=8, W=16), 1, 0, 0),
]


@pytest.mark.parametrize("base,kw,G,flags,row_tile", GROUP_CASES, ids=[c[1]["name"] for c in GROUP_CASES])
def test_scale_groups_match_the_oracle_with_the_same_groups(base, kw, G, flags, row_tile):
    cfg = wl.CONFIGS[base].with_(grad_scale=1e-12, **kw)
    theta, y0, target, gys = _group_inputs(cfg, spread=24)
    print(f"[case] scale groups {cfg.name} B={cfg.B} G={G} flags={flags} row_tile={row_tile}", flush=True)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", flags={"scale_group": G}, grad_ys=gys)
    assert emu["status"] == "ok"
    groups = -(-cfg.B // G)
    assert emu["scale_hist"].shape == (groups, cfg.N + 1)
    assert len({tuple(r) for r in emu["scale_hist"]}) > 1, "the groups must not all share one scale history"
    gpu = par.run_gpu(cfg, theta, y0, target, flags=flags, row_tile=row_tile, grad_ys=gys, scale_group=G,
                      want_grad_t=True)
    assert gpu["status"] == 0
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
    assert gpu["retries"] == emu["retries"]
    errs = par.compare(cfg, gpu, emu, par.TOL_EMUL, f"emulation oracle (scale groups of {G})")
    errs["grad_t"] = par.rel_err(gpu["grad_t"], emu["grad_t"])
    print("  vs emul:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert errs["grad_t"] <= 5 * par.TOL_EMUL
    # one scale for the whole batch: the small samples' cotangents sink towards the subnormals and the
    # result moves away from the fp64 gradient, which the grouped one stays close to
    f64 = par.run_oracle(cfg, theta, y0, target, "f64", grad_ys=gys)
    last = slice(-(cfg.B - (groups - 1) * G), None)
    e_grp = par.rel_err(gpu["grad_y0"][last], f64["grad_y0"][last])
    one = par.run_gpu(cfg, theta, y0, target, flags=flags, row_tile=row_tile, grad_ys=gys)
    e_one = par.rel_err(one["grad_y0"][last], f64["grad_y0"][last])
    print(f"  last group's dL/dy_0 vs fp64: own scale {e_grp:.2e}, batch-wide scale {e_one:.2e}", flush=True)
    assert e_grp <= par.TOL_F64[cfg.low] and e_grp <= e_one * 1.5


def test_scale_groups_retry_failure_and_overflow_are_per_group():
    # the amplifying network of the mid-pass retry tests, two groups; every group retries on its own
    cfg, theta, y0, target = _gain_case("cfg3", name="groups_retry", B=150, N=5, t1=0.09, gain=256.0, scaling="dynamic")
    G = 80
    print(f"[case] scale groups with retries {cfg.name} B={cfg.B} G={G}", flush=True)
    emu = par.run_oracle(cfg, theta, y0, target, "emul", flags={"scale_group": G})
    assert emu["status"] == "ok" and emu["retries"] >= 4 and emu["scale_hist"].shape == (2, cfg.N + 1)
    gpu = par.run_gpu(cfg, theta, y0, target, scale_group=G)
    np.testing.assert_array_equal(gpu["scale_hist"].astype(np.float64), emu["scale_hist"])
    assert gpu["retries"] == emu["retries"] and gpu["status"] == 0
    par.compare(cfg, gpu, emu, par.TOL_F64[cfg.low], "emulation oracle (amplifying network, scale groups)")
    # k_max = 1: the first group fails
    emu1 = par.run_oracle(cfg, theta, y0, target, "emul", k_max=1, flags={"scale_group": G})
    gpu1 = par.run_gpu(cfg, theta, y0, target, k_max=1, expect_error=True, scale_group=G)
    assert emu1["status"] == "scale_failed" and gpu1.get("error") == rb.ESCALE
    assert gpu1["info"].failed_step == emu1["failed_step"] and gpu1["info"].status == 2
    # unscaled-safe: an overflow in a group leaves +inf in ALL of dL/dy_0 and dL/dtheta
    big = cfg.with_(grad_scale=1e3 * cfg.B * cfg.d, scaling="none_safe")
    emu2 = par.run_oracle(big, theta, y0, target, "emul", flags={"scale_group": G})
    gpu2 = par.run_gpu(big, theta, y0, target, scale_group=G)
    assert emu2["status"] == "overflow_inf" and gpu2["status"] == 1
    assert np.all(np.isposinf(gpu2["grad_y0"])) and np.all(np.isposinf(gpu2["grad_theta"]))


def test_scale_group_sizes_that_cover_the_batch_are_the_default_path():
    cfg = wl.CONFIGS["cfg1"].with_(name="groups_whole", B=40)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    base = par.run_gpu(cfg, theta, y0, target)
    for G in (40, 1000):
        got = par.run_gpu(cfg, theta, y0, target, scale_group=G)
        assert got["scale_hist"].shape == (cfg.N + 1,)
        np.testing.assert_array_equal(got["grad_theta"], base["grad_theta"])
        np.testing.assert_array_equal(got["grad_y0"], base["grad_y0"])
