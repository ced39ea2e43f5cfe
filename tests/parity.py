"""Helpers shared by the GPU parity tests, the smoke check and the benchmark's CPU leg:
run one configuration through the CPU oracle and through the HIP library and compare.

The two pipelines are independent end to end: each integrates forward from the same
seeded inputs, forms the terminal-loss gradient from its OWN y_N with the shared fp32
loss formula of the workload module, and runs its own adjoint pass.
"""
from __future__ import annotations

import numpy as np

from paper_2510_23498_amd import workloads as wl

# tolerances (norm-wise relative error, 2-norm over the whole tensor)
TOL_EMUL = 1e-3                      # against the rounding-emulation oracle
TOL_F64 = {"f16": 2e-2, "bf16": 5e-2}  # against the fp64 oracle
# max-norm companion of TOL_EMUL:  max|x - ref| / max|ref|  <=  4 u_L.  The two sides sum their
# fp32 accumulators in different orders, so now and then a value lands on the other side of a
# 16-bit rounding boundary: an entry may be off by a couple of low-precision roundings (2 u_L
# each, relative to that entry, hence at most that relative to the largest entry), but not by
# more -- a wrong bias entry or a dropped ragged-tail element is an O(1) relative error there.
TOL_EMUL_MAX = {"f16": 4 * 2.0 ** -11, "bf16": 4 * 2.0 ** -8}


def rel_err(x, ref) -> float:
    x = np.asarray(x, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    if den == 0.0:
        return float(np.linalg.norm(x))
    return float(np.linalg.norm(x - ref) / den)


def max_err(x, ref) -> float:
    """max|x - ref| / max|ref| (absolute when ref is all zero)."""
    x = np.asarray(x, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    if x.size == 0:
        return 0.0
    den = float(np.max(np.abs(ref)))
    num = float(np.max(np.abs(x - ref)))
    return num if den == 0.0 else num / den


def make_inputs(cfg: wl.Config, bias_std: float = 0.0):
    theta = wl.make_theta(cfg, bias_std=bias_std)
    y0 = wl.make_y0(cfg)
    target = None if cfg.loss == "mean_sq" else wl.make_target(cfg)
    return theta, y0, target


# ------------------------------------------------------------------ oracle side
def oracle_velocity(cfg: wl.Config):
    from oracle import rampde_oracle as orc
    if cfg.kind == "mlp":
        return orc.MLPVelocity(cfg.widths, time_input=True)
    if cfg.kind == "cnf":
        return orc.CNFVelocity(cfg.widths[0], cfg.widths[1])
    if cfg.kind == "parabolic":
        return orc.ParabolicConvVelocity(cfg.C, cfg.H, cfg.W, n_intervals=cfg.n_intervals)
    return orc.Conv2Velocity(cfg.C, cfg.H, cfg.W, time_input=True)


def run_oracle(cfg: wl.Config, theta, y0, target, mode: str, scaling: str = None, k_max: int = 16,
               flags: dict = None, grad_ys=None, tgrid=None):
    """mode: 'emul' (round like the scheme, cfg.low) or 'f64'.  Returns a dict of fp64 arrays."""
    from oracle import rampde_oracle as orc
    vel = oracle_velocity(cfg)
    tab = wl.TABLEAUX[cfg.tableau]
    low = cfg.low if mode == "emul" else "f64"
    scaling = scaling or wl.resolve_scaling(cfg)
    pol = orc.Policy(low=low, scaling=scaling, k_max=k_max, **(flags or {}))
    tgrid = cfg.tgrid() if tgrid is None else np.asarray(tgrid, dtype=np.float64)
    y0f = y0.reshape(cfg.B, -1)
    yN, ckpt = orc.odeint_fwd(vel, theta, y0f, tgrid, tab, pol)
    yN32 = yN.astype(np.float32).reshape(cfg.state_shape)
    _, gyN = wl.loss_and_grad(cfg, yN32, target)
    res = orc.odeint_bwd(vel, theta, tgrid, tab, pol, ckpt, gyN.reshape(cfg.B, -1),
                         grad_ys=None if grad_ys is None else grad_ys.reshape(cfg.N + 1, cfg.B, -1))
    return dict(yN=yN.reshape(cfg.state_shape), ckpt=ckpt, grad_yN=gyN, grad_y0=res.grad_y0.reshape(cfg.state_shape),
                grad_theta=res.grad_theta, scale_hist=res.scale_hist, retries=res.retries, status=res.status,
                failed_step=res.failed_step, grad_t=res.grad_t)


def run_oracle_rows(cfg: wl.Config, theta, y0, target, rows, mode: str):
    """Oracle forward + adjoint on a sample of batch rows of a full-size workload.  Samples are
    independent in the forward recursion and in the adjoint (paper Sec. 3 assumes batch size one),
    so y_N, the stored states and dL/dy_0 of these rows are those of the full batch -- in fp64 mode
    exactly, in emulation mode as long as the batch-wide adjoint scale causes no range event.
    The mean-type losses are normalised by the FULL batch size."""
    from oracle import rampde_oracle as orc
    rows = np.asarray(rows)
    sub = cfg.with_(B=len(rows))
    vel = oracle_velocity(sub)
    tab = wl.TABLEAUX[cfg.tableau]
    low = cfg.low if mode == "emul" else "f64"
    pol = orc.Policy(low=low, scaling=wl.resolve_scaling(cfg))
    tgrid = cfg.tgrid()
    yN, ckpt = orc.odeint_fwd(vel, theta, y0[rows].reshape(len(rows), -1), tgrid, tab, pol)
    yN32 = yN.astype(np.float32).reshape(sub.state_shape)
    _, gyN = wl.loss_and_grad(sub, yN32, None if target is None else target[rows])
    if cfg.loss in ("mse", "mean_sq"):
        gyN = (gyN.astype(np.float64) * (len(rows) / cfg.B)).astype(np.float32)
    res = orc.odeint_bwd(vel, theta, tgrid, tab, pol, ckpt, gyN.reshape(len(rows), -1))
    return dict(yN=yN.reshape(sub.state_shape), ckpt=ckpt, grad_y0=res.grad_y0.reshape(sub.state_shape),
                status=res.status)


# ------------------------------------------------------------------ HIP side
def gpu_descriptors(cfg: wl.Config, scaling: str = None, k_max: int = 16, flags: int = 0, step_group: int = 0,
                    row_tile: int = 0, scale_group: int = 0, wgrad_tile: int = 0):
    from paper_2510_23498_amd import binding as rb
    if cfg.kind == "mlp":
        vel = rb.Velocity.mlp(cfg.widths, time_input=True)
    elif cfg.kind == "cnf":
        vel = rb.Velocity.cnf(cfg.widths[0], cfg.widths[1])
    elif cfg.kind == "parabolic":
        vel = rb.Velocity.parabolic(cfg.C, cfg.H, cfg.W, n_intervals=cfg.n_intervals)
    else:
        vel = rb.Velocity.conv2(cfg.C, cfg.H, cfg.W, time_input=True)
    t = wl.TABLEAUX[cfg.tableau]
    tab = rb.Tableau(t.A, t.b, t.c)
    pol = rb.Policy(low=cfg.low, scaling=scaling or wl.resolve_scaling(cfg), k_max=k_max, flags=flags,
                    step_group=step_group, row_tile=row_tile, scale_group=scale_group, wgrad_tile=wgrad_tile)
    return vel, tab, pol


def ckpt_to_boundary_layout(cfg: wl.Config, ckpt_np: np.ndarray) -> np.ndarray:
    """Library checkpoint layout -> [N+1, B, (state)] in the boundary (NCHW) element order."""
    if cfg.kind in ("mlp", "cnf"):
        return ckpt_np
    return np.ascontiguousarray(np.transpose(ckpt_np, (0, 1, 4, 2, 3)))


def run_gpu(cfg: wl.Config, theta, y0, target, scaling: str = None, k_max: int = 16, flags: int = 0,
            grad_ys=None, expect_error: bool = False, want_grad_t: bool = False, tgrid=None, step_group: int = 0,
            row_tile: int = 0, scale_group: int = 0, wgrad_tile: int = 0):
    import torch
    from paper_2510_23498_amd import binding as rb
    vel, tab, pol = gpu_descriptors(cfg, scaling, k_max, flags, step_group, row_tile, scale_group, wgrad_tile)
    dev = torch.device("cuda:0")
    th = torch.from_numpy(theta).to(dev)
    y0d = torch.from_numpy(np.ascontiguousarray(y0)).to(dev)
    tgrid = cfg.tgrid() if tgrid is None else np.asarray(tgrid, dtype=np.float64)
    yN, ckpt = rb.rampde_odeint_fwd(vel, th, y0d, tgrid, tab, pol)
    torch.cuda.synchronize()
    yN_np = yN.cpu().numpy()
    _, gyN = wl.loss_and_grad(cfg, yN_np, target)
    gyN_d = torch.from_numpy(np.ascontiguousarray(gyN)).to(dev)
    gys_d = None if grad_ys is None else torch.from_numpy(np.ascontiguousarray(grad_ys, dtype=np.float32)).to(dev)
    out = dict(yN=yN_np, ckpt=ckpt_to_boundary_layout(cfg, ckpt.float().cpu().numpy()), grad_yN=gyN)
    gt_d = torch.zeros(cfg.N + 1, dtype=torch.float32, device=dev) if want_grad_t else None
    try:
        gy0, gth, info = rb.rampde_odeint_bwd(vel, th, tgrid, tab, pol, ckpt, gyN_d, grad_ys=gys_d, grad_t=gt_d)
    except rb.RampdeError as e:
        if not expect_error:
            raise
        out.update(error=e.code, info=e.stats)
        return out
    torch.cuda.synchronize()
    if want_grad_t:
        out["grad_t"] = gt_d.cpu().numpy()
    out.update(grad_y0=gy0.cpu().numpy(), grad_theta=gth.cpu().numpy(), scale_hist=info.scale_hist,
               retries=info.retries, status=info.status, failed_step=info.failed_step, info=info)
    return out


def layer_slices(cfg: wl.Config):
    out = []
    for name, shp, off in wl.theta_layout(cfg):
        out.append((name, slice(off, off + int(np.prod(shp)))))
    return out


def compare(cfg: wl.Config, gpu: dict, ref: dict, tol: float, what: str, check_ckpt: bool = True,
            tol_max="auto"):
    """Assert norm-wise agreement of y_N, checkpoints, dL/dy_0 and dL/dtheta (overall and per tensor):
    relative 2-norm error <= tol and max-norm error <= tol_max (keys "max_*" of the returned dict).
    tol_max "auto": TOL_EMUL_MAX of the workload's precision for comparisons at the emulation
    tolerance, none for the looser comparisons with the fp64 oracle."""
    if tol_max == "auto":
        tol_max = TOL_EMUL_MAX[cfg.low] if tol <= TOL_EMUL else None
    errs = {}
    pairs = [("yN", gpu["yN"], ref["yN"])]
    if check_ckpt:
        pairs.append(("ckpt", gpu["ckpt"].reshape(ref["ckpt"].shape), ref["ckpt"]))
    pairs.append(("grad_y0", gpu["grad_y0"], ref["grad_y0"]))
    pairs.append(("grad_theta", gpu["grad_theta"], ref["grad_theta"]))
    for name, sl in layer_slices(cfg):
        if np.linalg.norm(ref["grad_theta"][sl]) > 0:
            pairs.append(("grad_" + name, gpu["grad_theta"][sl], ref["grad_theta"][sl]))
    for name, x, r in pairs:
        errs[name] = rel_err(x, r)
        if tol_max is not None:
            errs["max_" + name] = max_err(x, r)
    bad = {k: v for k, v in errs.items() if not (v <= (tol_max if k.startswith("max_") else tol))}
    assert not bad, f"{cfg.name} vs {what}: tolerance {tol:g} (max-norm {tol_max}) exceeded: {bad}; all: {errs}"
    return errs
