"""Host-side checks of the C-ABI library that need no GPU: the built library loads, exports every
symbol the header declares, sizes parameters and workspaces consistently, and rejects bad
arguments before anything is launched (paper Sec. 3 / Algorithms 1-2 define the arguments:
time partition, tableau, precision and scaling policy)."""
import ctypes as C
import os
import re
import subprocess
import sys

import numpy as np
import pytest

from paper_2510_23498_amd import binding as rb
from paper_2510_23498_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    text = open(os.path.join(ROOT, "include", "rampde.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rampde_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = rb.load_library()
    names = _header_functions()
    assert {"rampde_odeint_fwd", "rampde_odeint_bwd", "rampde_workspace_bytes", "rampde_num_params",
            "rampde_strerror", "rampde_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/rampde.h but not exported"
    assert set(rb.EXPORTS) <= set(names)
    assert rb.rampde_version() >= 100


def _descr(cfg, **kw):
    if cfg.kind == "mlp":
        vel = rb.Velocity.mlp(cfg.widths)
    elif cfg.kind == "cnf":
        vel = rb.Velocity.cnf(cfg.widths[0], cfg.widths[1])
    elif cfg.kind == "parabolic":
        vel = rb.Velocity.parabolic(cfg.C, cfg.H, cfg.W, n_intervals=cfg.n_intervals)
    else:
        vel = rb.Velocity.conv2(cfg.C, cfg.H, cfg.W)
    t = wl.TABLEAUX[cfg.tableau]
    return vel, rb.Tableau(t.A, t.b, t.c), rb.Policy(low=cfg.low, **kw)


@pytest.mark.parametrize("name", sorted(wl.CONFIGS))
def test_parameter_count_and_workspace_sizes(name):
    cfg = wl.CONFIGS[name]
    vel, tab, pol = _descr(cfg)
    assert rb.rampde_num_params(vel) == wl.n_params(cfg) == cfg.n_params
    wf = rb.rampde_workspace_bytes(vel, cfg.B, cfg.N, tab, pol, False)
    wb = rb.rampde_workspace_bytes(vel, cfg.B, cfg.N, tab, pol, True)
    assert 0 < wf < wb < 8 << 30
    # the per-layer path is a valid plan too
    pl = rb.Policy(low=cfg.low, flags=rb.PER_LAYER_KERNELS)
    assert rb.rampde_workspace_bytes(vel, cfg.B, cfg.N, tab, pl, True) > 0
    # with one step per launch the query is monotone in the batch size (the default plan gives the
    # parameter-gradient kernel shorter groups of steps at a larger batch, so its buffers need not grow)
    p1 = rb.Policy(low=cfg.low, step_group=1)
    assert (rb.rampde_workspace_bytes(vel, 2 * cfg.B, cfg.N, tab, p1, True)
            > rb.rampde_workspace_bytes(vel, cfg.B, cfg.N, tab, p1, True))


def test_checkpoint_store_is_half_of_fp32():
    # only the low-precision states are kept (paper Sec. 3): (N+1) * n * 2 bytes
    for cfg in wl.CONFIGS.values():
        vel, _, pol = _descr(cfg)
        n = int(np.prod(vel.ckpt_shape(cfg.B, cfg.N)))
        assert n == (cfg.N + 1) * cfg.B * cfg.d
        assert n * 2 * 2 == n * 4


def _call_fwd(vel, tab, pol, tgrid, B=4, theta=1, y0=1, ckpt=1, yN=1, ws=1, ws_bytes=1 << 40):
    """Call rampde_odeint_fwd with dummy non-null pointers: every case below must be rejected
    by the host-side checks, before any pointer is used."""
    lib = rb.load_library()
    tg = np.ascontiguousarray(np.asarray(tgrid, dtype=np.float64))
    pc = pol.c
    p = lambda x: C.c_void_p(int(0x1000 * x)) if x else None
    return lib.rampde_odeint_fwd(C.byref(vel.c), p(theta), p(y0), B, tg.ctypes.data_as(C.POINTER(C.c_double)),
                                 len(tg) - 1, C.byref(tab.c), C.byref(pc), p(ckpt), p(yN), p(ws), ws_bytes, None)


def test_forward_rejects_bad_arguments_without_touching_the_device():
    cfg = wl.CONFIGS["cfg1"]
    vel, tab, pol = _descr(cfg)
    grid = cfg.tgrid()
    assert _call_fwd(vel, tab, pol, grid, theta=0) == rb.EINVAL           # null pointer
    assert _call_fwd(vel, tab, pol, grid, ws=0) == rb.EINVAL
    assert _call_fwd(vel, tab, pol, grid, B=0) == rb.EINVAL
    assert _call_fwd(vel, tab, pol, grid, y0=1.001) == rb.EINVAL          # device pointer not 16-byte aligned
    assert _call_fwd(vel, tab, pol, grid, ckpt=1.002) == rb.EINVAL
    assert _call_fwd(vel, tab, pol, grid[::-1]) == rb.EINVAL              # decreasing grid
    assert _call_fwd(vel, tab, pol, [0.0, 0.5, 0.5, 1.0]) == rb.EINVAL    # not strictly increasing
    assert _call_fwd(vel, tab, pol, [0.0, np.nan, 1.0]) == rb.EINVAL
    assert _call_fwd(vel, tab, pol, [0.0]) == rb.EINVAL                   # N < 1
    bad_tab = rb.Tableau([[0.0, 0.5], [0.5, 0.0]], [0.5, 0.5], [0.0, 1.0])  # entry above the diagonal
    assert _call_fwd(vel, bad_tab, pol, grid) == rb.EINVAL
    implicit = rb.Tableau([[0.5]], [1.0], [0.5])                          # diagonal entry: implicit scheme
    assert _call_fwd(vel, implicit, pol, grid) == rb.EINVAL
    assert _call_fwd(vel, tab, rb.Policy(low="f32"), grid) == rb.EUNSUPPORTED
    nine = rb.Tableau(np.tril(np.ones((9, 9)), -1), np.ones(9) / 9, np.linspace(0, 1, 9))
    assert _call_fwd(vel, nine, pol, grid) == rb.EUNSUPPORTED             # more stages than supported
    assert _call_fwd(vel, tab, pol, grid, ws_bytes=16) == rb.EWORKSPACE   # too small
    bad_vel = rb.Velocity.mlp((4, 8, 5))                                  # output width != state width
    assert _call_fwd(bad_vel, tab, pol, grid) == rb.EINVAL
    assert rb.rampde_num_params(bad_vel) == 0
    assert rb.rampde_workspace_bytes(bad_vel, 4, 3, tab, pol, True) == 0


def test_backward_rejects_bad_arguments_without_touching_the_device():
    lib = rb.load_library()
    cfg = wl.CONFIGS["cfg1"]
    vel, tab, pol = _descr(cfg)
    tg = np.ascontiguousarray(cfg.tgrid())
    pc = pol.c
    p = lambda x: C.c_void_p(int(0x1000 * x)) if x else None

    def call(theta=1, ckpt=1, gyN=1, gy0=1, gth=1, ws=1, ws_bytes=1 << 40, N=cfg.N, B=4, pc=pc):
        return lib.rampde_odeint_bwd(C.byref(vel.c), p(theta), B, tg.ctypes.data_as(C.POINTER(C.c_double)), N,
                                     C.byref(tab.c), C.byref(pc), p(ckpt), p(gyN), None, p(gy0), p(gth), None, None,
                                     p(ws), ws_bytes, None)

    assert call(theta=0) == rb.EINVAL
    assert call(ckpt=0) == rb.EINVAL
    assert call(gth=0) == rb.EINVAL
    assert call(N=0) == rb.EINVAL
    assert call(ws_bytes=64) == rb.EWORKSPACE
    assert call(gyN=1.001) == rb.EINVAL                                   # not 16-byte aligned
    assert call(gy0=1.003) == rb.EINVAL
    # scale groups: negative size; a group whose slice of the buffers would not start 16-byte aligned
    # (cfg1 has 2 state elements per sample: 3 samples are 6 elements)
    assert call(B=8, pc=rb.Policy(low="f16", scaling="dynamic", scale_group=-1).c) == rb.EINVAL
    assert call(B=8, pc=rb.Policy(low="f16", scaling="dynamic", scale_group=3).c) == rb.EINVAL


def test_error_strings():
    for code in (rb.OK, rb.EINVAL, rb.EUNSUPPORTED, rb.EWORKSPACE, rb.ESCALE, rb.EHIP, 99):
        msg = rb.rampde_strerror(code)
        assert isinstance(msg, str) and msg
    assert "scaling" in rb.rampde_strerror(rb.ESCALE)


def test_timing_interface_rejects_bad_class():
    lib = rb.load_library()
    assert lib.rampde_timing_read(99, None) == rb.EINVAL


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr
