"""rampde_odeint_fwd_static, the forward entry point that allocates nothing (its workspace is a static
device array inside the library), against rampde_odeint_fwd on the same inputs: bit for bit -- both
run the same kernels, and the forward pass has no atomics.  Two calls in a row share the array, the
second with a smaller problem; stale contents of the first must not leak into it.

Collected last on purpose (file name): the array keeps whatever the last call left in it, and this
file must pass both alone in a fresh process and after every other test.
"""
import numpy as np
import pytest

import parity as par
from paper_2510_23498_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _fwd_pair(cfg, flags=0, row_tile=0):
    """(static entry point's yN, ckpt), (workspace entry point's yN, ckpt) as numpy arrays."""
    import torch
    from paper_2510_23498_amd import binding as rb
    vel, tab, pol = par.gpu_descriptors(cfg, None, 16, flags, 0, row_tile)
    dev = torch.device("cuda:0")
    theta, y0, _ = par.make_inputs(cfg, bias_std=0.1)
    th = torch.from_numpy(theta).to(dev)
    y0d = torch.from_numpy(np.ascontiguousarray(y0)).to(dev)
    tg = cfg.tgrid()
    need = rb.rampde_workspace_bytes(vel, cfg.B, cfg.N, tab, pol, False)
    print(f"[case] {cfg.name} B={cfg.B} N={cfg.N} flags={flags} row_tile={row_tile} workspace {need} B", flush=True)
    assert 0 < need <= rb.STATIC_SCRATCH_BYTES
    # outputs are the caller's: allocated here, before the call, and filled with a pattern
    ck_s = torch.full(vel.ckpt_shape(cfg.B, cfg.N), 7.0, dtype=pol.torch_low, device=dev)
    yN_s = torch.full_like(y0d, -3.0)
    torch.cuda.synchronize()
    rb.rampde_odeint_fwd_static(vel, th, y0d, tg, tab, pol, ck_s, yN_s)
    torch.cuda.synchronize()
    got = (yN_s.cpu().numpy(), ck_s.view(torch.int16).cpu().numpy())
    yN_w, ck_w = rb.rampde_odeint_fwd(vel, th, y0d, tg, tab, pol)
    torch.cuda.synchronize()
    ref = (yN_w.cpu().numpy(), ck_w.view(torch.int16).cpu().numpy())
    return got, ref


CASES = [
    # first the larger problem, then smaller ones on the same array
    ("wide", wl.CONFIGS["cfg3"].with_(name="static_wide", B=300, N=5), 0, 64),
    ("wide_small", wl.CONFIGS["cfg3"].with_(name="static_wide_small", B=65, N=3), 0, 64),
    ("tile", wl.CONFIGS["cfg2"].with_(name="static_tile", B=200, N=4), 0, 0),
    ("layer", wl.CONFIGS["cfg2"].with_(name="static_layer", B=70, N=3), 4, 0),
    ("conv", wl.CONFIGS["cfg4"].with_(name="static_conv", B=2, N=3, C=8, H=8, W=16), 0, 0),
    ("conv_small", wl.CONFIGS["cfg4"].with_(name="static_conv_small", B=1, N=2, C=8, H=8, W=16), 0, 0),
]


def test_two_calls_in_a_row_match_the_workspace_entry_point_bit_for_bit():
    for _, cfg, flags, row_tile in CASES:
        got, ref = _fwd_pair(cfg, flags, row_tile)
        np.testing.assert_array_equal(got[0], ref[0], err_msg=f"{cfg.name}: y_N")
        np.testing.assert_array_equal(got[1], ref[1], err_msg=f"{cfg.name}: checkpoints")
        assert np.isfinite(got[0]).all()


def test_static_entry_point_also_matches_the_oracle():
    import torch
    from paper_2510_23498_amd import binding as rb
    cfg = wl.CONFIGS["cfg3"].with_(name="static_oracle", B=70, N=3)
    theta, y0, target = par.make_inputs(cfg, bias_std=0.1)
    vel, tab, pol = par.gpu_descriptors(cfg, None, 16, 0, 0, 0)
    dev = torch.device("cuda:0")
    th = torch.from_numpy(theta).to(dev)
    y0d = torch.from_numpy(np.ascontiguousarray(y0)).to(dev)
    ck = torch.empty(vel.ckpt_shape(cfg.B, cfg.N), dtype=pol.torch_low, device=dev)
    yN = torch.empty_like(y0d)
    print(f"[case] {cfg.name} vs emulation oracle", flush=True)
    rb.rampde_odeint_fwd_static(vel, th, y0d, cfg.tgrid(), tab, pol, ck, yN)
    torch.cuda.synchronize()
    emu = par.run_oracle(cfg, theta, y0, target, "emul")
    assert par.rel_err(yN.cpu().numpy(), emu["yN"]) <= par.TOL_EMUL
    assert par.rel_err(ck.float().cpu().numpy(), emu["ckpt"]) <= par.TOL_EMUL


def test_problem_beyond_the_static_array_is_rejected_before_anything_runs():
    import torch
    from paper_2510_23498_amd import binding as rb
    cfg = wl.CONFIGS["cfg4"]  # full size: its forward workspace is about 128 MiB
    vel, tab, pol = par.gpu_descriptors(cfg, None, 16, 0, 0, 0)
    assert rb.rampde_workspace_bytes(vel, cfg.B, cfg.N, tab, pol, False) > rb.STATIC_SCRATCH_BYTES
    dev = torch.device("cuda:0")
    th = torch.zeros(rb.rampde_num_params(vel), dtype=torch.float32, device=dev)
    y0 = torch.zeros((cfg.B, cfg.C, cfg.H, cfg.W), dtype=torch.float32, device=dev)
    ck = torch.full(vel.ckpt_shape(cfg.B, cfg.N), 5.0, dtype=pol.torch_low, device=dev)
    yN = torch.full_like(y0, 9.0)
    print(f"[case] {cfg.name} full size must be refused", flush=True)
    with pytest.raises(rb.RampdeError) as e:
        rb.rampde_odeint_fwd_static(vel, th, y0, cfg.tgrid(), tab, pol, ck, yN)
    assert e.value.code == rb.EWORKSPACE
    torch.cuda.synchronize()
    assert float(yN.min()) == 9.0 and float(ck.float().min()) == 5.0, "outputs must be untouched"
    # ... and the array still serves the next call
    got, ref = _fwd_pair(wl.CONFIGS["cfg3"].with_(name="static_after_refusal", B=33, N=2))
    np.testing.assert_array_equal(got[0], ref[0])
    np.testing.assert_array_equal(got[1], ref[1])
