"""ctypes binding of librampde.so (argument marshalling only).

The functions carry the names of the C entry points declared in include/rampde.h.
torch is used for device memory and the current stream; no step of the method runs
here.  If the library has not been built the first call raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
import torch

from .build import LIB_PATH

F32, F16, BF16 = 0, 1, 2
SCALE_NONE, SCALE_NONE_SAFE, SCALE_DYNAMIC, SCALE_AUTO = 0, 1, 2, 3
VEL_MLP, VEL_CONV2, VEL_PARABOLIC, VEL_CNF = 0, 1, 2, 3
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, ESCALE, EHIP = 0, 1, 2, 3, 4, 5
_LOW = {"f32": F32, "f16": F16, "bf16": BF16}
_SCALING = {"none": SCALE_NONE, "none_safe": SCALE_NONE_SAFE, "dynamic": SCALE_DYNAMIC, "auto": SCALE_AUTO}
_TORCH_LOW = {F16: torch.float16, BF16: torch.bfloat16}

EXPORTS = ("rampde_num_params", "rampde_workspace_bytes", "rampde_odeint_fwd", "rampde_odeint_bwd",
           "rampde_odeint_bwd_tgrid", "rampde_strerror", "rampde_version", "rampde_timing_enable", "rampde_timing_read")

K_VELOCITY_GEMM, K_WGRAD_GEMM, K_COMBINE_STORE, K_ADJOINT_UPDATE, K_FUSED_FORWARD, K_FUSED_ADJOINT_STEP = range(6)
ROUND_INCREMENT, GROW_RAW_NORM, PER_LAYER_KERNELS, NAIVE_STATE = 1, 2, 4, 8


class _Tableau(C.Structure):
    _fields_ = [("s", C.c_int), ("A", C.POINTER(C.c_double)), ("b", C.POINTER(C.c_double)),
                ("c", C.POINTER(C.c_double))]


class _Velocity(C.Structure):
    _fields_ = [("kind", C.c_int), ("n_layers", C.c_int), ("widths", C.POINTER(C.c_int)),
                ("C", C.c_int), ("H", C.c_int), ("W", C.c_int), ("time_input", C.c_int), ("n_intervals", C.c_int)]


class _Policy(C.Structure):
    _fields_ = [("low", C.c_int), ("scaling", C.c_int), ("k_max", C.c_int), ("flags", C.c_uint),
                ("step_group", C.c_int), ("row_tile", C.c_int), ("wgrad_tile", C.c_int), ("scale_group", C.c_int)]


class _Stats(C.Structure):
    _fields_ = [("status", C.c_int), ("failed_step", C.c_int), ("retries", C.c_int),
                ("s_first", C.c_float), ("s_last", C.c_float), ("s_min", C.c_float), ("s_max", C.c_float)]


class _KernelTime(C.Structure):
    _fields_ = [("ms", C.c_double), ("launches", C.c_int64), ("work", C.c_double)]


class RampdeError(RuntimeError):
    def __init__(self, code: int, msg: str, stats=None):
        super().__init__(f"rampde error {code}: {msg}")
        self.code = code
        self.stats = stats


_lib = None


def load_library():
    """Load librampde.so (built in-tree by paper_2510_23498_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2510_23498_amd.build` first "
                           "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    lib.rampde_num_params.restype = C.c_int64
    lib.rampde_num_params.argtypes = [C.POINTER(_Velocity)]
    lib.rampde_workspace_bytes.restype = C.c_size_t
    lib.rampde_workspace_bytes.argtypes = [C.POINTER(_Velocity), C.c_int64, C.c_int, C.POINTER(_Tableau),
                                           C.POINTER(_Policy), C.c_int]
    lib.rampde_odeint_fwd.restype = C.c_int
    lib.rampde_odeint_fwd.argtypes = [C.POINTER(_Velocity), C.c_void_p, C.c_void_p, C.c_int64,
                                      C.POINTER(C.c_double), C.c_int, C.POINTER(_Tableau), C.POINTER(_Policy),
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.rampde_odeint_fwd_static.restype = C.c_int
    lib.rampde_odeint_fwd_static.argtypes = [C.POINTER(_Velocity), C.c_void_p, C.c_void_p, C.c_int64,
                                             C.POINTER(C.c_double), C.c_int, C.POINTER(_Tableau),
                                             C.POINTER(_Policy), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.rampde_odeint_bwd.restype = C.c_int
    lib.rampde_odeint_bwd.argtypes = [C.POINTER(_Velocity), C.c_void_p, C.c_int64, C.POINTER(C.c_double), C.c_int,
                                      C.POINTER(_Tableau), C.POINTER(_Policy), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.POINTER(C.c_float), C.POINTER(_Stats), C.c_void_p,
                                      C.c_size_t, C.c_void_p]
    lib.rampde_odeint_bwd_tgrid.restype = C.c_int
    lib.rampde_odeint_bwd_tgrid.argtypes = [C.POINTER(_Velocity), C.c_void_p, C.c_int64, C.POINTER(C.c_double), C.c_int,
                                            C.POINTER(_Tableau), C.POINTER(_Policy), C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_float),
                                            C.POINTER(_Stats), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.rampde_strerror.restype = C.c_char_p
    lib.rampde_strerror.argtypes = [C.c_int]
    lib.rampde_version.restype = C.c_int
    lib.rampde_timing_enable.restype = C.c_int
    lib.rampde_timing_enable.argtypes = [C.c_int]
    lib.rampde_timing_read.restype = C.c_int
    lib.rampde_timing_read.argtypes = [C.c_int, C.POINTER(_KernelTime)]
    _lib = lib
    return lib


# ------------------------------------------------------------------ descriptors
class Velocity:
    """Host-side velocity descriptor (mirrors rampde_velocity)."""

    def __init__(self, kind: str, widths: Sequence[int] = (), C_: int = 0, H: int = 0, W: int = 0,
                 time_input: bool = True, n_intervals: int = 0):
        self.kind = kind
        self.n_intervals = int(n_intervals)
        self.widths = tuple(int(w) for w in widths)
        self.C, self.H, self.W = int(C_), int(H), int(W)
        self.time_input = bool(time_input)
        self._warr = (C.c_int * max(1, len(self.widths)))(*self.widths) if self.widths else None
        self.c = _Velocity()
        self.c.kind = {"mlp": VEL_MLP, "conv2": VEL_CONV2, "parabolic": VEL_PARABOLIC, "cnf": VEL_CNF}[kind]
        self.c.n_intervals = self.n_intervals
        self.c.n_layers = len(self.widths) - 1 if kind in ("mlp", "cnf") else 2
        self.c.widths = C.cast(self._warr, C.POINTER(C.c_int)) if self._warr is not None else None
        self.c.C, self.c.H, self.c.W = self.C, self.H, self.W
        self.c.time_input = 1 if self.time_input else 0

    @staticmethod
    def mlp(widths, time_input=True):
        return Velocity("mlp", widths=widths, time_input=time_input)

    @staticmethod
    def conv2(C_, H, W, time_input=True):
        return Velocity("conv2", C_=C_, H=H, W=W, time_input=time_input)

    @staticmethod
    def cnf(d, H, time_input=True):
        """state [z; l] of d + 1 columns; velocity d -> H -> d with the exact trace row"""
        return Velocity("cnf", widths=(d, H, d), time_input=time_input)

    @staticmethod
    def parabolic(C_, H, W, n_intervals=1):
        return Velocity("parabolic", C_=C_, H=H, W=W, time_input=False, n_intervals=n_intervals)

    @property
    def d(self):
        if self.kind == "cnf":
            return self.widths[0] + 1
        return self.widths[0] if self.kind == "mlp" else self.C * self.H * self.W

    def state_shape(self, B):
        if self.kind == "cnf":
            return (B, self.widths[0] + 1)
        return (B, self.widths[0]) if self.kind == "mlp" else (B, self.C, self.H, self.W)

    def ckpt_shape(self, B, N):
        if self.kind == "cnf":
            return (N + 1, B, self.widths[0] + 1)
        return (N + 1, B, self.widths[0]) if self.kind == "mlp" else (N + 1, B, self.H, self.W, self.C)


class Tableau:
    """Explicit Butcher tableau (mirrors rampde_tableau); A is s x s, strictly lower triangular."""

    def __init__(self, A, b, c):
        self.A = np.ascontiguousarray(np.asarray(A, dtype=np.float64))
        self.b = np.ascontiguousarray(np.asarray(b, dtype=np.float64))
        self.cc = np.ascontiguousarray(np.asarray(c, dtype=np.float64))
        self.s = int(self.b.shape[0])
        self.c = _Tableau(self.s, self.A.ctypes.data_as(C.POINTER(C.c_double)),
                          self.b.ctypes.data_as(C.POINTER(C.c_double)),
                          self.cc.ctypes.data_as(C.POINTER(C.c_double)))


@dataclass
class Policy:
    low: str = "f16"
    scaling: str = "auto"
    k_max: int = 16
    flags: int = 0
    step_group: int = 0
    row_tile: int = 0
    scale_group: int = 0
    wgrad_tile: int = 0

    @property
    def c(self):
        return _Policy(_LOW[self.low], _SCALING[self.scaling], int(self.k_max), int(self.flags),
                       int(self.step_group), int(self.row_tile), int(self.wgrad_tile), int(self.scale_group))

    @property
    def torch_low(self):
        return _TORCH_LOW[_LOW[self.low]]


@dataclass
class BwdInfo:
    status: int
    failed_step: int
    retries: int
    s_first: float
    s_last: float
    s_min: float
    s_max: float
    scale_hist: Optional[np.ndarray]


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check_dev(t: torch.Tensor, dtype, numel, name):
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype and t.numel() == numel):
        raise ValueError(f"{name}: need a contiguous cuda tensor of {dtype} with {numel} elements, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")


def rampde_strerror(code: int) -> str:
    return load_library().rampde_strerror(code).decode()


def rampde_version() -> int:
    return load_library().rampde_version()


def rampde_timing_enable(on: bool) -> None:
    load_library().rampde_timing_enable(1 if on else 0)


def rampde_timing_read(kernel_class: int):
    """(total ms, launches, algorithmic work) of the recorded launches of one kernel class."""
    kt = _KernelTime()
    rc = load_library().rampde_timing_read(kernel_class, C.byref(kt))
    if rc != OK:
        raise RampdeError(rc, rampde_strerror(rc))
    return kt.ms, int(kt.launches), kt.work


def rampde_num_params(vel: Velocity) -> int:
    return int(load_library().rampde_num_params(C.byref(vel.c)))


def rampde_workspace_bytes(vel: Velocity, B: int, N: int, tab: Tableau, pol: Policy, is_backward: bool) -> int:
    pc = pol.c
    return int(load_library().rampde_workspace_bytes(C.byref(vel.c), B, N, C.byref(tab.c), C.byref(pc),
                                                     1 if is_backward else 0))


def alloc_workspace(vel, B, N, tab, pol, is_backward, device="cuda"):
    nbytes = rampde_workspace_bytes(vel, B, N, tab, pol, is_backward)
    if nbytes == 0:
        raise RampdeError(EINVAL, "workspace query rejected the arguments")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def rampde_odeint_fwd(vel: Velocity, theta: torch.Tensor, y0: torch.Tensor, tgrid, tab: Tableau, pol: Policy,
                      ckpt: Optional[torch.Tensor] = None, yN: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None, stream=None):
    """Forward pass (paper Algorithm 1).  Returns (yN fp32, ckpt low precision).  Asynchronous."""
    lib = load_library()
    B = int(y0.shape[0])
    tg = np.ascontiguousarray(np.asarray(tgrid, dtype=np.float64))
    N = int(tg.shape[0]) - 1
    P = rampde_num_params(vel)
    _check_dev(theta, torch.float32, P, "theta")
    _check_dev(y0, torch.float32, B * vel.d, "y0")
    if ckpt is None:
        ckpt = torch.empty(vel.ckpt_shape(B, N), dtype=pol.torch_low, device=y0.device)
    if yN is None:
        yN = torch.empty_like(y0)
    _check_dev(ckpt, pol.torch_low, (N + 1) * B * vel.d, "ckpt")
    _check_dev(yN, torch.float32, B * vel.d, "yN")
    if workspace is None:
        workspace = alloc_workspace(vel, B, N, tab, pol, False, y0.device)
    pc = pol.c
    rc = lib.rampde_odeint_fwd(C.byref(vel.c), _ptr(theta), _ptr(y0), B, tg.ctypes.data_as(C.POINTER(C.c_double)), N,
                               C.byref(tab.c), C.byref(pc), _ptr(ckpt), _ptr(yN), _ptr(workspace),
                               workspace.numel(), _stream_ptr(stream))
    if rc != OK:
        raise RampdeError(rc, rampde_strerror(rc))
    return yN, ckpt


STATIC_SCRATCH_BYTES = 32 << 20


def rampde_odeint_fwd_static(vel: Velocity, theta: torch.Tensor, y0: torch.Tensor, tgrid, tab: Tableau, pol: Policy,
                             ckpt: torch.Tensor, yN: torch.Tensor, stream=None):
    """rampde_odeint_fwd on the library's static scratch array: the caller passes every output, nothing
    is allocated here or in the library.  Raises RampdeError(EWORKSPACE) when the problem needs more
    than STATIC_SCRATCH_BYTES of workspace."""
    lib = load_library()
    B = int(y0.shape[0])
    tg = np.ascontiguousarray(np.asarray(tgrid, dtype=np.float64))
    N = int(tg.shape[0]) - 1
    _check_dev(theta, torch.float32, rampde_num_params(vel), "theta")
    _check_dev(y0, torch.float32, B * vel.d, "y0")
    _check_dev(ckpt, pol.torch_low, (N + 1) * B * vel.d, "ckpt")
    _check_dev(yN, torch.float32, B * vel.d, "yN")
    pc = pol.c
    rc = lib.rampde_odeint_fwd_static(C.byref(vel.c), _ptr(theta), _ptr(y0), B,
                                      tg.ctypes.data_as(C.POINTER(C.c_double)), N, C.byref(tab.c), C.byref(pc),
                                      _ptr(ckpt), _ptr(yN), _stream_ptr(stream))
    if rc != OK:
        raise RampdeError(rc, rampde_strerror(rc))
    return yN, ckpt


def rampde_odeint_bwd(vel: Velocity, theta: torch.Tensor, tgrid, tab: Tableau, pol: Policy, ckpt: torch.Tensor,
                      grad_yN: torch.Tensor, grad_ys: Optional[torch.Tensor] = None,
                      grad_y0: Optional[torch.Tensor] = None, grad_theta: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None, stream=None, want_info: bool = True,
                      grad_t: Optional[torch.Tensor] = None):
    """Discrete adjoint (paper Algorithm 2).  Returns (grad_y0, grad_theta, BwdInfo or None).

    grad_theta is accumulated into; when omitted a zero vector is created.  With `grad_t` (N+1 fp32
    on the device, accumulated into) the call goes to rampde_odeint_bwd_tgrid and also forms dL/dt.
    """
    lib = load_library()
    B = int(grad_yN.shape[0])
    tg = np.ascontiguousarray(np.asarray(tgrid, dtype=np.float64))
    N = int(tg.shape[0]) - 1
    P = rampde_num_params(vel)
    _check_dev(theta, torch.float32, P, "theta")
    _check_dev(grad_yN, torch.float32, B * vel.d, "grad_yN")
    _check_dev(ckpt, pol.torch_low, (N + 1) * B * vel.d, "ckpt")
    if grad_ys is not None:
        _check_dev(grad_ys, torch.float32, (N + 1) * B * vel.d, "grad_ys")
    if grad_y0 is None:
        grad_y0 = torch.empty_like(grad_yN)
    if grad_theta is None:
        grad_theta = torch.zeros(P, dtype=torch.float32, device=grad_yN.device)
    _check_dev(grad_y0, torch.float32, B * vel.d, "grad_y0")
    _check_dev(grad_theta, torch.float32, P, "grad_theta")
    if workspace is None:
        workspace = alloc_workspace(vel, B, N, tab, pol, True, grad_yN.device)
    pc = pol.c
    stats = _Stats()
    G = int(pol.scale_group)
    groups = (B + G - 1) // G if 0 < G < B else 1
    # one row of N + 1 scales per scale group (a plain vector without groups)
    hist = np.zeros(N + 1 if groups == 1 else (groups, N + 1), dtype=np.float32) if want_info else None
    hist_p = hist.ctypes.data_as(C.POINTER(C.c_float)) if want_info else None
    stats_p = C.byref(stats) if want_info else None
    if grad_t is not None:
        _check_dev(grad_t, torch.float32, N + 1, "grad_t")
        rc = lib.rampde_odeint_bwd_tgrid(C.byref(vel.c), _ptr(theta), B, tg.ctypes.data_as(C.POINTER(C.c_double)), N,
                                         C.byref(tab.c), C.byref(pc), _ptr(ckpt), _ptr(grad_yN), _ptr(grad_ys),
                                         _ptr(grad_y0), _ptr(grad_theta), _ptr(grad_t), hist_p, stats_p,
                                         _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    else:
        rc = lib.rampde_odeint_bwd(C.byref(vel.c), _ptr(theta), B, tg.ctypes.data_as(C.POINTER(C.c_double)), N,
                                   C.byref(tab.c), C.byref(pc), _ptr(ckpt), _ptr(grad_yN), _ptr(grad_ys),
                                   _ptr(grad_y0), _ptr(grad_theta), hist_p, stats_p, _ptr(workspace),
                                   workspace.numel(), _stream_ptr(stream))
    info = None
    if want_info:
        info = BwdInfo(stats.status, stats.failed_step, stats.retries, stats.s_first, stats.s_last, stats.s_min,
                       stats.s_max, hist)
    if rc != OK:
        raise RampdeError(rc, rampde_strerror(rc), info)
    return grad_y0, grad_theta, info


def rampde_odeint_bwd_tgrid(vel: Velocity, theta: torch.Tensor, tgrid, tab: Tableau, pol: Policy, ckpt: torch.Tensor,
                            grad_yN: torch.Tensor, grad_t: Optional[torch.Tensor] = None, **kw):
    """Discrete adjoint with the time-grid gradient (paper Sec. 3, update lines of t'; Algorithm 2).
    Returns (grad_y0, grad_theta, grad_t, BwdInfo or None); grad_t is accumulated into (zeros when omitted)."""
    if grad_t is None:
        grad_t = torch.zeros(len(tgrid), dtype=torch.float32, device=grad_yN.device)
    gy0, gth, info = rampde_odeint_bwd(vel, theta, tgrid, tab, pol, ckpt, grad_yN, grad_t=grad_t, **kw)
    return gy0, gth, grad_t, info
