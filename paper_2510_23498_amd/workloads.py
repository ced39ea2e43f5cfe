"""Seeded synthetic inputs for the mixed-precision neural-ODE time-stepping path.

This module only *describes and generates inputs*: configurations (sizes, grids,
Butcher tableaux, precision names), parameter/state/target tensors, and the
caller-side loss gradients.  It holds none of the method's arithmetic (no
rounding operators, no Runge-Kutta stepping, no adjoint), so both the HIP path
and the independent CPU oracle may be fed from it.

Random numbers: counter-based splitmix64 -> two uniforms -> Box-Muller in fp64
-> cast to fp32.  Every tensor has its own stream, keyed by (seed, name).

The five configurations follow the workloads the benchmark names: MLP velocity
fields  f = W_L tanh(... tanh(W_1 [y;t] + b_1) ...) + b_L  and a two-convolution
velocity field with a constant time channel, integrated with explicit
Runge-Kutta schemes on a uniform grid (paper Sec. 3, Algorithm 1).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

_MASK64 = (1 << 64) - 1


def _fnv1a64(name: str) -> int:
    h = 0xCBF29CE484222325
    for ch in name.encode("utf-8"):
        h ^= ch
        h = (h * 0x100000001B3) & _MASK64
    return h


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One splitmix64 output per 64-bit counter value (vectorised, wraps mod 2^64)."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def uniforms(seed: int, name: str, count: int) -> np.ndarray:
    """`count` uniforms in (0,1), fp64, from the stream (seed, name)."""
    base = (_fnv1a64(name) ^ ((seed * 0xD6E8FEB86659FD93) & _MASK64)) & _MASK64
    ctr = (np.arange(count, dtype=np.uint64) + np.uint64(base))
    bits = _splitmix64(ctr)
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / (1 << 53))


def normals(seed: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    """Standard normals (Box-Muller on consecutive uniform pairs), scaled, fp32."""
    count = int(np.prod(shape))
    m = (count + 1) // 2
    u = uniforms(seed, name, 2 * m)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    ang = 2.0 * np.pi * u[1::2]
    z = np.empty(2 * m, dtype=np.float64)
    z[0::2] = r * np.cos(ang)
    z[1::2] = r * np.sin(ang)
    return (std * z[:count]).astype(np.float32).reshape(shape)


# --------------------------------------------------------------------------
# Butcher tableaux (inputs of the method: data, not arithmetic)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Tableau:
    name: str
    A: Tuple[Tuple[float, ...], ...]
    b: Tuple[float, ...]
    c: Tuple[float, ...]

    @property
    def s(self) -> int:
        return len(self.b)


TABLEAUX: Dict[str, Tableau] = {
    "euler": Tableau("euler", ((0.0,),), (1.0,), (0.0,)),
    # explicit trapezoid
    "heun": Tableau("heun", ((0.0, 0.0), (1.0, 0.0)), (0.5, 0.5), (0.0, 1.0)),
    "rk4": Tableau(
        "rk4",
        ((0.0, 0.0, 0.0, 0.0), (0.5, 0.0, 0.0, 0.0), (0.0, 0.5, 0.0, 0.0), (0.0, 0.0, 1.0, 0.0)),
        (1.0 / 6.0, 1.0 / 3.0, 1.0 / 3.0, 1.0 / 6.0),
        (0.0, 0.5, 0.5, 1.0),
    ),
    # Kutta's third-order scheme: a non-trivial lower triangle (a31 and a32 both
    # non-zero), used by tests so that a transposed tableau cannot go unnoticed.
    "kutta3": Tableau(
        "kutta3",
        ((0.0, 0.0, 0.0), (0.5, 0.0, 0.0), (-1.0, 2.0, 0.0)),
        (1.0 / 6.0, 2.0 / 3.0, 1.0 / 6.0),
        (0.0, 0.5, 1.0),
    ),
}


# --------------------------------------------------------------------------
# Configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    kind: str  # "mlp", "conv2", "parabolic" or "cnf" (widths = (d, H, d); the state has d + 1 columns)
    B: int
    low: str  # "f16" | "bf16"
    tableau: str
    N: int
    t0: float
    t1: float
    widths: Tuple[int, ...] = ()  # mlp: (d, hidden..., d); the time column is implicit
    C: int = 0  # conv2, parabolic
    H: int = 0
    W: int = 0
    n_intervals: int = 1  # parabolic: pieces of the piecewise-constant parameters
    loss: str = "half_sse"  # "half_sse" | "mse" | "mean_sq"
    grad_scale: float = 1.0
    scaling: str = "auto"  # "none" | "dynamic" | "auto"
    seed: int = 0

    @property
    def d(self) -> int:
        if self.kind == "cnf":
            return self.widths[0] + 1
        return self.widths[0] if self.kind == "mlp" else self.C * self.H * self.W

    @property
    def state_shape(self) -> Tuple[int, ...]:
        if self.kind == "cnf":
            return (self.B, self.widths[0] + 1)
        return (self.B, self.widths[0]) if self.kind == "mlp" else (self.B, self.C, self.H, self.W)

    @property
    def n_params(self) -> int:
        if self.kind in ("mlp", "cnf"):
            return sum((self.widths[l] + (1 if l == 0 else 0)) * self.widths[l + 1] + self.widths[l + 1]
                       for l in range(len(self.widths) - 1))
        if self.kind == "parabolic":
            return self.n_intervals * (self.C * self.C * 9 + self.C)
        return 2 * (self.C * (self.C + 1) * 9 + self.C)

    def tgrid(self) -> np.ndarray:
        return np.linspace(self.t0, self.t1, self.N + 1, dtype=np.float64)

    def with_(self, **kw) -> "Config":
        return replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    "cfg1": Config("cfg1", "mlp", B=256, low="f16", tableau="rk4", N=8, t0=0.0, t1=1.0,
                   widths=(2, 32, 32, 2), loss="half_sse"),
    "cfg2": Config("cfg2", "mlp", B=4096, low="bf16", tableau="rk4", N=32, t0=0.0, t1=1.0,
                   widths=(64, 256, 256, 64), loss="mse"),
    "cfg3": Config("cfg3", "mlp", B=16384, low="f16", tableau="rk4", N=64, t0=0.0, t1=2.0,
                   widths=(128, 512, 512, 512, 128), loss="half_sse", grad_scale=1e-6,
                   scaling="dynamic"),
    "cfg4": Config("cfg4", "conv2", B=128, low="f16", tableau="rk4", N=16, t0=0.0, t1=1.0,
                   C=64, H=32, W=32, loss="mean_sq"),
    "cfg5": Config("cfg5", "mlp", B=1024, low="f16", tableau="rk4", N=256, t0=0.0, t1=1.0,
                   widths=(256, 1024, 1024, 256), loss="mse"),
    # normalising-flow state [z; l] with the exact trace row (Sec. 6.1), at the sizes of the paper's second
    # generative workload (Sec. 6.2): 63 features + time = 64 network inputs, width 1024, batch 512, 16 RK4 steps
    "cnf": Config("cnf", "cnf", B=512, low="f16", tableau="rk4", N=16, t0=0.0, t1=1.0,
                  widths=(63, 1024, 63), loss="half_sse", grad_scale=1e-3),
    # the middle neural-ODE block of the paper's image classifier (Sec. 6.3): 256 channels, 64 x 64
    # pixels, batch 16, four RK4 steps with weights that are constant on each step
    "parab": Config("parab", "parabolic", B=16, low="f16", tableau="rk4", N=4, t0=0.0, t1=1.0,
                    C=256, H=64, W=64, n_intervals=4, loss="mean_sq"),
}


def mlp_layer_shapes(widths) -> List[Tuple[int, int]]:
    """[(out, in_including_time_column)] per layer; only layer 1 has the time column."""
    return [(widths[l + 1], widths[l] + (1 if l == 0 else 0)) for l in range(len(widths) - 1)]


def theta_layout(cfg: Config) -> List[Tuple[str, Tuple[int, ...], int]]:
    """[(name, shape, offset)] of the flat fp32 parameter vector.

    MLP: per layer W_l[out, in] row-major (layer 1: in = d + 1, time column last),
    then b_l[out].  Conv: W[C_out, C_in + 1, 3, 3] (time channel last) then b[C_out],
    for each of the two convolutions.
    """
    out: List[Tuple[str, Tuple[int, ...], int]] = []
    off = 0
    if cfg.kind in ("mlp", "cnf"):
        for l, (o, i) in enumerate(mlp_layer_shapes(cfg.widths)):
            out.append((f"W{l + 1}", (o, i), off)); off += o * i
            out.append((f"b{l + 1}", (o,), off)); off += o
    elif cfg.kind == "parabolic":
        for q in range(cfg.n_intervals):
            out.append((f"W{q + 1}", (cfg.C, cfg.C, 3, 3), off)); off += cfg.C * cfg.C * 9
            out.append((f"b{q + 1}", (cfg.C,), off)); off += cfg.C
    else:
        for l in range(2):
            shp = (cfg.C, cfg.C + 1, 3, 3)
            out.append((f"W{l + 1}", shp, off)); off += int(np.prod(shp))
            out.append((f"b{l + 1}", (cfg.C,), off)); off += cfg.C
    return out


def n_params(cfg: Config) -> int:
    name, shp, off = theta_layout(cfg)[-1]
    return off + int(np.prod(shp))


def make_theta(cfg: Config, bias_std: float = 0.0) -> np.ndarray:
    """Flat fp32 parameter vector.

    MLP: W ~ N(0, 1/fan_in), fan_in counting the time column; b = 0.
    Conv: He-normal, std = sqrt(2/fan_in), fan_in = (C+1)*9; b = 0.
    Parabolic block: W ~ N(0, 1/fan_in), fan_in = 9 C (the normalised activation has unit variance and
    W^T W then has O(1) gain, so the state neither dies nor blows up over t in [0,1]); b = 0.
    `bias_std` > 0 draws non-zero biases (used by tests so that the bias path
    cannot be wrong unnoticed).
    """
    theta = np.zeros(n_params(cfg), dtype=np.float32)
    for name, shp, off in theta_layout(cfg):
        cnt = int(np.prod(shp))
        if name.startswith("W"):
            fan_in = int(np.prod(shp[1:]))
            std = (2.0 / fan_in) ** 0.5 if cfg.kind == "conv2" else (1.0 / fan_in) ** 0.5
            theta[off:off + cnt] = normals(cfg.seed, f"{cfg.name}.theta.{name}", (cnt,), std)
        elif bias_std > 0.0:
            theta[off:off + cnt] = normals(cfg.seed, f"{cfg.name}.theta.{name}", (cnt,), bias_std)
    return theta


def make_y0(cfg: Config) -> np.ndarray:
    return normals(cfg.seed, f"{cfg.name}.y0", cfg.state_shape)


def make_target(cfg: Config) -> np.ndarray:
    return normals(cfg.seed, f"{cfg.name}.target", cfg.state_shape)


def loss_and_grad(cfg: Config, yN: np.ndarray, target: Optional[np.ndarray]):
    """Caller-side terminal loss C(y_N) and its fp32 gradient dC/dy_N.

    The loss lives outside the library; the same fp32 formula feeds both the HIP
    path and the oracle.  `grad_scale` multiplies the gradient (and the loss).
    """
    y = yN.astype(np.float32)
    if cfg.loss == "half_sse":
        r = y - target.astype(np.float32)
        loss = 0.5 * float(np.sum(r.astype(np.float64) ** 2))
        g = r
    elif cfg.loss == "mse":
        r = y - target.astype(np.float32)
        loss = float(np.mean(r.astype(np.float64) ** 2))
        g = (np.float32(2.0 / r.size) * r)
    elif cfg.loss == "mean_sq":
        loss = float(np.mean(y.astype(np.float64) ** 2))
        g = (np.float32(2.0 / y.size) * y)
    else:
        raise ValueError(cfg.loss)
    gs = np.float32(cfg.grad_scale)
    return loss * float(gs), (gs * g).astype(np.float32)


def resolve_scaling(cfg: Config) -> str:
    """'auto': fp32/bf16 -> none, fp16 -> dynamic (paper Sec. 5, variant selection)."""
    if cfg.scaling != "auto":
        return cfg.scaling
    return "dynamic" if cfg.low == "f16" else "none"
