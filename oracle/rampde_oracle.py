"""CPU oracle for the mixed-precision neural-ODE time-stepping path.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, step-by-step NumPy
implementation (fp64 arithmetic) of what the HIP library computes.  It shares
no code with the HIP path and must never be imported by it: only tests, the
smoke check and the benchmark's CPU-baseline leg may use it.

Two modes, selected by `low`:

* ``"f64"``  -- every quantiser is the identity and the adjoint scale is 1.
  Forward = the explicit Runge-Kutta recursion  y_{i+1} = y_i + h_i Phi(y_i)
  (paper Sec. 3, single-step form); backward = the exact gradient of that
  discrete map (discretise-then-optimise, paper Sec. 2).
* ``"f16"`` / ``"bf16"`` / ``"f32"``  -- rounding emulation: the same control
  flow with values rounded (round-to-nearest-even, through fp32) at the points
  where the scheme stores a low-precision or fp32 tensor: paper Algorithm 1
  (forward) and Algorithm 2 (backward with dynamic adjoint scaling).

Rounding points (the tensors a fused implementation materialises):
  R1 weights once per pass; R2 checkpoints Q(y); R3 stage inputs; R4 stage
  times; R5 post-tanh activations; R6 stage slopes k_j; R7 fp32 state update;
  R8 scaled adjoint Q(S a); R9 every cotangent of the VJP chain.
Dot products are accumulated in fp64 and rounded once to fp32 (standing for a
matrix unit with fp32 accumulators, paper Sec. 2 "block FMA"), then to `low`.

Readings of the paper that this file fixes (all listed in the design notes):
  * adjoint update uses a PLUS sign:  a_i = a_{i+1} + h (dPhi/dy)^T a_{i+1},
    the derivative of y_{i+1} = y_i + h Phi(y_i)  (pinned by finite differences);
  * the b-weighted stage sum is added to y in fp32 without an intermediate
    16-bit rounding (flag ``round_increment`` gives the literal Alg. 1 line);
  * the per-step parameter-gradient contribution stays in fp32 (Lemma 4.5 model);
  * the scale is doubled when  k == 1  and  S * max|a| <= 1/(2 u_L)
    (flag ``grow_raw_norm`` gives the literal unscaled test of Alg. 2).

Parity status: every function here is pinned by tests in
tests/test_oracle_pins.py (closed forms, finite differences, brute force,
the paper's worked example); nothing in this file is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

# unit roundoffs of the low-precision formats (paper Sec. 3: fp16 2^-11, bf16 2^-8)
_P_BITS = {"f16": 11, "bf16": 8, "f32": 24, "f64": 53}


# --------------------------------------------------------------------------
# Quantisers (paper Sec. 2: Q16, Q32; round-to-nearest-even, Sec. 4)
# --------------------------------------------------------------------------
def round_f32(x):
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_bf16_from_f32(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 (1 sign, 8 exponent, 7 mantissa bits), ties to even; result as fp32."""
    shape = np.shape(x32)
    x32 = np.ascontiguousarray(x32, dtype=np.float32).reshape(-1)
    u = x32.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    r = (r & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    isnan = np.isnan(x32)
    if np.any(isnan):
        r = np.where(isnan, np.uint32(0x7FC00000), r)
    return r.view(np.float32).reshape(shape)


def make_quantisers(low: str):
    """Return (Q, R32): Q rounds fp64 -> fp32 -> `low`; R32 rounds fp64 -> fp32.

    Both return fp64 arrays holding representable values.  In "f64" mode both
    are the identity.
    """
    if low == "f64":
        ident = lambda x: np.asarray(x, dtype=np.float64)
        return ident, ident
    if low == "f32":
        return round_f32, round_f32
    if low == "f16":
        def Q(x):
            with np.errstate(over="ignore"):
                r = np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float16)
            return r.astype(np.float64)
        return Q, round_f32
    if low == "bf16":
        def Q(x):
            with np.errstate(over="ignore"):
                x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
            return round_bf16_from_f32(x32).astype(np.float64)
        return Q, round_f32
    raise ValueError(low)


# --------------------------------------------------------------------------
# Velocity networks f(t, y; theta)
# --------------------------------------------------------------------------
class MLPVelocity:
    """f = W_L tanh( ... tanh(W_1 [z; t] + b_1) ... ) + b_L.

    theta layout: per layer W_l[out, in] row-major then b_l[out]; layer 1 has
    in = d + 1 with the time column last (when `time_input`).  `activation`
    "identity" turns the network into a linear map (used for the linear-ODE pins).
    """

    def __init__(self, widths: Sequence[int], time_input: bool = True, activation: str = "tanh"):
        self.widths = tuple(int(w) for w in widths)
        self.time_input = bool(time_input)
        self.activation = activation
        self.L = len(self.widths) - 1
        self.shapes = []
        off = 0
        for l in range(self.L):
            o = self.widths[l + 1]
            i = self.widths[l] + (1 if (l == 0 and self.time_input) else 0)
            self.shapes.append((o, i, off, off + o * i))
            off += o * i + o
        self.n_params = off

    def state_size(self):
        return self.widths[0]

    def split(self, theta: np.ndarray):
        """[(W[:, :in_state], w_t or None, b)] views of a flat parameter vector."""
        out = []
        for l, (o, i, woff, boff) in enumerate(self.shapes):
            Wfull = theta[woff:woff + o * i].reshape(o, i)
            b = theta[boff:boff + o]
            if l == 0 and self.time_input:
                out.append((Wfull[:, :-1], Wfull[:, -1], b))
            else:
                out.append((Wfull, None, b))
        return out

    def _act(self, x):
        return np.tanh(x) if self.activation == "tanh" else x

    def _dact_from_out(self, a):
        return (1.0 - a * a) if self.activation == "tanh" else np.ones_like(a)

    def eval(self, theta_q, z, tau, Q, R32):
        """k = f(tau, z).  z: [B, d] values already representable in `low`.

        Hidden activations are rounded after tanh (R5); the pre-activation
        W a + w_t tau + b is formed in the fp32 accumulator and not stored.
        """
        layers = self.split(theta_q)
        acts = [z]
        k = None
        for l, (W, wt, b) in enumerate(layers):
            pre = acts[-1] @ W.T + b
            if wt is not None:
                pre = pre + tau * wt
            pre = R32(pre)
            if l < self.L - 1:
                acts.append(Q(R32(self._act(pre))))
            else:
                k = Q(pre)
        return k, (acts, tau)

    def vjp(self, theta_q, cache, kbar, Q, R32):
        """Cotangents through one evaluation (paper eq. (vjp), network part).

        Returns (zbar, dtheta (flat fp64, unrounded), finite flag of every
        low-precision cotangent formed, taubar).  tanh' is taken from the stored
        rounded activation: 1 - act^2.  taubar = kbar^T df/dtau summed over the
        batch (the time entry of J_Phi in eq. (vjp)): the layer-1 cotangent times
        the time column, unrounded like dtheta.
        """
        acts, tau = cache
        layers = self.split(theta_q)
        dtheta = np.zeros(self.n_params, dtype=np.float64)
        delta = kbar
        finite = True
        zbar = None
        taubar = 0.0
        for l in range(self.L - 1, -1, -1):
            W, wt, b = layers[l]
            o, i, woff, boff = self.shapes[l]
            dWfull = np.zeros((o, i), dtype=np.float64)
            dWfull[:, :W.shape[1]] = delta.T @ acts[l]
            colsum = delta.sum(axis=0)
            if wt is not None:
                dWfull[:, -1] = colsum * tau
                taubar = float(colsum @ wt)
            dtheta[woff:woff + o * i] = dWfull.ravel()
            dtheta[boff:boff + o] = colsum
            back = R32(delta @ W)
            if l > 0:
                delta = Q(R32(back * self._dact_from_out(acts[l])))
                finite = finite and bool(np.all(np.isfinite(delta)))
            else:
                zbar = Q(back)
                finite = finite and bool(np.all(np.isfinite(zbar)))
        return zbar, dtheta, finite, taubar


class Conv2Velocity:
    """f = conv3x3([tanh(conv3x3([z; t]) + b1); t]) + b2, zero padding 1, NCHW.

    A constant channel holding t is appended to the input of each convolution
    (so it is zero in the padding ring like every other channel).  theta layout:
    W1[C, C+1, 3, 3], b1[C], W2[C, C+1, 3, 3], b2[C].
    """

    def __init__(self, C: int, H: int, W: int, time_input: bool = True):
        self.C, self.H, self.W = int(C), int(H), int(W)
        self.time_input = bool(time_input)
        self.Cin = self.C + (1 if self.time_input else 0)
        wsz = self.C * self.Cin * 9
        self.offs = [(0, wsz), (wsz + self.C, 2 * wsz + self.C)]
        self.n_params = 2 * (wsz + self.C)

    def state_size(self):
        return self.C * self.H * self.W

    def split(self, theta):
        out = []
        for (woff, boff) in self.offs:
            Wt = theta[woff:woff + self.C * self.Cin * 9].reshape(self.C, self.Cin, 3, 3)
            b = theta[boff:boff + self.C]
            out.append((Wt, b))
        return out

    def _with_time(self, x, tau):
        if not self.time_input:
            return x
        B = x.shape[0]
        tch = np.full((B, 1, self.H, self.W), tau, dtype=np.float64)
        return np.concatenate([x, tch], axis=1)

    def _conv(self, x, Wt):
        """out[b,o,y,x] = sum_{c,ky,kx} W[o,c,ky,kx] * xpad[b,c,y+ky,x+kx]."""
        B = x.shape[0]
        xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
        out = np.zeros((B, self.C, self.H, self.W), dtype=np.float64)
        for ky in range(3):
            for kx in range(3):
                out += np.einsum("oc,bchw->bohw", Wt[:, :, ky, kx],
                                 xp[:, :, ky:ky + self.H, kx:kx + self.W], optimize=True)
        return out, xp

    def _conv_T(self, delta, Wt):
        """Transpose of _conv with respect to its input (all input channels)."""
        B = delta.shape[0]
        dp = np.zeros((B, Wt.shape[1], self.H + 2, self.W + 2), dtype=np.float64)
        for ky in range(3):
            for kx in range(3):
                dp[:, :, ky:ky + self.H, kx:kx + self.W] += np.einsum(
                    "oc,bohw->bchw", Wt[:, :, ky, kx], delta, optimize=True)
        return dp[:, :, 1:-1, 1:-1]

    def _conv_dW(self, delta, xp):
        dW = np.zeros((self.C, xp.shape[1], 3, 3), dtype=np.float64)
        for ky in range(3):
            for kx in range(3):
                dW[:, :, ky, kx] = np.einsum("bohw,bchw->oc", delta,
                                             xp[:, :, ky:ky + self.H, kx:kx + self.W], optimize=True)
        return dW

    def eval(self, theta_q, z, tau, Q, R32):
        z4 = z.reshape(-1, self.C, self.H, self.W)
        (W1, b1), (W2, b2) = self.split(theta_q)
        pre1, xp1 = self._conv(self._with_time(z4, tau), W1)
        act1 = Q(R32(np.tanh(R32(pre1 + b1[None, :, None, None]))))
        pre2, xp2 = self._conv(self._with_time(act1, tau), W2)
        k = Q(R32(pre2 + b2[None, :, None, None]))
        return k.reshape(z.shape), (xp1, act1, xp2)

    def vjp(self, theta_q, cache, kbar, Q, R32):
        xp1, act1, xp2 = cache
        (W1, b1), (W2, b2) = self.split(theta_q)
        d2 = kbar.reshape(-1, self.C, self.H, self.W)
        dtheta = np.zeros(self.n_params, dtype=np.float64)
        (w1o, b1o), (w2o, b2o) = self.offs
        wsz = self.C * self.Cin * 9
        dtheta[w2o:w2o + wsz] = self._conv_dW(d2, xp2).ravel()
        dtheta[b2o:b2o + self.C] = d2.sum(axis=(0, 2, 3))
        full2 = self._conv_T(d2, W2)
        back2 = R32(full2[:, :self.C])
        d1 = Q(R32(back2 * (1.0 - act1 * act1)))
        dtheta[w1o:w1o + wsz] = self._conv_dW(d1, xp1).ravel()
        dtheta[b1o:b1o + self.C] = d1.sum(axis=(0, 2, 3))
        full1 = self._conv_T(d1, W1)
        zbar = Q(R32(full1[:, :self.C]))
        finite = bool(np.all(np.isfinite(d1))) and bool(np.all(np.isfinite(zbar)))
        # time cotangent: the input cotangent of the constant time channel of both convolutions
        taubar = float(full2[:, self.C].sum() + full1[:, self.C].sum()) if self.time_input else 0.0
        return zbar.reshape(kbar.shape), dtheta, finite, taubar


# 3x3 convolution, zero padding 1, stride 1 (NCHW), its transpose with respect to the input, and its
# weight gradient, written out tap by tap from the definition
def _conv3x3(x, Wt):
    """out[b,o,y,x] = sum_{c,ky,kx} W[o,c,ky,kx] * xpad[b,c,y+ky,x+kx]."""
    B, _, H, Wd = x.shape
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    out = np.zeros((B, Wt.shape[0], H, Wd), dtype=np.float64)
    for ky in range(3):
        for kx in range(3):
            out += np.einsum("oc,bchw->bohw", Wt[:, :, ky, kx], xp[:, :, ky:ky + H, kx:kx + Wd], optimize=True)
    return out


def _conv3x3_T(v, Wt):
    """in[b,c,y,x] = sum_{o,ky,kx} W[o,c,ky,kx] * vpad[b,o,y-ky+2,x-kx+2]: the transpose of _conv3x3 in x."""
    B, _, H, Wd = v.shape
    dp = np.zeros((B, Wt.shape[1], H + 2, Wd + 2), dtype=np.float64)
    for ky in range(3):
        for kx in range(3):
            dp[:, :, ky:ky + H, kx:kx + Wd] += np.einsum("oc,bohw->bchw", Wt[:, :, ky, kx], v, optimize=True)
    return dp[:, :, 1:-1, 1:-1]


def _conv3x3_dW(v, x):
    """d<v, conv3x3(x, W)>/dW[o,c,ky,kx] = sum_{b,y,x} v[b,o,y,x] * xpad[b,c,y+ky,x+kx]."""
    B, _, H, Wd = x.shape
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    dW = np.zeros((v.shape[1], x.shape[1], 3, 3), dtype=np.float64)
    for ky in range(3):
        for kx in range(3):
            dW[:, :, ky, kx] = np.einsum("bohw,bchw->oc", v, xp[:, :, ky:ky + H, kx:kx + Wd], optimize=True)
    return dW


class ParabolicConvVelocity:
    """f(y; W, b) = -W^T N( relu( W y + b ) )   (paper Sec. 6.3, eq. (NODE_STL10); App. "parabolic").

    W is a 3x3 convolution with C input and C output channels (zero padding 1), W^T its exact
    transpose with the SAME weights, N the instance normalisation: per sample and channel, over the
    H*W pixels, (r - mean) / sqrt(var + eps) with the biased variance and no affine parameters.
    Weights and biases are piecewise constant in time (Sec. 6.3: constant on each time interval):
    theta holds `n_intervals` blocks (W[C,C,3,3], b[C]); step i of an N-step grid uses block
    i * n_intervals // N for all of its stages.  There is no explicit time input.

    Rounding points in emulation mode (readings; the paper runs this block under autocast): the
    post-ReLU activation, the normalised activation and the slope are rounded to `low`; the
    convolution sums, the statistics (mean, variance, 1/sqrt) and the normalisation arithmetic are
    fp32.  The VJP of N uses the stored (rounded) normalised activation and the fp32 statistics; the
    ReLU mask is r > 0 of the stored activation; dn, du and zbar are rounded to `low`.
    """

    time_input = False

    def __init__(self, C: int, H: int, W: int, n_intervals: int = 1, eps: float = 1e-5):
        self.C, self.H, self.W = int(C), int(H), int(W)
        self.n_intervals = int(n_intervals)
        self.eps = float(eps)
        self.block = self.C * self.C * 9 + self.C
        self.n_params = self.n_intervals * self.block

    def state_size(self):
        return self.C * self.H * self.W

    def step_slice(self, i: int, N: int) -> slice:
        j = (i * self.n_intervals) // N
        return slice(j * self.block, (j + 1) * self.block)

    def _split(self, theta_blk):
        wsz = self.C * self.C * 9
        return theta_blk[:wsz].reshape(self.C, self.C, 3, 3), theta_blk[wsz:wsz + self.C]

    def eval(self, theta_blk, z, tau, Q, R32):
        Wt, b = self._split(theta_blk)
        z4 = z.reshape(-1, self.C, self.H, self.W)
        r = Q(R32(np.maximum(R32(_conv3x3(z4, Wt) + b[None, :, None, None]), 0.0)))
        mu = R32(r.mean(axis=(2, 3), keepdims=True))
        var = R32(((r - mu) ** 2).mean(axis=(2, 3), keepdims=True))
        rstd = R32(1.0 / np.sqrt(var + self.eps))
        n = Q(R32((r - mu) * rstd))
        k = Q(R32(-_conv3x3_T(n, Wt)))
        return k.reshape(z.shape), (z4, r, n, rstd)

    def vjp(self, theta_blk, cache, kbar, Q, R32):
        z4, r, n, rstd = cache
        Wt, b = self._split(theta_blk)
        kb4 = kbar.reshape(z4.shape)
        dn = Q(R32(-_conv3x3(kb4, Wt)))
        m1 = R32(dn.mean(axis=(2, 3), keepdims=True))
        m2 = R32((dn * n).mean(axis=(2, 3), keepdims=True))
        du = Q(R32(rstd * (dn - m1 - n * m2)) * (r > 0.0))
        zbar = Q(R32(_conv3x3_T(du, Wt)))
        dtheta = np.zeros(self.block, dtype=np.float64)
        wsz = self.C * self.C * 9
        # k = -W^T n is linear in W with "input" kbar and "output cotangent" n
        dtheta[:wsz] = (_conv3x3_dW(du, z4) - _conv3x3_dW(n, kb4)).ravel()
        dtheta[wsz:] = du.sum(axis=(0, 2, 3))
        finite = bool(np.all(np.isfinite(dn))) and bool(np.all(np.isfinite(du))) and bool(np.all(np.isfinite(zbar)))
        return zbar.reshape(kbar.shape), dtheta, finite, None


class CNFVelocity:
    """Augmented state of a continuous normalising flow (paper Sec. 6.1):  y = [z; l],

        dz/dt = v(t, z),      dl/dt = -tr(dv/dz),

    with the trace formed analytically (the paper replaces the stochastic estimator by the direct
    trace).  The velocity is one hidden layer, v = W2 tanh(W1 [z; t] + b1) + b2 -- the summed-tanh-units
    form of the paper's CNF velocity with the weights given directly instead of through a hypernetwork --
    for which   tr(dv/dz) = sum_h c_h (1 - a_h^2),   c_h = sum_i W2[i,h] W1[h,i],   a = tanh(.).
    theta layout: that of MLPVelocity((d, H, d)): W1[H, d+1] (time column last), b1[H], W2[d, H], b2[d].
    The state has d + 1 columns; the velocity does not depend on l.

    Rounding points in emulation mode: those of the MLP (activation, slope) plus: c_h and the trace sum
    are fp32 (from the rounded weights and the rounded activation), dl/dt is rounded to `low` like the
    other slope entries; in the VJP the cotangent of the activation gets the extra term 2 kbar_l c_h a_h
    inside the fp32 sum before the tanh' factor and the rounding.
    """

    time_input = True

    def __init__(self, d: int, H: int):
        self.d, self.H = int(d), int(H)
        self.mlp = MLPVelocity((self.d, self.H, self.d), time_input=True)
        self.n_params = self.mlp.n_params

    def state_size(self):
        return self.d + 1

    def eval(self, theta_q, y, tau, Q, R32):
        (W1, wt, b1), (W2, _, b2) = self.mlp.split(theta_q)
        z = y[:, :self.d]
        a = Q(R32(np.tanh(R32(z @ W1.T + tau * wt + b1))))
        v = Q(R32(a @ W2.T + b2))
        c = R32(np.einsum("ih,hi->h", W2, W1))
        ldot = Q(R32(-((1.0 - a * a) @ c)))
        return np.concatenate([v, ldot[:, None]], axis=1), (z, a, c, tau)

    def vjp(self, theta_q, cache, kbar, Q, R32):
        z, a, c, tau = cache
        (W1, wt, b1), (W2, _, b2) = self.mlp.split(theta_q)
        (o1, i1, w1off, b1off), (o2, i2, w2off, b2off) = self.mlp.shapes
        kz, kl = kbar[:, :self.d], kbar[:, self.d]
        dtheta = np.zeros(self.n_params, dtype=np.float64)
        s = kl @ (1.0 - a * a)                       # cotangent of -c_h (batch sums)
        dW2 = kz.T @ a - W1.T * s[None, :]
        dtheta[w2off:w2off + o2 * i2] = dW2.ravel()
        dtheta[b2off:b2off + o2] = kz.sum(axis=0)
        back = R32(kz @ W2 + 2.0 * kl[:, None] * (c[None, :] * a))
        d1 = Q(R32(back * (1.0 - a * a)))
        dW1 = np.zeros((o1, i1))
        dW1[:, :self.d] = d1.T @ z - W2.T * s[:, None]
        colsum = d1.sum(axis=0)
        dW1[:, -1] = colsum * tau
        dtheta[w1off:w1off + o1 * i1] = dW1.ravel()
        dtheta[b1off:b1off + o1] = colsum
        zbar = Q(R32(d1 @ W1))
        finite = bool(np.all(np.isfinite(d1))) and bool(np.all(np.isfinite(zbar)))
        ybar = np.concatenate([zbar, np.zeros((len(zbar), 1))], axis=1)
        return ybar, dtheta, finite, float(colsum @ wt)


class PolyDecayVelocity:
    """Scalar test problem of the paper's Example 3.1:  y' = -(th1 t^2 + th2 t + th3) y.

    Every elementwise operation is rounded to `low` (the paper does not state
    the rounding granularity inside this f; this is what eager 16-bit execution
    would do).  The time passed in is the unrounded stage time: the example's
    lambda(t) is evaluated from t inside the low-precision arithmetic.
    """
    n_params = 3
    time_input = True
    exact_time = True  # stage time is rounded inside eval, not by the stepper

    def state_size(self):
        return 1

    def eval(self, theta_q, z, tau, Q, R32):
        t = tau
        t2 = Q(t * t)
        lam = Q(Q(Q(theta_q[0] * t2) + Q(theta_q[1] * t)) + theta_q[2])
        k = Q(-(lam * z))
        return k, (z, t, t2, lam)

    def vjp(self, theta_q, cache, kbar, Q, R32):
        z, t, t2, lam = cache
        zbar = Q(-(lam * kbar))
        lbar = Q(-(z * kbar))                      # cotangent of lambda, per sample
        dtheta = np.array([np.sum(Q(lbar * t2)), np.sum(Q(lbar * t)), np.sum(lbar)], dtype=np.float64)
        finite = bool(np.all(np.isfinite(zbar))) and bool(np.all(np.isfinite(lbar))) \
            and bool(np.all(np.isfinite(dtheta)))
        return zbar, dtheta, finite, None   # (time cotangent not formed for this test problem)


# --------------------------------------------------------------------------
# Policy / results
# --------------------------------------------------------------------------
@dataclass
class Policy:
    low: str = "f64"                 # "f64" | "f32" | "f16" | "bf16"
    scaling: str = "none"            # "none" | "none_safe" | "dynamic"
    k_max: int = 16
    round_increment: bool = False    # literal Alg. 1: round sum_j b_j k_j to low before the fp32 add
    grow_raw_norm: bool = False      # literal Alg. 2 growth test on the unscaled norm
    naive_state: bool = False        # oracle-only: keep y and a in low precision (no fp32 accumulator)
    scale_group: int = 0             # samples that share one adjoint scale; 0 = the whole batch (see odeint_bwd)


@dataclass
class BwdResult:
    grad_y0: np.ndarray
    grad_theta: np.ndarray
    scale_hist: np.ndarray           # [N+1]: S_N at index N, accepted S_i at index i ([groups, N+1] with scale groups)
    retries: int
    status: str                      # "ok" | "overflow_inf" | "scale_failed"
    failed_step: int = -1
    grad_t: np.ndarray = None        # [N+1] dL/dt (None when the velocity forms no time cotangent)


class ScaleFailure(Exception):
    """Dynamic adjoint scaling failed at a step (paper Alg. 2, error branch)."""

    def __init__(self, step):
        super().__init__(f"dynamic adjoint scaling failed at step {step}")
        self.step = step


def initial_scale(amax: float, low: str) -> float:
    """S_N = 2^floor(-log2(u_L * ||a||_inf))  (paper Sec. 3 / Alg. 2, initialisation).

    Edge cases the paper leaves open: ||a|| = 0 -> 1; result clamped to [2^-126, 2^126].
    """
    if amax == 0.0:
        return 1.0
    u = 2.0 ** (-_P_BITS[low])
    e = math.floor(-math.log2(u * amax))
    e = max(-126, min(126, e))
    return 2.0 ** e


# --------------------------------------------------------------------------
# Stage recursion shared by forward and backward recomputation
# --------------------------------------------------------------------------
def _step_theta(vel, theta_q, i, N):
    """The parameters step i uses: all of them, or the step's block when the velocity's parameters are
    piecewise constant in time (paper Sec. 6.3)."""
    return theta_q[vel.step_slice(i, N)] if hasattr(vel, "step_slice") else theta_q


def _stages(vel, theta_q, yhat, t_i, h, tab_A, tab_c, Q, R32):
    """Stage inputs z_j, times tau_j, slopes k_j of one explicit RK step (Phi's inside)."""
    s = len(tab_c)
    ks, caches = [], []
    for j in range(s):
        if j == 0:
            z = yhat
        else:
            incr = np.zeros_like(yhat)
            for l in range(j):
                if tab_A[j][l] != 0.0:
                    incr = incr + tab_A[j][l] * ks[l]
            z = Q(yhat + h * incr)                                   # R3
        tau = Q(R32(t_i + tab_c[j] * h))                                # R4
        k, cache = vel.eval(theta_q, z, float(tau), Q, R32)            # R5, R6
        ks.append(k)
        caches.append(cache)
    return ks, caches


def odeint_fwd(vel, theta, y0, tgrid, tableau, policy: Policy):
    """Mixed-precision forward pass (paper Algorithm 1).

    Returns (y_N in the accumulator precision, checkpoints [N+1, ...] in `low`),
    both as fp64 arrays holding representable values.
    """
    Q, R32 = make_quantisers(policy.low)
    A, b, c = tableau.A, tableau.b, tableau.c
    tgrid = np.asarray(tgrid, dtype=np.float64)
    N = len(tgrid) - 1
    theta_q = Q(np.asarray(theta, dtype=np.float64))                   # R1
    y = R32(np.asarray(y0, dtype=np.float64)).reshape(len(y0), -1)
    if policy.naive_state:
        y = Q(y)
    ckpt = [Q(y)]                                                      # R2
    for i in range(N):
        h = float(R32(tgrid[i + 1] - tgrid[i]))
        yhat = ckpt[i]
        ks, _ = _stages(vel, _step_theta(vel, theta_q, i, N), yhat, tgrid[i], h, A, c, Q, R32)
        incr = np.zeros_like(y)
        for j in range(len(b)):
            incr = incr + b[j] * ks[j]
        if policy.round_increment:
            incr = Q(incr)
        y = R32(y + h * incr)                                          # R7
        if policy.naive_state:
            y = Q(y)
        ckpt.append(Q(y))                                              # R2
    return y.reshape(np.shape(y0)), np.stack(ckpt).reshape((N + 1,) + tuple(np.shape(y0)))


def odeint_bwd(vel, theta, tgrid, tableau, policy: Policy, ckpt, grad_yN,
               grad_theta_init=None, grad_ys=None, grad_t_init=None) -> BwdResult:
    """Algorithm 2 on a batch, with the scope of the adjoint scale made explicit.

    The paper states Alg. 2 for one sample: one adjoint vector, one scale S.  With a batch,
    policy.scale_group = 0 treats the whole batch tensor as that vector (one S for all samples).
    policy.scale_group = G > 0 applies Alg. 2 to every block of G consecutive samples (the last block:
    the remainder) on its own: own S_N from the block's max-norm, own retries, own growth; the blocks
    share theta, and each adds its h/S-unscaled share to the one gradient accumulator g (and t'), in
    batch order.  Samples do not interact in the velocity, so without overflow or underflow both give
    the same gradient up to the order of the fp32 sums.
    """
    B = np.shape(grad_yN)[0]
    G = int(policy.scale_group)
    if not 0 < G < B:
        return _odeint_bwd_one_scale(vel, theta, tgrid, tableau, policy, ckpt, grad_yN, grad_theta_init, grad_ys,
                                     grad_t_init)
    ckpt = np.asarray(ckpt)
    grad_yN = np.asarray(grad_yN)
    g, tp = grad_theta_init, grad_t_init
    a0, hists, retries = [], [], 0
    for b0 in range(0, B, G):
        rows = slice(b0, min(b0 + G, B))
        res = _odeint_bwd_one_scale(vel, theta, tgrid, tableau, policy, ckpt[:, rows], grad_yN[rows], g,
                                    None if grad_ys is None else np.asarray(grad_ys)[:, rows], tp)
        retries += res.retries
        hists.append(res.scale_hist)
        if res.status == "scale_failed":
            # (outputs are undefined after a failure: the groups that never ran are left as NaN)
            part = np.full(np.shape(grad_yN), np.nan)
            part[:rows.start] = np.concatenate(a0, axis=0) if a0 else part[:0]
            part[rows] = res.grad_y0
            return BwdResult(part, res.grad_theta, np.stack(hists), retries, res.status, res.failed_step)
        if res.status == "overflow_inf":
            return BwdResult(np.full(np.shape(grad_yN), np.inf), res.grad_theta, np.stack(hists), retries,
                             res.status, res.failed_step)
        a0.append(res.grad_y0)
        g, tp = res.grad_theta, res.grad_t
    return BwdResult(np.concatenate(a0, axis=0), g, np.stack(hists), retries, "ok", -1, tp)


def _odeint_bwd_one_scale(vel, theta, tgrid, tableau, policy: Policy, ckpt, grad_yN,
                          grad_theta_init=None, grad_ys=None, grad_t_init=None) -> BwdResult:
    """Mixed-precision discrete adjoint with dynamic adjoint scaling (paper Algorithm 2).

    `grad_ys` (optional, [N+1, ...]) are per-step cotangents dL/dy_i of a running
    cost, added in high precision.

    Time-grid gradient t' = dL/dt (paper Sec. 3, the two update lines for t'_i and
    t'_{i+1}; Alg. 2): with the step y_{i+1} = y_i + h Phi(y_i, t_i, h), h = t_{i+1} - t_i,
        dt = lambda^T dPhi/dt = sum_j taubar_j,
        dh = lambda^T dPhi/dh = sum_j ( c_j taubar_j + zbar_j^T sum_l a_jl k_l ),
        t'_i     += (h/S)(dt - dh) - Phi^T a_{i+1},      t'_{i+1} += (h/S) dh + Phi^T a_{i+1},
    where taubar_j, zbar_j come from the same low-precision cotangent chain as da and
    dg, the sums are formed in the accumulator precision (not rounded to `low`, like
    dg), Phi = sum_j b_j k_j from the low-precision slopes, and a_{i+1} is the fp32
    adjoint before this step's update.  `grad_t_init` is the explicit dL/dt it starts from.
    """
    Q, R32 = make_quantisers(policy.low)
    A, b, c = tableau.A, tableau.b, tableau.c
    s = len(b)
    tgrid = np.asarray(tgrid, dtype=np.float64)
    N = len(tgrid) - 1
    B = np.shape(grad_yN)[0]
    flat = lambda x: np.asarray(x, dtype=np.float64).reshape(B, -1)
    dynamic = policy.scaling == "dynamic" and policy.low != "f64"
    check = dynamic or policy.scaling == "none_safe"
    u_low = 2.0 ** (-_P_BITS[policy.low])

    a = R32(flat(grad_yN))
    if grad_ys is not None:
        a = R32(a + flat(grad_ys[N]))
    if policy.naive_state:
        a = Q(a)
    g = np.zeros(vel.n_params) if grad_theta_init is None else R32(np.asarray(grad_theta_init, np.float64))
    theta_q = Q(np.asarray(theta, dtype=np.float64))
    scale_hist = np.ones(N + 1)
    retries = 0
    tp = np.zeros(N + 1) if grad_t_init is None else R32(np.asarray(grad_t_init, np.float64)).copy()
    have_t = True

    if dynamic:
        amax = float(np.max(np.abs(a))) if a.size else 0.0
        if not math.isfinite(amax):
            return BwdResult(a.reshape(np.shape(grad_yN)), g, scale_hist, 0, "scale_failed", N)
        S = initial_scale(amax, policy.low)
    else:
        S = 1.0
    scale_hist[N] = S

    for i in range(N - 1, -1, -1):
        h = float(R32(tgrid[i + 1] - tgrid[i]))
        yhat = flat(ckpt[i])
        th_i = _step_theta(vel, theta_q, i, N)
        ks, caches = _stages(vel, th_i, yhat, tgrid[i], h, A, c, Q, R32)   # recompute

        k_used = 0
        k_lim = policy.k_max if dynamic else 1
        while True:
            k_used += 1
            lam = Q(R32(S * a))                                        # R8
            finite = bool(np.all(np.isfinite(lam)))
            zbars = [None] * s
            taubars = [0.0] * s
            dth = np.zeros(len(th_i))
            for j in range(s - 1, -1, -1):
                kb = b[j] * lam
                for l in range(j + 1, s):
                    if A[l][j] != 0.0:
                        kb = kb + h * A[l][j] * zbars[l]
                kb = Q(R32(kb))                                        # R9a
                finite = finite and bool(np.all(np.isfinite(kb)))
                zbars[j], dth_j, fin_j, taubars[j] = vel.vjp(th_i, caches[j], kb, Q, R32)   # R9b, R9c
                finite = finite and fin_j
                dth = dth + dth_j
            if finite or not check:
                break
            if not dynamic:
                break
            if k_used >= k_lim:
                break
            S = S / 2.0
            retries += 1

        if check and not finite:
            if dynamic:
                return BwdResult(a.reshape(np.shape(grad_yN)), g, scale_hist, retries, "scale_failed", i)
            inf_a = np.full_like(a, np.inf)
            return BwdResult(inf_a.reshape(np.shape(grad_yN)), np.full_like(g, np.inf), scale_hist,
                             retries, "overflow_inf", i)

        scale_hist[i] = S
        hs = float(R32(h / S))
        da = np.zeros_like(a)
        for j in range(s):
            da = da + zbars[j]
        if have_t and taubars[0] is None:
            have_t = False
        if have_t:
            dt = 0.0
            dh = 0.0
            phi = np.zeros_like(a)
            for j in range(s):
                dt += taubars[j]
                stage_incr = np.zeros_like(a)
                for l in range(j):
                    if A[j][l] != 0.0:
                        stage_incr = stage_incr + A[j][l] * ks[l]
                dh += c[j] * taubars[j] + float(np.sum(zbars[j] * stage_incr))
                phi = phi + b[j] * ks[j]
            phi_a = float(R32(np.sum(phi * a)))
            tp[i] = R32(tp[i] + hs * float(R32(dt - dh)) - phi_a)
            tp[i + 1] = R32(tp[i + 1] + hs * float(R32(dh)) + phi_a)
        a_new = a + hs * da
        if grad_ys is not None:
            a_new = a_new + flat(grad_ys[i])
        a = R32(a_new)
        if policy.naive_state:
            a = Q(a)
        if hasattr(vel, "step_slice"):
            # parameters that are piecewise constant in time: the step's gradient goes to its own block
            blk = vel.step_slice(i, N)
            g[blk] = R32(g[blk] + hs * R32(dth))
        else:
            g = R32(g + hs * R32(dth))
        if dynamic and k_used == 1:
            amax = float(np.max(np.abs(a))) if a.size else 0.0
            test = amax if policy.grow_raw_norm else S * amax
            if test <= 1.0 / (2.0 * u_low) and S < 2.0 ** 126:
                S = 2.0 * S
    return BwdResult(a.reshape(np.shape(grad_yN)), g, scale_hist, retries, "ok", -1, tp if have_t else None)


def checkpoint_bytes(N: int, n_state: int, low: str) -> int:
    """Bytes held by the low-precision state trajectory (paper Sec. 3: only states are kept)."""
    return (N + 1) * n_state * {"f16": 2, "bf16": 2, "f32": 4, "f64": 8}[low]
