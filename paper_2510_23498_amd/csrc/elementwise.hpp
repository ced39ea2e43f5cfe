// Streaming kernels of the time stepper: weight rounding, stage inputs, the fp32
// solution update with the low-precision checkpoint store (paper Algorithm 1), and the
// adjoint-side kernels: scale-and-round, overflow detection, fp32 adjoint update and
// the scale state machine (paper Algorithm 2).
#pragma once
#include <algorithm>
#include "common.hpp"

namespace rampde {

struct Coefs {
  float v[kMaxStages];
};

__device__ inline bool poisoned(const Ctl* ctl) { return ctl && ctl->poison; }

// theta (fp32) -> padded low-precision operands of one dense layer:
//   Wp [Npad][Kpad]  (W rounded, zero padded),  WTp [Kpad][Npad]  (its transpose),
//   bias_f[Npad], wt_f[Npad]: rounded bias / time-column, kept as fp32 for the epilogue.
template <class T>
__global__ void cast_dense_layer(const float* __restrict__ W, const float* __restrict__ b, int out, int in,
                                 int in_full, int has_time, uint16_t* Wp, uint16_t* WTp, float* bias_f,
                                 float* wt_f, int Npad, int Kpad) {
  int k = blockIdx.x * blockDim.x + threadIdx.x;
  int n = blockIdx.y;
  if (k >= Kpad) return;
  uint16_t q = 0;
  if (n < out && k < in) q = Low<T>::from_f32(W[(size_t)n * in_full + k]);
  Wp[(size_t)n * Kpad + k] = q;
  WTp[(size_t)k * Npad + n] = q;
  if (k == 0) {
    bias_f[n] = (n < out) ? Low<T>::to_f32(Low<T>::from_f32(b[n])) : 0.f;
    wt_f[n] = (n < out && has_time) ? Low<T>::to_f32(Low<T>::from_f32(W[(size_t)n * in_full + in])) : 0.f;
  }
}

// theta (fp32) -> padded low-precision operands of one 3x3 convolution, channels-last taps:
//   Wp  [Cpad][9*Cpad] : Wp[co][tap*Cpad + ci]  = Q(W[co][ci][tap])          (forward)
//   WTp [Cpad][9*Cpad] : WTp[ci][tap*Cpad + co] = Q(W[co][ci][8 - tap])      (input cotangent:
//         the transposed convolution is a convolution with the flipped kernel)
//   wt_f [9][Cpad] time-channel weights per tap, bias_f[Cpad].
template <class T>
__global__ void cast_conv_layer(const float* __restrict__ W, const float* __restrict__ b, int C, int Cin,
                                int has_time, uint16_t* Wp, uint16_t* WTp, float* bias_f, float* wt_f, int Cpad) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;  // over Cpad * 9 * Cpad
  int total = Cpad * 9 * Cpad;
  if (idx >= total) return;
  int ci = idx % Cpad, tap = (idx / Cpad) % 9, co = idx / (9 * Cpad);
  uint16_t q = 0;
  if (co < C && ci < C) q = Low<T>::from_f32(W[((size_t)co * Cin + ci) * 9 + tap]);
  Wp[(size_t)co * 9 * Cpad + tap * Cpad + ci] = q;
  WTp[(size_t)ci * 9 * Cpad + (8 - tap) * Cpad + co] = q;
  if (ci == 0) {
    float w = 0.f;
    if (co < C && has_time) w = Low<T>::to_f32(Low<T>::from_f32(W[((size_t)co * Cin + C) * 9 + tap]));
    wt_f[tap * Cpad + co] = w;
    if (tap == 0) bias_f[co] = (co < C) ? Low<T>::to_f32(Low<T>::from_f32(b[co])) : 0.f;
  }
}

// fp32 NCHW <-> channels-last [B*H*W][C]: per sample a transposition [rows][cols] -> [cols][rows] through LDS tiles of
// 32 x 32 (both the reads and the writes are runs of 128 bytes).  grid (cols / 32, rows / 32, samples), 32 x 8 threads.
// fill_inf: write +inf instead once a cotangent chain has been rejected (ctl may be null otherwise).
__global__ __launch_bounds__(256) void transpose_samples(const float* __restrict__ src, float* __restrict__ dst, int rows,
                                                         int cols, int nsamples, const Ctl* ctl, int fill_inf) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x, ty = threadIdx.y;
  const bool inf = fill_inf && ctl->poison;
  for (int b = blockIdx.z; b < nsamples; b += gridDim.z) {
    const float* s = src + (size_t)b * rows * cols;
    float* d = dst + (size_t)b * rows * cols;
    const int c = blockIdx.x * 32 + tx;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int r = blockIdx.y * 32 + ty + 8 * k;
      tile[ty + 8 * k][tx] = (r < rows && c < cols) ? s[(size_t)r * cols + c] : 0.f;
    }
    __syncthreads();
    const int oc = blockIdx.y * 32 + tx;   // column of the output = row of the input
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int orow = blockIdx.x * 32 + ty + 8 * k;
      if (orow < cols && oc < rows) d[(size_t)orow * rows + oc] = inf ? __builtin_inff() : tile[tx][ty + 8 * k];
    }
    __syncthreads();
  }
}
inline dim3 transpose_grid(int rows, int cols, int64_t nsamples) {
  return dim3((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32), (unsigned)std::min<int64_t>(nsamples, 65535));
}

// y <- y0 (fp32), ckpt[0] <- Q(y0)     (paper Alg. 1: initialisation and first stored state)
template <class T>
// naive: the low-precision baseline that keeps the state itself in low precision (paper Table 5,
// "naive" rows): y <- Q(y0) as well
__global__ void init_state(const float* __restrict__ y0, float* __restrict__ y, uint16_t* __restrict__ ck0,
                           int64_t n, int copy_y, int naive) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = y0[i];
  const uint16_t q = Low<T>::from_f32(v);
  if (naive) v = Low<T>::to_f32(q);
  if (copy_y || naive) y[i] = v;
  ck0[i] = q;
}

// Stage input  z_j = Q( yhat + h * sum_{l<j} a_jl k_l ),  yhat = stored checkpoint.
// Output in the padded layout [R][ld]; pad columns are written as zero.
template <class T>
__global__ void stage_input(const uint16_t* __restrict__ ck, int d, const uint16_t* __restrict__ K,
                            int64_t stage_stride, int j, Coefs arow, float h, uint16_t* __restrict__ z,
                            int ld, int64_t R, const Ctl* ctl) {
  if (poisoned(ctl)) return;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= R * ld) return;
  int64_t r = i / ld;
  int c = (int)(i % ld);
  uint16_t q = 0;
  if (c < d) {
    q = ck[r * d + c];
    if (j > 0) {
      float incr = 0.f;
      for (int l = 0; l < j; ++l)
        if (arow.v[l] != 0.f) incr = fmaf(arow.v[l], Low<T>::to_f32(K[l * stage_stride + i]), incr);
      q = Low<T>::from_f32(fmaf(h, incr, Low<T>::to_f32(q)));
    }
  }
  z[i] = q;
}

// y <- y + h * sum_j b_j k_j  in fp32;  ckpt[i+1] <- Q(y)     (paper Alg. 1, accumulate + store)
template <class T>
__global__ void combine_store(float* __restrict__ y, const uint16_t* __restrict__ K, int64_t stage_stride, int s,
                              Coefs b, float h, int round_incr, uint16_t* __restrict__ ck_next, int d, int ld,
                              int64_t R) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= R * d) return;
  int64_t r = i / d;
  int c = (int)(i % d);
  float incr = 0.f;
  for (int j = 0; j < s; ++j) incr = fmaf(b.v[j], Low<T>::to_f32(K[j * stage_stride + r * ld + c]), incr);
  if (round_incr & 1) incr = Low<T>::to_f32(Low<T>::from_f32(incr));
  float v = fmaf(h, incr, y[i]);
  const uint16_t q = Low<T>::from_f32(v);
  if (round_incr & 2) v = Low<T>::to_f32(q);  // naive baseline: the state is kept in low precision
  y[i] = v;
  ck_next[i] = q;
}

// ------------------------------------------------------------------------- backward
// also marks every step "not accepted yet" (scale 0): a step's parameter-gradient kernel runs
// only once the step's scale has been recorded
__global__ void ctl_reset(Ctl* ctl, float* scale_hist, int N) {
  for (int i = 0; i < N; ++i) scale_hist[i] = 0.f;
  ctl->S = 1.f; ctl->attempt = 1; ctl->poison = 0; ctl->failed_step = -1; ctl->nonfinite = 0;
  ctl->amax_bits = 0; ctl->retries = 0; ctl->s_min = 1.f; ctl->s_max = 1.f; ctl->done = 0; ctl->S_step = 1.f;
}

// a <- dL/dy_N (+ running-cost cotangent), max|a|   (paper Alg. 2, initialisation)
// naive_low: 0, or the low precision (1 fp16, 2 bf16) in which the naive baseline keeps the adjoint
__global__ void init_adjoint(const float* __restrict__ gyN, const float* __restrict__ gys_last,
                             float* __restrict__ a, int64_t n, Ctl* ctl, int copy, int naive_low) {
  unsigned bits = 0;  // (grid-stride: one atomic per workgroup, and few workgroups)
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    float v = gyN[i];
    if (gys_last) v += gys_last[i];
    if (naive_low == 1) v = Low<F16>::to_f32(Low<F16>::from_f32(v));
    if (naive_low == 2) v = Low<BF16>::to_f32(Low<BF16>::from_f32(v));
    if (copy || gys_last || naive_low) a[i] = v;
    const unsigned bb = __builtin_bit_cast(unsigned, fabsf(v));
    bits = bb > bits ? bb : bits;
  }
  block_amax(bits, &ctl->amax_bits);
}

// S_N = 2^floor(-log2(u_L * max|a|)) from the exponent of max|a|; exact in integers.
// A non-finite dL/dy_N is a range event only for the variants that check for them (detect: dynamic
// scaling reports a failure at step N, unscaled-safe returns infinite gradients); the plain unscaled
// variant has no checks (paper Sec. 5) and lets the NaN / inf run through the ordinary arithmetic.
__global__ void scale_init(Ctl* ctl, float* scale_hist, int N, int p_bits, int dynamic, int detect) {
  unsigned bits = ctl->amax_bits;
  float S = 1.f;
  if (bits >= 0x7F800000u) {  // non-finite dL/dy_N
    if (detect) {
      ctl->poison = 1;
      ctl->failed_step = N;
    }
  } else if (dynamic && bits != 0) {
    int e;
    float m = frexpf(__builtin_bit_cast(float, bits), &e);  // amax = m * 2^e, m in [0.5, 1)
    int E = p_bits - e + (m == 0.5f ? 1 : 0);
    E = E > 126 ? 126 : (E < -126 ? -126 : E);
    S = ldexpf(1.f, E);
  }
  ctl->S = S;
  ctl->s_min = S;
  ctl->s_max = S;
  ctl->amax_bits = 0;
  scale_hist[N] = S;
}

// kbar_j = Q( b_j * Q(S a) + h * sum_{l>j} a_lj zbar_l )   (paper eq. (vjp): the cotangent
// Q16(S a) pushed through the stage recursion of Phi).  Padded output layout.
template <class T>
__global__ void stage_cotangent(const float* __restrict__ a, int d, const uint16_t* __restrict__ zbar,
                                int64_t stage_stride, int j, int s, float bj, Coefs acol, float h,
                                uint16_t* __restrict__ kbar, int ld, int64_t R, Ctl* ctl, int detect) {
  if (ctl->poison) return;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool bad = false;
  if (i < R * ld) {
    int64_t r = i / ld;
    int c = (int)(i % ld);
    uint16_t q = 0;
    if (c < d) {
      uint16_t lam = Low<T>::from_f32(ctl->S * a[r * d + c]);
      float v = bj * Low<T>::to_f32(lam);
      float acc = 0.f;
      for (int l = j + 1; l < s; ++l)
        if (acol.v[l] != 0.f) acc = fmaf(acol.v[l], Low<T>::to_f32(zbar[l * stage_stride + i]), acc);
      v = fmaf(h, acc, v);
      q = Low<T>::from_f32(v);
      bad = Low<T>::nonfinite(lam) || Low<T>::nonfinite(q);
    }
    kbar[i] = q;
  }
  if (detect) raise_if_any(bad, ctl);
}

// after the cotangent chain of a step: accept or poison   (paper Alg. 2, finiteness test)
__global__ void chain_decide(Ctl* ctl, int step, int detect) {
  if (ctl->poison) return;
  if (detect && ctl->nonfinite) {
    ctl->poison = 1;
    ctl->failed_step = step;
  } else {
    ctl->S_step = ctl->S;
  }
}

// host-requested retry of the poisoned step with half the scale   (paper Alg. 2, halve and retry)
__global__ void chain_retry(Ctl* ctl) {
  ctl->S *= 0.5f;
  ctl->attempt += 1;
  ctl->retries += 1;
  ctl->poison = 0;
  ctl->nonfinite = 0;
  ctl->failed_step = -1;
}

// dL/dt[m] += tpart[m][0] + tpart[m - 1][1]   (paper Sec. 3: the two update lines of t'; the per-step
// sums were collected while the steps ran and are folded in once every step is accepted)
__global__ void fold_time_sums(float* __restrict__ grad_t, const float* __restrict__ tpart, int N, const Ctl* ctl) {
  if (ctl->poison) return;
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m > N) return;
  float v = 0.f;
  if (m < N) v += tpart[2 * m];
  if (m > 0) v += tpart[2 * (m - 1) + 1];
  grad_t[m] += v;
}

// a <- a + (h/S) * sum_j zbar_j (+ running-cost cotangent), fp32; new max|a|
template <class T>
__global__ void adjoint_update(float* __restrict__ a, int d, const uint16_t* __restrict__ zbar,
                               int64_t stage_stride, int s, float h, const float* __restrict__ gys_i, int ld,
                               int64_t R, Ctl* ctl, int naive) {
  if (ctl->poison) return;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  unsigned bits = 0;
  if (i < R * d) {
    int64_t r = i / d;
    int c = (int)(i % d);
    float da = 0.f;
    for (int j = 0; j < s; ++j) da += Low<T>::to_f32(zbar[j * stage_stride + r * ld + c]);
    float v = fmaf(h / ctl->S, da, a[i]);
    if (gys_i) v += gys_i[i];
    if (naive) v = Low<T>::to_f32(Low<T>::from_f32(v));  // naive baseline: adjoint kept in low precision
    a[i] = v;
    bits = __builtin_bit_cast(unsigned, fabsf(v));
  }
  block_amax(bits, &ctl->amax_bits);
}

// end of a step: record S_i, decide growth   (paper Alg. 2, doubling rule)
// (slots: per-workgroup maxima of |a| written by adjoint_update_v8 instead of one atomic per workgroup on
// a single address -- a thousand of those cost as much as a third of that kernel's streaming time;
// folded here by the workgroup's threads, launched with 256 threads)
__global__ void scale_grow(Ctl* ctl, float* scale_hist, int step, int p_bits, int dynamic, int raw_norm,
                           const unsigned* __restrict__ slots, int nslots) {
  if (ctl->poison) return;
  unsigned bits = 0;
  for (int i = threadIdx.x; i < nslots; i += blockDim.x) bits = slots[i] > bits ? slots[i] : bits;
  block_amax(bits, &ctl->amax_bits);
  __syncthreads();
  if (threadIdx.x != 0) return;
  __threadfence();
  float S = ctl->S;
  scale_hist[step] = S;
  ctl->s_min = fminf(ctl->s_min, S);
  ctl->s_max = fmaxf(ctl->s_max, S);
  if (dynamic && ctl->attempt == 1) {
    float amax = __builtin_bit_cast(float, atomicMax(&ctl->amax_bits, 0u));
    float test = raw_norm ? amax : S * amax;
    if (test <= ldexpf(1.f, p_bits - 1) && S < ldexpf(1.f, 126)) ctl->S = 2.f * S;
  }
  ctl->attempt = 1;
  ctl->amax_bits = 0;
  ctl->nonfinite = 0;
}

// Column sums of the cotangents for bias and time-weight gradients:
//   db[c]  += (h/S) * sum_rows delta[row][c]
//   dwt[c] += (h/S) * sum_j tau_j sum_{rows of stage j} delta[row][c]          (dense layer 1)
//   conv: dwt[c][tap] += (h/S) * sum_j tau_j sum_{pixels whose tap neighbour exists} delta
// rows = stages * R; `taus` gives tau_j.  Grid: (column blocks of 64, row chunks).
// With `tpart` (time-grid gradient, paper Sec. 3): the time cotangent of stage j is
// taubar_j = sum_{rows of stage j, c (, taps)} delta * w_t (wt: the rounded time weights, dense
// [ncols], conv [9][ld]); the step's sums get   tpart[0] += (h/S) sum_j (1 - c_j) taubar_j
// (the time part of dt - dh) and tpart[1] += (h/S) sum_j c_j taubar_j (the time part of dh).
template <class T, bool CONV>
__global__ __launch_bounds__(256) void column_sums(const uint16_t* __restrict__ delta, int ld, int64_t R, int s,
                                                   int ncols, Coefs taus, float h, float* __restrict__ gb,
                                                   float* __restrict__ gwt, int wt_stride, int H, int Wd,
                                                   int rows_per_block, const Ctl* ctl, const float* __restrict__ wt,
                                                   Coefs cs, float* __restrict__ tpart) {
  if (ctl->poison) return;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + tx;
  const int64_t rows = (int64_t)s * R;
  int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  int64_t r1 = r0 + rows_per_block;
  if (r1 > rows) r1 = rows;
  constexpr int NT = CONV ? 9 : 1;
  float sb = 0.f, st[NT], sc[NT], s1[NT];  // st: tau-weighted, sc: c_j-weighted, s1: unweighted
#pragma unroll
  for (int t = 0; t < NT; ++t) st[t] = sc[t] = s1[t] = 0.f;
  for (int64_t r = r0 + ty; r < r1; r += 4) {
    float v = Low<T>::to_f32(delta[r * ld + c]);
    const int j = (int)(r / R);
    float tau = taus.v[j], cj = cs.v[j];
    sb += v;
    if (CONV) {
      int x = (int)(r % Wd), y = (int)((r / Wd) % H);
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
        if (yy >= 0 && yy < H && xx >= 0 && xx < Wd) {
          st[t] = fmaf(tau, v, st[t]);
          sc[t] = fmaf(cj, v, sc[t]);
          s1[t] += v;
        }
      }
    } else {
      st[0] = fmaf(tau, v, st[0]);
      sc[0] = fmaf(cj, v, sc[0]);
      s1[0] += v;
    }
  }
  __shared__ float red[4][64][3 * NT + 1];
  red[ty][tx][0] = sb;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    red[ty][tx][1 + t] = st[t];
    red[ty][tx][1 + NT + t] = sc[t];
    red[ty][tx][1 + 2 * NT + t] = s1[t];
  }
  __syncthreads();
  if (ty == 0) {
    const float scale = h / ctl->S_step;
    float p0 = 0.f, p1 = 0.f;
    if (c < ncols) {
      float v = red[0][tx][0] + red[1][tx][0] + red[2][tx][0] + red[3][tx][0];
      unsafeAtomicAdd(&gb[c], scale * v);
      if (gwt) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float w = red[0][tx][1 + t] + red[1][tx][1 + t] + red[2][tx][1 + t] + red[3][tx][1 + t];
          unsafeAtomicAdd(&gwt[(size_t)c * wt_stride + t], scale * w);
        }
      }
      if (tpart && wt) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const float wc = red[0][tx][1 + NT + t] + red[1][tx][1 + NT + t] + red[2][tx][1 + NT + t] +
                           red[3][tx][1 + NT + t];
          const float w1 = red[0][tx][1 + 2 * NT + t] + red[1][tx][1 + 2 * NT + t] + red[2][tx][1 + 2 * NT + t] +
                           red[3][tx][1 + 2 * NT + t];
          const float wv = CONV ? wt[t * ld + c] : wt[c];
          p0 = fmaf(wv, w1 - wc, p0);
          p1 = fmaf(wv, wc, p1);
        }
      }
    }
    if (tpart && wt) {  // (wavefront 0: sum over its 64 columns)
      for (int o = 32; o > 0; o >>= 1) {
        p0 += __shfl_xor(p0, o);
        p1 += __shfl_xor(p1, o);
      }
      if (tx == 0) {  // (this workgroup's slot of the launch's table: see fold_time_slots)
        float* slot = tpart + 2 * ((size_t)blockIdx.y * gridDim.x + blockIdx.x);
        slot[0] = scale * p0;
        slot[1] = scale * p1;
      }
    }
  }
}

// State-shaped terms of the time-grid gradient of one accepted step (paper Sec. 3, update lines of t'):
//   phia = sum_i (sum_j b_j k_j[i]) a[i]                      (Phi^T a_{i+1}, a before this step's update)
//   dhz  = sum_i sum_j zbar_j[i] * (sum_{l<j} a_jl k_l[i])    (the stage-input part of dh)
//   tpart[0] += -(h/S) dhz - phia,   tpart[1] += (h/S) dhz + phia.
struct CoefMat {
  float v[kMaxStages * kMaxStages];
};
template <class T>
__global__ __launch_bounds__(256) void time_grid_terms(const float* __restrict__ a, int d,
                                                       const uint16_t* __restrict__ K,
                                                       const uint16_t* __restrict__ zbar, int64_t stage_stride, int s,
                                                       Coefs bw, CoefMat A, float h, int ld, int64_t R, const Ctl* ctl,
                                                       float* __restrict__ tpart) {
  if (ctl->poison) return;
  float pa = 0.f, dz = 0.f;
  const int64_t n = R * d;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t off = (i / d) * ld + (i % d);
    float k[kMaxStages];
    float phi = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxStages; ++j) {
      k[j] = (j < s) ? Low<T>::to_f32(K[j * stage_stride + off]) : 0.f;
      phi = fmaf(bw.v[j], k[j], phi);
    }
    pa = fmaf(phi, a[i], pa);
#pragma unroll
    for (int j = 1; j < kMaxStages; ++j) {
      if (j < s) {
        float incr = 0.f;
#pragma unroll
        for (int l = 0; l < j; ++l) incr = fmaf(A.v[j * kMaxStages + l], k[l], incr);
        dz = fmaf(Low<T>::to_f32(zbar[j * stage_stride + off]), incr, dz);
      }
    }
  }
  const float hs = h / ctl->S_step;
  block_sum2(-hs * dz - pa, fmaf(hs, dz, pa), tpart + 2 * (size_t)blockIdx.x);
}

// Per-workgroup slots of the time-grid sums -> the per-step sums, in a fixed order: workgroup b of this kernel takes the
// slots [b * per_step, (b + 1) * per_step) (pairs) and adds their sum to dst[2 (step0 - b)], dst[2 (step0 - b) + 1];
// thread t sums the slots t, t + 256, ... and the 256 partial sums are added up in order.  The slots are cleared for
// the next launch (the kernels that fill them write only the slots of the workgroups that have something to add).
__global__ __launch_bounds__(256) void fold_time_slots(float* __restrict__ slots, int per_step, float* __restrict__ dst, int step0,
                                                       const Ctl* ctl) {
  if (ctl->poison) return;
  __shared__ float part[256][2];
  float* base = slots + 2 * (size_t)blockIdx.x * per_step;
  float s0 = 0.f, s1 = 0.f;
  for (int i = threadIdx.x; i < per_step; i += 256) {
    s0 += base[2 * i];
    s1 += base[2 * i + 1];
    base[2 * i] = 0.f;
    base[2 * i + 1] = 0.f;
  }
  part[threadIdx.x][0] = s0;
  part[threadIdx.x][1] = s1;
  __syncthreads();
  if (threadIdx.x == 0) {
    float a = 0.f, b = 0.f;
    for (int i = 0; i < 256; ++i) {
      a += part[i][0];
      b += part[i][1];
    }
    float* d = dst + 2 * (size_t)(step0 - (int)blockIdx.x);
    d[0] += a;
    d[1] += b;
  }
}

// NONE_SAFE outcome: overflow => gradients are +inf
__global__ void fill_inf_if_poisoned(float* p, int64_t n, const Ctl* ctl) {
  if (!ctl->poison) return;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = __builtin_inff();
}


// ----------------------------------------------------------------------------------------
// 8-wide versions of the streaming kernels above, for state widths that are multiples of 8:
// 16-byte accesses to the 16-bit arrays, 2 x 16-byte to the fp32 ones, one index division per
// 8 elements, grid-stride loops.  Same arithmetic, element for element.
template <class T>
__device__ inline void unpack8(const u16x8& v, float (&f)[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = Low<T>::to_f32(v[e]);
}
template <class T>
__device__ inline u16x8 pack8(const float (&f)[8]) {
  u16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = Low<T>::from_f32(f[e]);
  return v;
}
__device__ inline void load8f(const float* p, float (&f)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}
__device__ inline void store8f(float* p, const float (&f)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
}

template <class T>
__global__ __launch_bounds__(256) void stage_input_v8(const uint16_t* __restrict__ ck, int d,
                                                      const uint16_t* __restrict__ K, int64_t stage_stride, int j,
                                                      Coefs arow, float h, uint16_t* __restrict__ z, int ld, int64_t R,
                                                      const Ctl* ctl) {
  if (poisoned(ctl)) return;
  const int gpr = ld >> 3;  // groups of 8 per padded row
  const int64_t G = R * gpr;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < G; g += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = g / gpr;
    const int c = (int)(g - r * gpr) << 3;
    u16x8 q = {0, 0, 0, 0, 0, 0, 0, 0};
    if (c < d) {
      q = *reinterpret_cast<const u16x8*>(ck + r * d + c);
      if (j > 0) {
        float incr[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, base[8], kl[8];
        for (int l = 0; l < j; ++l) {
          if (arow.v[l] != 0.f) {
            unpack8<T>(*reinterpret_cast<const u16x8*>(K + l * stage_stride + r * ld + c), kl);
#pragma unroll
            for (int e = 0; e < 8; ++e) incr[e] = fmaf(arow.v[l], kl[e], incr[e]);
          }
        }
        unpack8<T>(q, base);
#pragma unroll
        for (int e = 0; e < 8; ++e) base[e] = fmaf(h, incr[e], base[e]);
        q = pack8<T>(base);
      }
    }
    *reinterpret_cast<u16x8*>(z + r * ld + c) = q;
  }
}

template <class T>
__global__ __launch_bounds__(256) void combine_store_v8(float* __restrict__ y, const uint16_t* __restrict__ K,
                                                        int64_t stage_stride, int s, Coefs b, float h, int round_incr,
                                                        uint16_t* __restrict__ ck_next, int d, int ld, int64_t R) {
  const int gpr = d >> 3;
  const int64_t G = R * gpr;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < G; g += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = g / gpr;
    const int c = (int)(g - r * gpr) << 3;
    float incr[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, kj[8], yv[8];
    for (int j = 0; j < s; ++j) {
      unpack8<T>(*reinterpret_cast<const u16x8*>(K + j * stage_stride + r * ld + c), kj);
#pragma unroll
      for (int e = 0; e < 8; ++e) incr[e] = fmaf(b.v[j], kj[e], incr[e]);
    }
    load8f(y + r * d + c, yv);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (round_incr & 1) incr[e] = Low<T>::to_f32(Low<T>::from_f32(incr[e]));
      yv[e] = fmaf(h, incr[e], yv[e]);
    }
    const u16x8 q = pack8<T>(yv);
    if (round_incr & 2) unpack8<T>(q, yv);  // naive baseline: the state is kept in low precision
    store8f(y + r * d + c, yv);
    *reinterpret_cast<u16x8*>(ck_next + r * d + c) = q;
  }
}

template <class T>
__global__ __launch_bounds__(256) void stage_cotangent_v8(const float* __restrict__ a, int d,
                                                          const uint16_t* __restrict__ zbar, int64_t stage_stride,
                                                          int j, int s, float bj, Coefs acol, float h,
                                                          uint16_t* __restrict__ kbar, int ld, int64_t R, Ctl* ctl,
                                                          int detect) {
  if (ctl->poison) return;
  const int gpr = ld >> 3;
  const int64_t G = R * gpr;
  const float S = ctl->S;
  bool bad = false;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < G; g += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = g / gpr;
    const int c = (int)(g - r * gpr) << 3;
    u16x8 q = {0, 0, 0, 0, 0, 0, 0, 0};
    if (c < d) {
      float av[8], acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, zl[8], v[8];
      load8f(a + r * d + c, av);
      for (int l = j + 1; l < s; ++l) {
        if (acol.v[l] != 0.f) {
          unpack8<T>(*reinterpret_cast<const u16x8*>(zbar + l * stage_stride + r * ld + c), zl);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = fmaf(acol.v[l], zl[e], acc[e]);
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint16_t lam = Low<T>::from_f32(S * av[e]);
        v[e] = fmaf(h, acc[e], bj * Low<T>::to_f32(lam));
        bad = bad || Low<T>::nonfinite(lam);
      }
      q = pack8<T>(v);
#pragma unroll
      for (int e = 0; e < 8; ++e) bad = bad || Low<T>::nonfinite(q[e]);
    }
    *reinterpret_cast<u16x8*>(kbar + r * ld + c) = q;
  }
  if (detect) raise_if_any(bad, ctl);
}

template <class T>
__global__ __launch_bounds__(256) void adjoint_update_v8(float* __restrict__ a, int d,
                                                         const uint16_t* __restrict__ zbar, int64_t stage_stride, int s,
                                                         float h, const float* __restrict__ gys_i, int ld, int64_t R,
                                                         Ctl* ctl, int naive, unsigned* __restrict__ slots) {
  const int gpr = d >> 3;
  const int64_t G = R * gpr;
  unsigned bits = 0;
  // The streaming loads of a thread's first group are requested BEFORE the control block is looked at:
  // the rejected-chain flag and the scale are one more memory round trip, which would otherwise sit in
  // front of every load of a kernel that runs for a few tens of microseconds.  Nothing is stored before
  // the flag is known.
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  u16x8 zq[kMaxStages];
  float av[8];
  auto request = [&](int64_t gi) {
    const int64_t r = gi / gpr;
    const int c = (int)(gi - r * gpr) << 3;
#pragma unroll
    for (int j = 0; j < kMaxStages; ++j)
      if (j < s) zq[j] = *reinterpret_cast<const u16x8*>(zbar + j * stage_stride + r * ld + c);
    load8f(a + r * d + c, av);
  };
  if (g < G) request(g);
  const int poison = ctl->poison;
  const float hs = h / ctl->S;
  if (poison) return;
  for (; g < G;) {
    const int64_t r = g / gpr;
    const int c = (int)(g - r * gpr) << 3;
    float da[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, zj[8];
#pragma unroll
    for (int j = 0; j < kMaxStages; ++j)
      if (j < s) {
        unpack8<T>(zq[j], zj);
#pragma unroll
        for (int e = 0; e < 8; ++e) da[e] += zj[e];
      }
    float out[8];
    if (gys_i) {
      float gy[8];
      load8f(gys_i + r * d + c, gy);
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = fmaf(hs, da[e], av[e]) + gy[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = fmaf(hs, da[e], av[e]);
    }
    if (naive) unpack8<T>(pack8<T>(out), out);
    const int64_t gn = g + (int64_t)gridDim.x * blockDim.x;
    if (gn < G) request(gn);  // (a different group: no overlap with the store below)
    store8f(a + r * d + c, out);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const unsigned bb = __builtin_bit_cast(unsigned, fabsf(out[e]));
      bits = bb > bits ? bb : bits;
    }
    g = gn;
  }
  // the workgroup's maximum goes to its own slot (folded by scale_grow)
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned other = __shfl_xor(bits, o);
    bits = bits > other ? bits : other;
  }
  __shared__ unsigned wmax[4];
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = bits;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned m = wmax[0];
    for (int i = 1; i < 4; ++i) m = wmax[i] > m ? wmax[i] : m;
    slots[blockIdx.x] = m;
  }
}

}  // namespace rampde
