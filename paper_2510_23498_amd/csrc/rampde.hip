// C-ABI entry points of the gfx950 mixed-precision neural-ODE time stepper: argument
// validation, workspace planning and the launch sequences of the forward pass (paper
// Algorithm 1) and of the discrete adjoint with dynamic adjoint scaling (paper Algorithm 2).
// Every step of the method runs in the kernels of gemm.hpp / elementwise.hpp; the host only
// orders launches and, under dynamic scaling, re-enqueues from a step whose cotangent chain
// overflowed (halve-and-retry of Algorithm 2).
#include "../../include/rampde.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "common.hpp"
#include "elementwise.hpp"
#include "gemm.hpp"

namespace rampde {

static inline int pad64(int x) { return (x + kPad - 1) / kPad * kPad; }
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// host-side rounding of a scalar to the low-precision format (stage times, paper Alg. 1:
// the velocity sees its time argument in low precision)
static float round_low_host(float x, rampde_dtype low) {
  if (low == RAMPDE_F16) return (float)(_Float16)x;
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return x;
  u += 0x7FFFu + ((u >> 16) & 1u);
  u &= 0xFFFF0000u;
  float r;
  memcpy(&r, &u, 4);
  return r;
}

struct Layer {
  int out, in, in_full;  // in: state/activation inputs; in_full: + time column (dense layer 1)
  int Npad, Kpad;        // padded out / in
  int has_time;
  size_t theta_w, theta_b;  // offsets (elements) into theta
  // workspace offsets (bytes)
  size_t Wp, WTp, bias_f, wt_f;
  int ldw;  // K extent of the forward GEMM (dense: Kpad; conv: 9 * Cpad)
};

struct Plan {
  bool ok = false;
  bool conv = false;
  int L = 0;
  int s = 0;
  int64_t R = 0;     // rows: B (dense) or B*H*W (conv)
  int d = 0;         // features per row at the boundary (dense: d; conv: C)
  int dpad = 0;
  int64_t n = 0;     // state elements R * d
  int H = 0, Wd = 0;
  int64_t P = 0;
  std::vector<Layer> layers;
  // workspace offsets (bytes)
  size_t ctl = 0, scale_hist = 0, y_rows = 0, a_rows = 0, gys_rows = 0;
  size_t Z = 0, K = 0, KBAR = 0, ZBAR = 0;
  std::vector<size_t> ACT, DELTA;  // per hidden layer l = 0..L-2: output of layer l / its cotangent
  size_t total = 0;
  int64_t stage_stride = 0;  // elements between stages in Z/K/KBAR/ZBAR: R * dpad
};

static bool build_layers(const rampde_velocity* vel, Plan& p) {
  if (!vel) return false;
  size_t off = 0;
  if (vel->kind == RAMPDE_VEL_MLP) {
    if (vel->n_layers < 1 || vel->n_layers > 16 || !vel->widths) return false;
    p.L = vel->n_layers;
    for (int l = 0; l <= p.L; ++l)
      if (vel->widths[l] < 1 || vel->widths[l] > 16384) return false;
    if (vel->widths[0] != vel->widths[p.L]) return false;
    p.conv = false;
    p.d = vel->widths[0];
    for (int l = 0; l < p.L; ++l) {
      Layer y{};
      y.out = vel->widths[l + 1];
      y.in = vel->widths[l];
      y.has_time = (l == 0 && vel->time_input) ? 1 : 0;
      y.in_full = y.in + y.has_time;
      y.Npad = pad64(y.out);
      y.Kpad = pad64(y.in);
      y.ldw = y.Kpad;
      y.theta_w = off;
      off += (size_t)y.out * y.in_full;
      y.theta_b = off;
      off += y.out;
      p.layers.push_back(y);
    }
  } else if (vel->kind == RAMPDE_VEL_CONV2) {
    if (vel->C < 1 || vel->C > 4096 || vel->H < 1 || vel->W < 1 || vel->H > 4096 || vel->W > 4096) return false;
    p.conv = true;
    p.L = 2;
    p.d = vel->C;
    p.H = vel->H;
    p.Wd = vel->W;
    for (int l = 0; l < 2; ++l) {
      Layer y{};
      y.out = vel->C;
      y.in = vel->C;
      y.has_time = vel->time_input ? 1 : 0;
      y.in_full = y.in + y.has_time;
      y.Npad = pad64(y.out);
      y.Kpad = pad64(y.in);
      y.ldw = 9 * y.Kpad;
      y.theta_w = off;
      off += (size_t)y.out * y.in_full * 9;
      y.theta_b = off;
      off += y.out;
      p.layers.push_back(y);
    }
  } else {
    return false;
  }
  p.P = (int64_t)off;
  p.dpad = pad64(p.d);
  return true;
}

static Plan make_plan(const rampde_velocity* vel, int64_t B, int N, const rampde_tableau* tab, int is_backward) {
  Plan p;
  if (!build_layers(vel, p)) return p;
  if (B < 1 || N < 1 || !tab || tab->s < 1 || tab->s > kMaxStages) return p;
  p.s = tab->s;
  p.R = p.conv ? B * (int64_t)p.H * p.Wd : B;
  if (p.R > (int64_t)1 << 30) return p;
  p.n = p.R * p.d;
  p.stage_stride = p.R * p.dpad;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += align256(bytes);
    return o;
  };
  p.ctl = take(sizeof(Ctl));
  p.scale_hist = take(sizeof(float) * (size_t)(N + 1));
  for (auto& y : p.layers) {
    size_t wel = (size_t)y.Npad * (p.conv ? 9 * y.Kpad : y.Kpad);
    y.Wp = take(wel * 2);
    y.WTp = take(wel * 2);
    y.bias_f = take(sizeof(float) * y.Npad);
    y.wt_f = take(sizeof(float) * y.Npad * (p.conv ? 9 : 1));
  }
  const int sbuf = is_backward ? p.s : 1;  // forward keeps one stage of inputs/activations
  if (p.conv) {
    p.y_rows = take(sizeof(float) * (size_t)p.n);
    if (is_backward) {
      p.a_rows = p.y_rows;
      p.gys_rows = take(sizeof(float) * (size_t)p.n);
    }
  }
  p.Z = take((size_t)sbuf * p.R * p.dpad * 2);
  p.K = take((size_t)p.s * p.R * p.dpad * 2);
  for (int l = 0; l + 1 < p.L; ++l) p.ACT.push_back(take((size_t)sbuf * p.R * p.layers[l].Npad * 2));
  if (is_backward) {
    p.KBAR = take((size_t)p.s * p.R * p.dpad * 2);
    p.ZBAR = take((size_t)p.s * p.R * p.dpad * 2);
    for (int l = 0; l + 1 < p.L; ++l) p.DELTA.push_back(take((size_t)p.s * p.R * p.layers[l].Npad * 2));
  }
  p.total = off;
  p.ok = true;
  return p;
}

static int check_common(const rampde_velocity* vel, const double* tgrid, int N, const rampde_tableau* tab,
                        const rampde_policy* pol) {
  if (!vel || !tgrid || !tab || !pol || N < 1) return RAMPDE_EINVAL;
  if (tab->s < 1 || !tab->A || !tab->b || !tab->c) return RAMPDE_EINVAL;
  if (tab->s > kMaxStages) return RAMPDE_EUNSUPPORTED;
  for (int i = 0; i < tab->s; ++i)
    for (int j = i; j < tab->s; ++j)
      if (tab->A[i * tab->s + j] != 0.0) return RAMPDE_EINVAL;
  for (int i = 0; i <= N; ++i)
    if (!std::isfinite(tgrid[i])) return RAMPDE_EINVAL;
  for (int i = 0; i < N; ++i)
    if (!(tgrid[i + 1] > tgrid[i])) return RAMPDE_EINVAL;
  if (pol->low != RAMPDE_F16 && pol->low != RAMPDE_BF16) return pol->low == RAMPDE_F32 ? RAMPDE_EUNSUPPORTED : RAMPDE_EINVAL;
  if ((int)pol->scaling < 0 || (int)pol->scaling > 3) return RAMPDE_EINVAL;
  return RAMPDE_OK;
}

static thread_local char g_hip_msg[256] = "no HIP error recorded";
static int hip_fail(hipError_t e, const char* where) {
  snprintf(g_hip_msg, sizeof g_hip_msg, "HIP error in %s: %s", where, hipGetErrorString(e));
  return RAMPDE_EHIP;
}
#define HIP_TRY(expr)                                  \
  do {                                                 \
    hipError_t e_ = (expr);                            \
    if (e_ != hipSuccess) return hip_fail(e_, #expr);  \
  } while (0)

static inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// ---------------------------------------------------------------- optional per-kernel timing
// When enabled, launches of the kernel classes below are bracketed by HIP events on the
// caller's stream; rampde_timing_read sums the elapsed times.  Process-global, not thread safe:
// a measurement aid for the benchmark, off by default.
struct TimedLaunch {
  hipEvent_t e0, e1;
  int cls;
  double work;
};
static bool g_timing = false;
static std::vector<TimedLaunch> g_timed;

struct TimeScope {
  bool on;
  hipStream_t st;
  TimedLaunch t;
  TimeScope(int cls, double work, hipStream_t stream) : on(g_timing), st(stream) {
    if (!on) return;
    t.cls = cls;
    t.work = work;
    if (hipEventCreate(&t.e0) != hipSuccess || hipEventCreate(&t.e1) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(t.e0, st);
  }
  ~TimeScope() {
    if (!on) return;
    (void)hipEventRecord(t.e1, st);
    g_timed.push_back(t);
  }
};

// ---------------------------------------------------------------- typed launch sequences
template <class T>
struct Runner {
  const Plan& p;
  char* ws;
  hipStream_t st;
  Ctl* ctl;
  Runner(const Plan& plan, void* workspace, hipStream_t stream)
      : p(plan), ws((char*)workspace), st(stream), ctl((Ctl*)((char*)workspace + plan.ctl)) {}

  uint16_t* u16(size_t off) const { return (uint16_t*)(ws + off); }
  float* f32(size_t off) const { return (float*)(ws + off); }

  void cast_weights(const float* theta) {
    for (const Layer& y : p.layers) {
      if (p.conv) {
        int total = y.Npad * 9 * y.Kpad;
        cast_conv_layer<T><<<blocks_for(total, 256), 256, 0, st>>>(theta + y.theta_w, theta + y.theta_b, y.out, y.in_full,
                                                                   y.has_time, u16(y.Wp), u16(y.WTp), f32(y.bias_f),
                                                                   f32(y.wt_f), y.Kpad);
      } else {
        dim3 grid(blocks_for(y.Kpad, 64), y.Npad);
        cast_dense_layer<T><<<grid, 64, 0, st>>>(theta + y.theta_w, theta + y.theta_b, y.out, y.in, y.in_full, y.has_time,
                                                 u16(y.Wp), u16(y.WTp), f32(y.bias_f), f32(y.wt_f), y.Npad, y.Kpad);
      }
    }
  }

  void launch_nt(const GemmNT& g) {
    TimeScope ts(RAMPDE_K_VELOCITY_GEMM, 2.0 * g.M * (double)g.N * g.K, st);
    if (p.conv) {
      dim3 grid(blocks_for(g.M, 128), g.N / 64);
      gemm_nt<T, 2, 1, true><<<grid, 256, 0, st>>>(g);
    } else if (g.N % 128 == 0 && g.M >= 2048) {
      dim3 grid(blocks_for(g.M, 128), g.N / 128);
      gemm_nt<T, 2, 2, false><<<grid, 256, 0, st>>>(g);
    } else if (g.M >= 2048) {
      dim3 grid(blocks_for(g.M, 128), g.N / 64);
      gemm_nt<T, 2, 1, false><<<grid, 256, 0, st>>>(g);
    } else {
      dim3 grid(blocks_for(g.M, 64), g.N / 64);
      gemm_nt<T, 1, 1, false><<<grid, 256, 0, st>>>(g);
    }
  }

  // stage inputs, stage times and slopes of one step (the inside of Phi), from checkpoint ck.
  // keep != 0: every stage keeps its own input / activation buffers (backward recomputation).
  void stages(const uint16_t* ck, double t_i, float h, const rampde_tableau* tab, rampde_dtype low, int keep,
              float* taus_out, Ctl* c) {
    const int s = p.s;
    for (int j = 0; j < s; ++j) {
      const int jb = keep ? j : 0;
      uint16_t* z = u16(p.Z) + (size_t)jb * p.stage_stride;
      Coefs arow{};
      for (int l = 0; l < j; ++l) arow.v[l] = (float)tab->A[j * s + l];
      stage_input<T><<<blocks_for(p.R * p.dpad, 256), 256, 0, st>>>(ck, p.d, u16(p.K), p.stage_stride, j, arow, h, z,
                                                                   p.dpad, p.R, c);
      const float tau = round_low_host((float)(t_i + tab->c[j] * (double)h), low);
      if (taus_out) taus_out[j] = tau;
      const uint16_t* in = z;
      for (int l = 0; l < p.L; ++l) {
        const Layer& y = p.layers[l];
        GemmNT g{};
        g.A = in;
        g.lda = y.Kpad;
        g.W = u16(y.Wp);
        g.ldw = y.ldw;
        const bool last = (l == p.L - 1);
        uint16_t* out = last ? u16(p.K) + (size_t)j * p.stage_stride
                             : u16(p.ACT[l]) + (size_t)jb * p.R * y.Npad;
        g.C = out;
        g.ldc = y.Npad;
        g.M = (int)p.R;
        g.N = y.Npad;
        g.K = y.ldw;
        g.bias = f32(y.bias_f);
        g.wt = y.has_time ? f32(y.wt_f) : nullptr;
        g.tau = tau;
        g.act_tanh = last ? 0 : 1;
        g.dact = nullptr;
        g.ldd = 0;
        g.ctl = c;
        g.detect = 0;
        g.H = p.H;
        g.Wd = p.Wd;
        g.Cpad = y.Kpad;
        launch_nt(g);
        in = out;
      }
    }
  }

  int forward(const float* theta, const float* y0, const double* tgrid, int N, const rampde_tableau* tab,
              const rampde_policy* pol, uint16_t* ckpt, float* yN) {
    cast_weights(theta);
    float* y = yN;
    if (p.conv) {
      y = f32(p.y_rows);
      nchw_to_rows<<<blocks_for(p.n, 256), 256, 0, st>>>(y0, y, p.R, p.d, p.H * p.Wd);
      init_state<T><<<blocks_for(p.n, 256), 256, 0, st>>>(y, y, ckpt, p.n, 0);
    } else {
      init_state<T><<<blocks_for(p.n, 256), 256, 0, st>>>(y0, y, ckpt, p.n, 1);
    }
    Coefs bw{};
    for (int j = 0; j < p.s; ++j) bw.v[j] = (float)tab->b[j];
    for (int i = 0; i < N; ++i) {
      const float h = (float)(tgrid[i + 1] - tgrid[i]);
      const uint16_t* ck = ckpt + (size_t)i * p.n;
      stages(ck, tgrid[i], h, tab, pol->low, 0, nullptr, nullptr);
      // bytes per state element: read y (4) + s slopes (2 each) + write y (4) + write checkpoint (2)
      TimeScope ts(RAMPDE_K_COMBINE_STORE, (double)p.n * (10.0 + 2.0 * p.s), st);
      combine_store<T><<<blocks_for(p.n, 256), 256, 0, st>>>(y, u16(p.K), p.stage_stride, p.s, bw, h,
                                                            (pol->flags & RAMPDE_ROUND_INCREMENT) ? 1 : 0,
                                                            ckpt + (size_t)(i + 1) * p.n, p.d, p.dpad, p.R);
    }
    if (p.conv) rows_to_nchw<<<blocks_for(p.n, 256), 256, 0, st>>>(y, yN, p.R, p.d, p.H * p.Wd, nullptr, 0);
    HIP_TRY(hipGetLastError());
    return RAMPDE_OK;
  }

  // one step of the adjoint recursion: recompute, cotangent chain, decision, fp32 updates
  void backward_step(int i, const double* tgrid, const rampde_tableau* tab, const rampde_policy* pol,
                     const uint16_t* ckpt, float* a, const float* gys_i, float* grad_theta, int dynamic, int detect,
                     bool recompute) {
    const int s = p.s;
    const float h = (float)(tgrid[i + 1] - tgrid[i]);
    Coefs taus{};
    if (recompute) {
      stages(ckpt + (size_t)i * p.n, tgrid[i], h, tab, pol->low, 1, taus.v, ctl);
    } else {
      for (int j = 0; j < s; ++j) taus.v[j] = round_low_host((float)(tgrid[i] + tab->c[j] * (double)h), pol->low);
    }
    // cotangent chain, stages in reverse
    for (int j = s - 1; j >= 0; --j) {
      Coefs acol{};
      for (int l = j + 1; l < s; ++l) acol.v[l] = (float)tab->A[l * s + j];
      uint16_t* kbar = u16(p.KBAR) + (size_t)j * p.stage_stride;
      stage_cotangent<T><<<blocks_for(p.R * p.dpad, 256), 256, 0, st>>>(a, p.d, u16(p.ZBAR), p.stage_stride, j, s,
                                                                       (float)tab->b[j], acol, h, kbar, p.dpad, p.R,
                                                                       ctl, detect);
      const uint16_t* delta = kbar;
      for (int l = p.L - 1; l >= 0; --l) {
        const Layer& y = p.layers[l];
        GemmNT g{};
        g.A = delta;
        g.lda = y.Npad;
        g.W = u16(y.WTp);
        g.ldw = p.conv ? 9 * y.Npad : y.Npad;
        uint16_t* out = (l == 0) ? u16(p.ZBAR) + (size_t)j * p.stage_stride
                                 : u16(p.DELTA[l - 1]) + (size_t)j * p.R * y.Kpad;
        g.C = out;
        g.ldc = y.Kpad;
        g.M = (int)p.R;
        g.N = y.Kpad;
        g.K = g.ldw;
        g.bias = nullptr;
        g.wt = nullptr;
        g.tau = 0.f;
        g.act_tanh = 0;
        if (l > 0) {
          g.dact = u16(p.ACT[l - 1]) + (size_t)j * p.R * y.Kpad;
          g.ldd = y.Kpad;
        }
        g.ctl = ctl;
        g.detect = detect;
        g.H = p.H;
        g.Wd = p.Wd;
        g.Cpad = y.Npad;
        launch_nt(g);
        delta = out;
      }
    }
    if (detect) chain_decide<<<1, 1, 0, st>>>(ctl, i);
    // parameter gradient: contraction over all stages and rows at once
    const int64_t rows = (int64_t)s * p.R;
    for (int l = 0; l < p.L; ++l) {
      const Layer& y = p.layers[l];
      GemmTN g{};
      g.A = (l == p.L - 1) ? u16(p.KBAR) : u16(p.DELTA[l]);
      g.lda = y.Npad;
      g.B = (l == 0) ? u16(p.Z) : u16(p.ACT[l - 1]);
      g.ldb = y.Kpad;
      g.rows = rows;
      // split the contraction so that about 1024 workgroups are in flight
      const int tiles = ((y.Npad + 127) / 128) * ((y.Kpad + 127) / 128) * (p.conv ? 9 : 1);
      int64_t want = (1024 + tiles - 1) / tiles;
      int64_t per = (rows + want - 1) / want;
      per = (per + BK - 1) / BK * BK;
      if (per < 4 * BK) per = 4 * BK;
      g.rows_per_split = (int)per;
      const int splits = (int)((rows + per - 1) / per);
      g.G = grad_theta + y.theta_w;
      g.ldg = p.conv ? y.in_full * 9 : y.in_full;
      g.Na = y.out;
      g.Nb = y.in;
      g.NaPad = y.Npad;
      g.NbPad = y.Kpad;
      g.h = h;
      g.ctl = ctl;
      g.H = p.H;
      g.Wd = p.Wd;
      g.taps = p.conv ? 9 : 1;
      dim3 grid((y.Npad + 127) / 128, (y.Kpad + 127) / 128, splits * g.taps);
      {
        TimeScope ts(RAMPDE_K_WGRAD_GEMM, 2.0 * rows * (double)y.Npad * y.Kpad * g.taps, st);
        if (p.conv)
          gemm_tn<T, true><<<grid, 256, 0, st>>>(g);
        else
          gemm_tn<T, false><<<grid, 256, 0, st>>>(g);
      }
      // bias and time-weight gradients
      int rpb = (int)((rows + 255) / 256);
      if (rpb < 64) rpb = 64;
      dim3 cgrid(y.Npad / 64, blocks_for(rows, rpb));
      float* gb = grad_theta + y.theta_b;
      float* gwt = y.has_time ? grad_theta + y.theta_w + (p.conv ? (size_t)y.in * 9 : (size_t)y.in) : nullptr;
      if (p.conv)
        column_sums<T, true><<<cgrid, 256, 0, st>>>(g.A, y.Npad, p.R, s, y.out, taus, h, gb, gwt, y.in_full * 9, p.H,
                                                    p.Wd, rpb, ctl);
      else
        column_sums<T, false><<<cgrid, 256, 0, st>>>(g.A, y.Npad, p.R, s, y.out, taus, h, gb, gwt, y.in_full, p.H,
                                                     p.Wd, rpb, ctl);
    }
    {
      // bytes per state element: read a (4) + s stage cotangents (2 each) + write a (4)
      TimeScope ts(RAMPDE_K_ADJOINT_UPDATE, (double)p.n * (8.0 + 2.0 * s), st);
      adjoint_update<T><<<blocks_for(p.n, 256), 256, 0, st>>>(a, p.d, u16(p.ZBAR), p.stage_stride, s, h, gys_i, p.dpad,
                                                             p.R, ctl);
    }
    scale_grow<<<1, 1, 0, st>>>(ctl, f32(p.scale_hist), i, Low<T>::p_bits, dynamic,
                                (pol->flags & RAMPDE_GROW_RAW_NORM) ? 1 : 0);
  }

  int backward(const float* theta, const double* tgrid, int N, const rampde_tableau* tab, const rampde_policy* pol,
               rampde_scaling scaling, const uint16_t* ckpt, const float* grad_yN, const float* grad_ys,
               float* grad_y0, float* grad_theta, float* scale_hist, rampde_stats* stats) {
    const int dynamic = scaling == RAMPDE_SCALE_DYNAMIC;
    const int detect = dynamic || scaling == RAMPDE_SCALE_NONE_SAFE;
    const int k_max = pol->k_max > 0 ? pol->k_max : 16;
    const int HW = p.H * p.Wd;
    ctl_reset<<<1, 1, 0, st>>>(ctl);
    cast_weights(theta);
    float* a = grad_y0;
    float* gys_rows = nullptr;
    auto gys_at = [&](int i) -> const float* {
      if (!grad_ys) return nullptr;
      const float* src = grad_ys + (size_t)i * p.n;
      if (!p.conv) return src;
      nchw_to_rows<<<blocks_for(p.n, 256), 256, 0, st>>>(src, gys_rows, p.R, p.d, HW);
      return gys_rows;
    };
    if (p.conv) {
      a = f32(p.a_rows);
      gys_rows = f32(p.gys_rows);
      nchw_to_rows<<<blocks_for(p.n, 256), 256, 0, st>>>(grad_yN, a, p.R, p.d, HW);
      init_adjoint<<<blocks_for(p.n, 256), 256, 0, st>>>(a, gys_at(N), a, p.n, ctl, 0);
    } else {
      init_adjoint<<<blocks_for(p.n, 256), 256, 0, st>>>(grad_yN, gys_at(N), a, p.n, ctl, 1);
    }
    scale_init<<<1, 1, 0, st>>>(ctl, f32(p.scale_hist), N, Low<T>::p_bits, dynamic);

    Ctl hctl;
    memset(&hctl, 0, sizeof hctl);
    int from = N - 1;
    bool recompute_first = true;
    int status = RAMPDE_OK;
    const bool must_sync = detect || stats || scale_hist;
    for (;;) {
      for (int i = from; i >= 0; --i) {
        backward_step(i, tgrid, tab, pol, ckpt, a, gys_at(i), grad_theta, dynamic, detect,
                      i == from ? recompute_first : true);
      }
      HIP_TRY(hipGetLastError());
      if (!must_sync) break;
      HIP_TRY(hipMemcpyAsync(&hctl, ctl, sizeof(Ctl), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      if (!hctl.poison) break;
      if (!dynamic) break;  // NONE_SAFE: handled below
      if (hctl.failed_step >= N || hctl.attempt >= k_max) {
        status = RAMPDE_ESCALE;
        break;
      }
      chain_retry<<<1, 1, 0, st>>>(ctl);
      from = hctl.failed_step;
      recompute_first = false;  // the stage values of the failed step are still in the workspace
    }
    int st_code = 0;
    if (must_sync && hctl.poison) {
      if (dynamic) {
        st_code = 2;
        status = RAMPDE_ESCALE;
      } else {
        st_code = 1;
        fill_inf_if_poisoned<<<blocks_for(p.n, 256), 256, 0, st>>>(a, p.n, ctl);
        fill_inf_if_poisoned<<<blocks_for(p.P, 256), 256, 0, st>>>(grad_theta, p.P, ctl);
      }
    }
    if (p.conv) rows_to_nchw<<<blocks_for(p.n, 256), 256, 0, st>>>(a, grad_y0, p.R, p.d, HW, nullptr, 0);
    HIP_TRY(hipGetLastError());
    if (scale_hist) {
      HIP_TRY(hipMemcpyAsync(scale_hist, f32(p.scale_hist), sizeof(float) * (size_t)(N + 1), hipMemcpyDeviceToHost, st));
    }
    if (must_sync) HIP_TRY(hipStreamSynchronize(st));
    if (stats) {
      stats->status = st_code;
      stats->failed_step = hctl.poison ? hctl.failed_step : -1;
      stats->retries = hctl.retries;
      stats->s_min = hctl.s_min;
      stats->s_max = hctl.s_max;
      stats->s_first = 0.f;
      stats->s_last = 0.f;
      if (scale_hist) {
        stats->s_first = scale_hist[N];
        stats->s_last = scale_hist[0];
      }
    }
    return status;
  }
};

static rampde_scaling resolve_scaling(const rampde_policy* pol) {
  if (pol->scaling != RAMPDE_SCALE_AUTO) return pol->scaling;
  return pol->low == RAMPDE_F16 ? RAMPDE_SCALE_DYNAMIC : RAMPDE_SCALE_NONE;
}

}  // namespace rampde

using namespace rampde;

extern "C" {

int64_t rampde_num_params(const rampde_velocity* vel) {
  Plan p;
  if (!build_layers(vel, p)) return 0;
  return p.P;
}

size_t rampde_workspace_bytes(const rampde_velocity* vel, int64_t B, int N, const rampde_tableau* tab,
                              const rampde_policy* pol, int is_backward) {
  (void)pol;
  Plan p = make_plan(vel, B, N, tab, is_backward);
  return p.ok ? p.total : 0;
}

int rampde_odeint_fwd(const rampde_velocity* vel, const float* theta, const float* y0, int64_t B,
                      const double* tgrid, int N, const rampde_tableau* tab, const rampde_policy* pol, void* ckpt,
                      float* yN, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(vel, tgrid, N, tab, pol);
  if (rc) return rc;
  if (!theta || !y0 || !ckpt || !yN || !workspace || B < 1) return RAMPDE_EINVAL;
  Plan p = make_plan(vel, B, N, tab, 0);
  if (!p.ok) return RAMPDE_EINVAL;
  if (workspace_bytes < p.total || ((uintptr_t)workspace & 255)) return RAMPDE_EWORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (pol->low == RAMPDE_F16) {
    Runner<F16> r(p, workspace, st);
    return r.forward(theta, y0, tgrid, N, tab, pol, (uint16_t*)ckpt, yN);
  }
  Runner<BF16> r(p, workspace, st);
  return r.forward(theta, y0, tgrid, N, tab, pol, (uint16_t*)ckpt, yN);
}

int rampde_odeint_bwd(const rampde_velocity* vel, const float* theta, int64_t B, const double* tgrid, int N,
                      const rampde_tableau* tab, const rampde_policy* pol, const void* ckpt, const float* grad_yN,
                      const float* grad_ys, float* grad_y0, float* grad_theta, float* scale_hist,
                      rampde_stats* stats, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(vel, tgrid, N, tab, pol);
  if (rc) return rc;
  if (!theta || !ckpt || !grad_yN || !grad_y0 || !grad_theta || !workspace || B < 1) return RAMPDE_EINVAL;
  Plan p = make_plan(vel, B, N, tab, 1);
  if (!p.ok) return RAMPDE_EINVAL;
  if (workspace_bytes < p.total || ((uintptr_t)workspace & 255)) return RAMPDE_EWORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const rampde_scaling sc = resolve_scaling(pol);
  if (pol->low == RAMPDE_F16) {
    Runner<F16> r(p, workspace, st);
    return r.backward(theta, tgrid, N, tab, pol, sc, (const uint16_t*)ckpt, grad_yN, grad_ys, grad_y0, grad_theta,
                      scale_hist, stats);
  }
  Runner<BF16> r(p, workspace, st);
  return r.backward(theta, tgrid, N, tab, pol, sc, (const uint16_t*)ckpt, grad_yN, grad_ys, grad_y0, grad_theta,
                    scale_hist, stats);
}

const char* rampde_strerror(int code) {
  switch (code) {
    case RAMPDE_OK: return "ok";
    case RAMPDE_EINVAL: return "invalid argument";
    case RAMPDE_EUNSUPPORTED: return "unsupported dtype, velocity kind or shape";
    case RAMPDE_EWORKSPACE: return "workspace too small or not 256-byte aligned";
    case RAMPDE_ESCALE: return "dynamic adjoint scaling failed (no finite scale within k_max attempts)";
    case RAMPDE_EHIP: return g_hip_msg;
    default: return "unknown status code";
  }
}

int rampde_version(void) { return 100; }

int rampde_timing_enable(int on) {
  for (auto& t : g_timed) {
    (void)hipEventDestroy(t.e0);
    (void)hipEventDestroy(t.e1);
  }
  g_timed.clear();
  g_timing = on != 0;
  return RAMPDE_OK;
}

int rampde_timing_read(int kernel_class, rampde_kernel_time* out) {
  if (!out || kernel_class < 0 || kernel_class >= RAMPDE_K_CLASSES) return RAMPDE_EINVAL;
  out->ms = 0.0;
  out->launches = 0;
  out->work = 0.0;
  for (auto& t : g_timed) {
    if (t.cls != kernel_class) continue;
    HIP_TRY(hipEventSynchronize(t.e1));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, t.e0, t.e1));
    out->ms += ms;
    out->launches += 1;
    out->work += t.work;
  }
  return RAMPDE_OK;
}

}  // extern "C"
