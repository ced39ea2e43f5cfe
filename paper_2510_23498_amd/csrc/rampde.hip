// C-ABI entry points of the gfx950 mixed-precision neural-ODE time stepper: argument
// validation, workspace planning and the launch sequences of the forward pass (paper
// Algorithm 1) and of the discrete adjoint with dynamic adjoint scaling (paper Algorithm 2).
// Every step of the method runs in the kernels of gemm.hpp / elementwise.hpp; the host only
// orders launches and, under dynamic scaling, re-enqueues from a step whose cotangent chain
// overflowed (halve-and-retry of Algorithm 2).
#include "../../include/rampde.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <type_traits>
#include <vector>

#include "common.hpp"
#include "elementwise.hpp"
#include "fused_launch.hpp"
#include "wide.hpp"
#include "gemm.hpp"
#include "wgrad_slab.hpp"
#include "gemm_slab.hpp"
#include "conv_wgrad_tr.hpp"
#include "conv.hpp"
#include "norm.hpp"
#include "cnf.hpp"

namespace rampde {

static inline int pad64(int x) { return (x + kPad - 1) / kPad * kPad; }
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
// the kernels read states, gradients and checkpoints with 16-byte vector loads
static inline bool aligned16(const void* ptr) { return ((uintptr_t)ptr & 15) == 0; }

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
  size_t Wf, WTf;  // fragment-major copies (row-tile-persistent kernels)
  int ldw;  // K extent of the forward GEMM (dense: Kpad; conv: 9 * Cpad)
  // all-taps convolution weight gradient: K-chunk length, chunk count, the chunks' private copies
  int cw_per = 0, cw_splits = 0;
  size_t cw_part = 0;
  size_t cw_floats = 0;  // fp32 elements of all the copies
};

struct Plan {
  bool ok = false;
  bool conv = false;
  // parabolic block -W^T N(relu(W y + b)) (Sec. 6.3): one convolution used forward and transposed, an
  // instance normalisation between them, parameters piecewise constant over n_intervals pieces of the grid
  bool parabolic = false;
  // normalising-flow state [z; l] with the exact trace row (Sec. 6.1): the one-hidden-layer velocity on the
  // dense per-layer kernels, state width d + 1
  bool cnf = false;
  size_t cnf_c = 0, cnf_s = 0;       // c_h and the per-step sums s_h, fp32 [Hpad]
  int n_intervals = 1;
  int64_t Pblk = 0;                  // parameters of one piece
  size_t nstat = 0, nstat_vjp = 0, npart = 0;  // statistics [stage][B][Cpad][2], VJP means, chunk sums
  int norm_chunks = 1, norm_rpc = 0;
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
  // row-tile-persistent path (dense networks whose widest layer fits the LDS tiles)
  bool fused = false;
  int MT = 1;          // row tile = 16 * MT
  bool wide = false;   // 64-row tiles of the kernels for 512-wide networks (wide.hpp)
  int ldp = 0;         // LDS row pitch (elements)
  size_t lds_bytes = 0;
  size_t steptab = 0, a_alt = 0, bsum = 0;
  size_t tpart = 0;                 // [N][2] fp32 per-step sums of the time-grid gradient
  size_t tslots = 0;                // per-workgroup slots of the launch that is adding to them (kTimeSlotPairs pairs)
  size_t amax_slots = 0;            // [4096] per-workgroup maxima of |a| (per-layer path)
  int nparam = 0, wt_off = 0;
  bool k_in_lds = false;
  bool overlap_wgrad = false;       // narrow nets: 4-wave adjoint kernel + parameter gradients on a helper stream
  int64_t Rp = 0, ldk = 0;          // feature-major buffers: k = stage * Rp + row
  int ksplits = 1, kchunk = 64;     // K-chunks of the parameter-gradient contraction
  bool cw_blocks = false;           // convolutions: keep the weight-gradient kernel with 64 x 64 channel blocks (policy.wgrad_tile = 64)
  bool wgrad_slab = false;          // per-step parameter gradients by the 128 x 128-per-wavefront kernel
  int wgrad_group = 1;              // ... of this many adjoint steps per launch (each step has a buffer set of its own)
  size_t gpart = 0;                 // ksplits copies of the gradient vector
  size_t ZT = 0, KBART = 0;
  size_t fm_stride = 0;             // distance between the sets of feature-group-major buffers
  int act_lds_off = 0;              // adjoint kernel: LDS offset (16-bit elements) of the activation copy, 0 = none
  int nsets = 2;                    // sets: step i uses set i % nsets
  int step_group = 1;               // adjoint steps per kernel launch (> 1: fixed scale, no detection)
  std::vector<size_t> ACTT, DELTAT;
};

static bool build_layers(const rampde_velocity* vel, Plan& p, int hidden_pad = kPad) {
  if (!vel) return false;
  size_t off = 0;
  if (vel->kind == RAMPDE_VEL_MLP || vel->kind == RAMPDE_VEL_CNF) {
    if (vel->n_layers < 1 || vel->n_layers > 16 || !vel->widths) return false;
    if (vel->kind == RAMPDE_VEL_CNF && vel->n_layers != 2) return false;
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
      // hidden widths may be padded further (the row-tile-persistent kernels want multiples of 256)
      y.Npad = (l + 1 < p.L) ? (y.out + hidden_pad - 1) / hidden_pad * hidden_pad : pad64(y.out);
      y.Kpad = (l > 0) ? (y.in + hidden_pad - 1) / hidden_pad * hidden_pad : pad64(y.in);
      y.ldw = y.Kpad;
      y.theta_w = off;
      off += (size_t)y.out * y.in_full;
      y.theta_b = off;
      off += y.out;
      p.layers.push_back(y);
    }
    if (vel->kind == RAMPDE_VEL_CNF) {
      // the state carries one more column (l) than the velocity reads or writes: it meets zero weights
      p.cnf = true;
      p.d = vel->widths[0] + 1;
      p.layers[0].Kpad = p.layers[0].ldw = pad64(p.d);
      p.layers[1].Npad = pad64(p.d);
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
  } else if (vel->kind == RAMPDE_VEL_PARABOLIC) {
    if (vel->C < 1 || vel->C > 4096 || vel->H < 1 || vel->W < 1 || vel->H > 4096 || vel->W > 4096) return false;
    if (vel->n_intervals < 0 || vel->n_intervals > 65536 || vel->time_input) return false;
    p.conv = true;
    p.parabolic = true;
    p.n_intervals = vel->n_intervals > 0 ? vel->n_intervals : 1;
    p.L = 1;
    p.d = vel->C;
    p.H = vel->H;
    p.Wd = vel->W;
    Layer y{};
    y.out = y.in = y.in_full = vel->C;
    y.has_time = 0;
    y.Npad = y.Kpad = pad64(vel->C);
    y.ldw = 9 * y.Kpad;
    y.theta_w = 0;
    y.theta_b = (size_t)vel->C * vel->C * 9;
    p.layers.push_back(y);
    p.Pblk = (int64_t)y.theta_b + vel->C;
    off = (size_t)p.Pblk * p.n_intervals;
  } else {
    return false;
  }
  p.P = (int64_t)off;
  p.dpad = pad64(p.d);
  return true;
}

static rampde_scaling resolve_scaling(const rampde_policy* pol);
struct Plan;
// the all-taps convolution weight-gradient kernel: image lines of a multiple of 8 pixels, at most
// 64, and whole 128-row k-steps within a stage
static bool conv_wgrad_applies(const Plan& p);
// Time-grid gradient: every workgroup that adds to a step's sums writes a slot of its own, and a one-workgroup kernel
// folds the launch's slots in a fixed order (no floating-point atomics: the result does not depend on the order in
// which workgroups finish).  Slots of one launch: workgroups x steps of the launch.
constexpr size_t kTimeSlotPairs = size_t(1) << 19;
static bool conv_wgrad_tr_applies(const Plan& p);
static bool conv_wgrad_tr64_applies(const Plan& p, const Layer& y);
// compute units of the current device (256 on MI355X; also the answer when no device is visible,
// e.g. a workspace query on a host without a GPU)
static int device_compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  return cus;
}

static bool fused_candidate(const rampde_velocity* vel, const rampde_policy* pol) {
  if (!vel || vel->kind != RAMPDE_VEL_MLP || (pol && (pol->flags & RAMPDE_PER_LAYER_KERNELS))) return false;
  if (vel->n_layers < 1 || vel->n_layers > kMaxLayers || !vel->widths) return false;
  const int dp = pad64(vel->widths[0]);
  return dp == 64 || dp == 128 || dp == 256;
}

// allow_wide = false: never the kernels of wide.hpp (the backward pass that also forms the time-grid
// gradient runs on the other row-tile kernels)
static Plan make_plan(const rampde_velocity* vel, int64_t B, int N, const rampde_tableau* tab,
                      const rampde_policy* pol, int is_backward, bool allow_wide = true) {
  Plan p;
  const bool allow_fused = fused_candidate(vel, pol);
  if (!build_layers(vel, p, allow_fused ? 256 : kPad)) return p;
  if (B < 1 || N < 1 || !tab || tab->s < 1 || tab->s > kMaxStages) return p;
  p.s = tab->s;
  p.cw_blocks = pol && pol->wgrad_tile == 64;
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
  if (allow_fused) {
    int maxw = 0, nparam = 0;
    for (auto& y : p.layers) {
      maxw = std::max(maxw, std::max(y.Npad, y.Kpad));
      nparam += y.Npad;
    }
    p.wt_off = nparam;
    p.nparam = nparam + p.layers[0].Npad;
    p.ldp = maxw + 8;
    const size_t lds_limit = 159 * 1024;  // 160 KB per compute unit minus the kernels' small static arrays
    auto lds_need = [&](int mt, bool with_k) {
      const size_t tm = 16 * (size_t)mt;
      return (size_t)p.nparam * 4 + tm * (p.dpad + 8) * 2 + 2 * tm * p.ldp * 2 +
             (with_k ? (size_t)p.s * tm * (p.dpad + 8) * 2 : 0);
    };
    // (the adjoint kernel carries more per-tile state in registers: it spills beyond 32-row tiles)
    int mt = is_backward ? 2 : 4;
    const int want_rows = pol ? pol->row_tile : 0;
    if (want_rows == 16 || want_rows == 32 || (want_rows == 64 && !is_backward)) mt = want_rows / 16;
    // largest row tile that still gives every compute unit a workgroup and fits the LDS tiles
    while (mt > 1 && ((want_rows == 0 && (p.R + 16 * mt - 1) / (16 * mt) < 256) || lds_need(mt, false) > lds_limit)) mt >>= 1;
    // Networks with 512-wide hidden layers and a 128-wide state: the 64-row-tile kernels of wide.hpp,
    // forward and adjoint, when the batch gives at least half of the compute units a tile (or on
    // request).  Not for the time-grid gradient, and not where a fixed scale lets the other adjoint
    // kernel run groups of steps per launch.
    bool all512 = p.L >= 2;
    for (int l = 0; l + 1 < p.L; ++l) all512 = all512 && p.layers[l].Npad == 512;
    const bool fixed_scale = pol && resolve_scaling(pol) == RAMPDE_SCALE_NONE;
    if (allow_wide && all512 && p.d == 128 && !(is_backward && fixed_scale) &&
        (want_rows == 64 || (want_rows == 0 && (p.R + 63) / 64 >= 128)) &&
        (size_t)p.nparam * 4 + 64 * (size_t)(128 + 8) * 2 + 2 * 64 * (size_t)(512 + 8) * 2 <= lds_limit) {
      p.wide = true;
      mt = 4;
    }
    if (p.wide || lds_need(mt, false) <= lds_limit) {
      p.fused = true;
      p.MT = mt;
      p.k_in_lds = !p.wide && lds_need(mt, true) <= lds_limit;
      p.overlap_wgrad = (mt == 1 && maxw <= 256);
      p.lds_bytes = p.wide ? (size_t)p.nparam * 4 + 64 * (size_t)(128 + 8) * 2 + 2 * 64 * (size_t)(512 + 8) * 2
                           : lds_need(mt, p.k_in_lds);
      if (is_backward && p.L > 1 && !p.wide) {
        // a copy of the step's hidden activations for the tanh' factors, when it still fits
        const size_t act_bytes = (size_t)p.s * (p.L - 1) * 16 * mt * p.ldp * 2;
        if (p.lds_bytes + act_bytes <= lds_limit) {
          p.act_lds_off = (int)(p.lds_bytes / 2);
          p.lds_bytes += act_bytes;
        }
      }
      for (auto& y : p.layers) {
        y.Wf = take((size_t)y.Npad * y.Kpad * 2);
        y.WTf = take((size_t)y.Npad * y.Kpad * 2);
      }
      p.steptab = take(sizeof(float) * (size_t)N * (1 + p.s));
      if (is_backward) p.a_alt = take(sizeof(float) * (size_t)p.n);
    } else {
      // the tiles do not fit in LDS: fall back to the per-layer kernels with their own padding
      rampde_policy pl = pol ? *pol : rampde_policy{};
      pl.flags |= RAMPDE_PER_LAYER_KERNELS;
      return make_plan(vel, B, N, tab, &pl, is_backward, allow_wide);
    }
  }
  const int sbuf = is_backward ? p.s : 1;  // forward keeps one stage of inputs/activations
  if (p.conv) {
    p.y_rows = take(sizeof(float) * (size_t)p.n);
    if (is_backward) {
      p.a_rows = p.y_rows;
      p.gys_rows = take(sizeof(float) * (size_t)p.n);
    }
  }
  if (p.cnf) {
    p.cnf_c = take(sizeof(float) * p.layers[0].Npad);
    p.cnf_s = take(sizeof(float) * p.layers[0].Npad);
  }
  if (p.fused) {
    // row-tile-persistent kernels: slopes / stage cotangents only when they do not fit in LDS;
    // the adjoint stores everything the parameter-gradient contraction (and tanh') reads
    // feature-group-major
    p.K = take((size_t)p.s * p.R * p.dpad * 2);
    if (p.wide && !is_backward) p.bsum = take(sizeof(float) * (size_t)p.R * p.dpad);
    if (is_backward) {
      p.ZBAR = take((size_t)p.s * p.R * p.dpad * 2);
      p.Rp = (p.R + 63) / 64 * 64;
      p.ldk = (int64_t)p.s * p.Rp;
      size_t per_set = 2 * (size_t)p.dpad * p.ldk * 2;
      for (int l = 0; l + 1 < p.L; ++l) per_set += 2 * (size_t)p.layers[l].Npad * p.ldk * 2;
      const int64_t fit = (int64_t)((size_t(4) << 30) / per_set);  // buffer sets in about 4 GiB
      {
        // Without overflow detection nothing is decided between steps: a launch of the adjoint
        // kernel then runs a group of steps (the adjoint stays in registers) and the parameter
        // gradients of the whole group are one contraction.  Every step of a group needs its own
        // set of buffers; groups are as long as about 4 GiB of sets allow.
        const int64_t want_group = (pol && pol->step_group > 0) ? pol->step_group : kMaxWgradSteps;
        const int64_t cap = std::min<int64_t>(want_group, std::min<int64_t>(fit, kMaxWgradSteps));
        if (pol && resolve_scaling(pol) == RAMPDE_SCALE_NONE && cap >= 2) {
          p.step_group = (int)std::min<int64_t>(N, cap);
          p.nsets = p.step_group;
          p.overlap_wgrad = false;
        }
      }
      {
        // Long contractions (one launch per step, kernel not sharing the CUs): the kernel whose
        // wavefronts own 128 x 128 blocks and stream the operands through LDS without registers.
        // The adjoint kernel runs step by step under overflow detection (a step must be accepted before the
        // next one starts), but the parameter gradients of several accepted steps can be ONE contraction over
        // their buffer sets: one pass over the private gradient copies per group instead of one per step.
        // That pays as long as the group's buffer sets are still in the memory-side cache when they are read
        // (about half of its 256 MB is left to them); the headline workload's set is larger than that.
        const int want_tile = pol ? pol->wgrad_tile : 0;
        const int64_t cached = std::max<int64_t>(1, (int64_t)((size_t(128) << 20) / per_set));
        const int64_t want = (pol && pol->step_group > 0) ? pol->step_group : cached;
        const int64_t group = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, fit), std::min<int64_t>(N, kMaxWgradSteps)));
        // (the kernel addresses a lane's part of an operand tensor by a 32-bit byte offset)
        bool offsets_fit = (size_t)p.dpad * p.ldk * 2 < (size_t(1) << 32);
        for (auto& y : p.layers) offsets_fit = offsets_fit && (size_t)std::max(y.Npad, y.Kpad) * p.ldk * 2 < (size_t(1) << 32);
        p.wgrad_slab = !p.overlap_wgrad && p.step_group <= 1 && offsets_fit &&
                       (want_tile == 256 || (want_tile != 128 && group * p.ldk >= kSlabMinK));
        if (p.wgrad_slab) {
          p.wgrad_group = (int)group;
          p.nsets = p.wgrad_group;
        }
        int tiles = 0;
        for (auto& y : p.layers) {
          if (p.wgrad_slab) {
            const SlabShape sh = slab_shape(y.Npad, y.Kpad);
            tiles += ((y.Npad + slab_tile_a(sh) - 1) / slab_tile_a(sh)) * ((y.Kpad + slab_tile_b(sh) - 1) / slab_tile_b(sh));
          } else {
            tiles += ((y.Npad + 127) / 128) * ((y.Kpad + 127) / 128);
          }
        }
        // K-chunks: as many workgroups as are resident at once (two per CU; one when the kernel
        // shares the CUs with the adjoint kernel or needs a CU's whole LDS) and no more -- a second,
        // partial round of workgroups costs more than it spreads --, but at least 256 k per chunk
        const int resident = device_compute_units() * ((p.overlap_wgrad || p.wgrad_slab) ? 1 : 2);
        int64_t ks = std::max(1, resident / tiles);
        // (a group of steps multiplies a workgroup's k-steps: chunks can be shorter)
        const int64_t min_chunk = p.step_group > 1 ? 128 : 256;
        ks = std::max<int64_t>(1, std::min<int64_t>(ks, p.ldk / min_chunk > 0 ? p.ldk / min_chunk : 1));
        const int64_t kc = ((p.ldk + ks - 1) / ks + 63) / 64 * 64;
        p.kchunk = (int)kc;
        p.ksplits = (int)((p.ldk + kc - 1) / kc);
        p.gpart = take(sizeof(float) * (size_t)p.ksplits * p.P);
      }
      // two sets of the per-step buffers: the parameter-gradient kernel of step i reads set i % 2
      // on a helper stream while the adjoint kernel of step i - 1 already fills the other set
      const size_t fm_begin = off;
      p.ZT = take((size_t)p.dpad * p.ldk * 2);
      p.KBART = take((size_t)p.dpad * p.ldk * 2);
      for (int l = 0; l + 1 < p.L; ++l) {
        p.ACTT.push_back(take((size_t)p.layers[l].Npad * p.ldk * 2));
        p.DELTAT.push_back(take((size_t)p.layers[l].Npad * p.ldk * 2));
      }
      p.fm_stride = off - fm_begin;
      for (int q = 1; q < p.nsets; ++q) take(p.fm_stride);  // the other sets
    }
  } else {
    p.Z = take((size_t)sbuf * p.R * p.dpad * 2);
    p.K = take((size_t)p.s * p.R * p.dpad * 2);
    for (int l = 0; l + 1 < p.L; ++l) p.ACT.push_back(take((size_t)sbuf * p.R * p.layers[l].Npad * 2));
    if (p.parabolic) {
      // ACT[0] = post-ReLU activation r, ACT[1] = normalised activation n; per-stage statistics
      const Layer& y = p.layers[0];
      const int64_t HW = (int64_t)p.H * p.Wd, Bn = p.R / HW;
      for (int q = 0; q < 2; ++q) p.ACT.push_back(take((size_t)sbuf * p.R * y.Npad * 2));
      p.nstat = take(sizeof(float) * 2 * (size_t)sbuf * Bn * y.Npad);
      p.nstat_vjp = take(sizeof(float) * 2 * (size_t)Bn * y.Npad);
      // pixel chunks of the statistics sums: enough workgroups to fill the device, at least 256 pixels each
      const int64_t base = (int64_t)(y.Npad / 64) * Bn;
      int64_t chunks = std::max<int64_t>(1, std::min<int64_t>(16, (2 * device_compute_units() + base - 1) / base));
      int64_t rpc = std::max<int64_t>(256, ((HW + chunks - 1) / chunks + 31) / 32 * 32);
      p.norm_rpc = (int)rpc;
      p.norm_chunks = (int)((HW + rpc - 1) / rpc);
      p.npart = take(sizeof(float) * 2 * (size_t)p.norm_chunks * Bn * y.Npad);
    }
    if (is_backward) {
      p.KBAR = take((size_t)p.s * p.R * p.dpad * 2);
      p.ZBAR = take((size_t)p.s * p.R * p.dpad * 2);
      for (int l = 0; l + 1 < p.L; ++l) p.DELTA.push_back(take((size_t)p.s * p.R * p.layers[l].Npad * 2));
      if (p.parabolic)  // DELTA[0] = cotangent of n, DELTA[1] = cotangent of the pre-activation
        for (int q = 0; q < 2; ++q) p.DELTA.push_back(take((size_t)p.s * p.R * p.layers[0].Npad * 2));
      if (conv_wgrad_applies(p)) {
        // every (K-chunk, 64 x 64 channel block) accumulates its 9 tap blocks over all steps in a
        // copy of its own; one workgroup per compute unit (its LDS holds one), at least 4 k-steps
        // each: fewer, longer chunks keep the read-modify-write of the copies and the pipeline
        // fill small against the multiplication
        const int64_t rows = (int64_t)p.s * p.R;
        if (conv_wgrad_tr_applies(p)) {
          // many channels: (128 x 128 channels, one dy) per workgroup, K-chunks of whole image lines, one workgroup per
          // compute unit
          Layer& y = p.layers[0];
          const int tiles_a = y.Npad / 128, gsize = y.Kpad / 128 * 3, tiles = tiles_a * gsize;
          const int64_t lines = rows / p.Wd;
          // (a group -- the workgroups of one output-channel block and K-chunk -- runs on one XCD: as many whole groups
          // as an XCD's compute units hold)
          const int per_xcd = std::max(1, device_compute_units() / 8 / gsize);
          const int64_t want = std::max<int64_t>(1, 8 * per_xcd / tiles_a);
          const int64_t per = std::max<int64_t>((lines + want - 1) / want, std::min<int64_t>(lines, 4 * (64 / p.Wd)));
          y.cw_per = (int)per;
          y.cw_splits = (int)((lines + per - 1) / per);
          y.cw_floats = (size_t)y.cw_splits * tiles * CT_SLOT;
          y.cw_part = take(sizeof(float) * y.cw_floats);
        } else
        for (auto& y : p.layers) {
          const int tiles = (y.Npad / 64) * (y.Kpad / 64);
          const int64_t want = std::max<int64_t>(1, device_compute_units() / tiles);
          int64_t per = ((rows + want - 1) / want + CW_KS - 1) / CW_KS * CW_KS;
          if (per < 4 * CW_KS) per = 4 * CW_KS;
          y.cw_per = (int)per;
          y.cw_splits = (int)((rows + per - 1) / per);
          y.cw_floats = (size_t)y.cw_splits * tiles * CW_SLOT;
          y.cw_part = take(sizeof(float) * y.cw_floats);
        }
      }
    }
  }
  if (is_backward) p.tpart = take(sizeof(float) * 2 * (size_t)N);
  if (is_backward) p.tslots = take(sizeof(float) * 2 * (size_t)kTimeSlotPairs);
  if (is_backward) p.amax_slots = take(sizeof(unsigned) * 4096);  // per-workgroup maxima of the streaming adjoint update
  p.total = off;
  p.ok = true;
  return p;
}

static bool conv_wgrad_applies(const Plan& p) { return p.conv && !p.fused && p.Wd % 8 == 0 && p.Wd <= 64 && p.R % CW_KS == 0; }
// (64 x 64 channels, 16 / 32 / 64 pixels per line: conv_wgrad's drop-in built on transposing LDS reads)
static bool conv_wgrad_tr64_applies(const Plan& p, const Layer& y) {
  return conv_wgrad_applies(p) && !p.cw_blocks && y.Npad == 64 && y.Kpad == 64 && (p.Wd == 16 || p.Wd == 32 || p.Wd == 64);
}
// (the kernel built on transposing LDS reads: the parabolic block's one layer, channel counts in multiples of 128)
static bool conv_wgrad_tr_applies(const Plan& p) {
  return conv_wgrad_applies(p) && p.parabolic && !p.cw_blocks &&
         (p.Wd == 16 || p.Wd == 32 || p.Wd == 64) && p.layers[0].Npad % 128 == 0 && p.layers[0].Kpad % 128 == 0 &&
         !p.layers[0].has_time;
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

__global__ void fill_u32(uint32_t* p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void fill_zero_u32(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

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

// Host floats -> device memory by way of kernel arguments (copied at launch: no host buffer has
// to outlive the call, and the write is an ordinary kernel node for a caller capturing a graph).
struct FloatChunk {
  float v[768];
};
__global__ void write_floats(FloatChunk c, float* dst, int count) {
  for (int i = threadIdx.x; i < count; i += blockDim.x) dst[i] = c.v[i];
}

// Helper stream on which the parameter-gradient kernel of step i runs while the adjoint kernel
// of step i - 1 runs on the caller's stream (fork / join by events: from the caller's point of
// view all work is still ordered on its stream).  One per process, default priority, created
// on first use; events are pooled.  Calls of the backward pass from several host threads at
// once would share it: they are serialised by the pool's owner (not supported concurrently).
struct SideStream {
  hipStream_t stream = nullptr;
  std::vector<hipEvent_t> ev;  // 2 per step: adjoint done, parameter gradient done
  static SideStream& get() {
    static SideStream s;
    return s;
  }
  int prepare(int N) {
    if (!stream) HIP_TRY(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));
    while ((int)ev.size() < 2 * N) {
      hipEvent_t e;
      HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
      ev.push_back(e);
    }
    return RAMPDE_OK;
  }
  hipEvent_t adjoint_done(int i) { return ev[2 * i]; }
  hipEvent_t wgrad_done(int i) { return ev[2 * i + 1]; }
};

// ---------------------------------------------------------------- typed launch sequences
template <class T>
struct Runner {
  const Plan& p;
  char* ws;
  hipStream_t st;
  Ctl* ctl;
  // elements from one stored state (and one running-cost cotangent) to the next: the rows of this pass
  // may be a slice (a scale group) of the batch that the caller's buffers hold
  int64_t step_elems;
  Runner(const Plan& plan, void* workspace, hipStream_t stream)
      : p(plan), ws((char*)workspace), st(stream), ctl((Ctl*)((char*)workspace + plan.ctl)), step_elems(plan.n) {}

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
    if (p.cnf) {
      const Layer &y0 = p.layers[0], &y1 = p.layers[1];
      cnf_trace_coef<T><<<blocks_for(y0.Npad, 256), 256, 0, st>>>(u16(y0.Wp), y0.Kpad, u16(y1.Wp), y1.Kpad, y0.in, y0.out,
                                                                 y0.Npad, f32(p.cnf_c));
    }
  }

  // the convolution tile kernel keeps a layer's weights in LDS: more than the default limit
  hipError_t allow_conv_tile_lds() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_slab<T, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kNtSlabLdsBytes);
    if (e != hipSuccess) return e;
    for (const void* f : {reinterpret_cast<const void*>(&conv_nt_lines<T, 1>), reinterpret_cast<const void*>(&conv_nt_lines<T, 2>),
                          reinterpret_cast<const void*>(&conv_nt_lines<T, 4>)}) {
      e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, NtLines<4>::LDS);
      if (e != hipSuccess) return e;
    }
    if (p.Wd < 8 || p.Wd > 64) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&conv3x3_tile<T, 8>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)conv_tile_lds_bytes(p.Wd));
  }

  void launch_nt(const GemmNT& g) {
    TimeScope ts(RAMPDE_K_VELOCITY_GEMM, 2.0 * g.M * (double)g.N * g.K, st);
    if (p.conv && !p.parabolic && conv_tile_applies(g.Cpad, g.N, g.H, g.Wd, g.M)) {
      // persistent: one workgroup per CU (its LDS holds the layer's weights), tiles of 256 pixels
      const int ntiles = (int)(g.M / CT_TILE);
      conv3x3_tile<T, 8><<<std::min(ntiles, device_compute_units()), 512, conv_tile_lds_bytes(g.Wd), st>>>(g);
    } else if (p.conv && !p.cw_blocks && conv_nt_lines_applies(g)) {
      // ... with the input staged by image lines: a block of input channels serves all nine taps from LDS
      dim3 grid(g.M / 512, g.N / 128);
      if (g.Wd == 16) conv_nt_lines<T, 1><<<grid, 256, NtLines<1>::LDS, st>>>(g);
      else if (g.Wd == 32) conv_nt_lines<T, 2><<<grid, 256, NtLines<2>::LDS, st>>>(g);
      else conv_nt_lines<T, 4><<<grid, 256, NtLines<4>::LDS, st>>>(g);
    } else if (p.conv && gemm_nt_slab_applies(g, true)) {
      // wide convolutions (the parabolic block): 256 x 256 workgroup tiles fed by direct global->LDS loads
      dim3 grid(blocks_for(g.M, 256), g.N / 256);
      gemm_nt_slab<T, true><<<grid, 256, kNtSlabLdsBytes, st>>>(g);
    } else if (p.conv) {
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

  // ---- parabolic block (Sec. 6.3): instance-normalisation statistics of stage buffer jb, then the
  // elementwise part; vjp: the two means of the normalisation's cotangent formula
  void norm_stats(const uint16_t* X, const uint16_t* Nrm, float* stat, bool vjp, Ctl* c) {
    const Layer& y = p.layers[0];
    const int64_t HW = (int64_t)p.H * p.Wd, Bn = p.R / HW;
    NormPartial a{};
    a.X = X; a.Nrm = Nrm; a.ld = y.Npad; a.Cpad = y.Npad; a.B = (int)Bn; a.HW = HW;
    a.rows_per_chunk = p.norm_rpc; a.part = f32(p.npart); a.ctl = c;
    dim3 grid(y.Npad / 64, (unsigned)Bn, p.norm_chunks);
    const int64_t n = Bn * y.Npad;
    if (vjp) {
      instnorm_partial<T, true><<<grid, 256, 0, st>>>(a);
      instnorm_finalize<true><<<blocks_for(n, 256), 256, 0, st>>>(f32(p.npart), p.norm_chunks, n, 1.f / (float)HW, kNormEps, stat, c);
    } else {
      instnorm_partial<T, false><<<grid, 256, 0, st>>>(a);
      instnorm_finalize<false><<<blocks_for(n, 256), 256, 0, st>>>(f32(p.npart), p.norm_chunks, n, 1.f / (float)HW, kNormEps, stat, c);
    }
  }
  float* norm_stat_of(int jb) const {
    const int64_t Bn = p.R / ((int64_t)p.H * p.Wd);
    return f32(p.nstat) + 2 * (size_t)jb * Bn * p.layers[0].Npad;
  }
  // k_j = -W^T N(relu(W z_j + b)) from the stage input z (stage buffers jb)
  // caller's NCHW fp32 <-> channels-last rows (per sample: [C][H W] <-> [H W][C])
  void to_rows(const float* nchw, float* rows) {
    const int HW = p.H * p.Wd;
    transpose_samples<<<transpose_grid(p.d, HW, p.R / HW), dim3(32, 8), 0, st>>>(nchw, rows, p.d, HW, (int)(p.R / HW), nullptr, 0);
  }
  void to_nchw(const float* rows, float* nchw) {
    const int HW = p.H * p.Wd;
    transpose_samples<<<transpose_grid(HW, p.d, p.R / HW), dim3(32, 8), 0, st>>>(rows, nchw, HW, p.d, (int)(p.R / HW), nullptr, 0);
  }
  // row blocks x samples of the normalisation's elementwise kernels: about 8 workgroups per compute unit
  dim3 norm_apply_grid(int Cpad) const {
    const int64_t Bn = p.R / ((int64_t)p.H * p.Wd), HW = (int64_t)p.H * p.Wd;
    const int rpi = instnorm_apply_threads(Cpad) / std::min(Cpad / 8, 256);
    const int64_t want = std::max<int64_t>(1, (8 * (int64_t)device_compute_units() + Bn - 1) / Bn);
    return dim3((unsigned)std::max<int64_t>(1, std::min<int64_t>(want, (HW + rpi - 1) / rpi)), (unsigned)std::min<int64_t>(Bn, 65535));
  }
  void parabolic_eval(const uint16_t* z, int j, int jb, Ctl* c) {
    const Layer& y = p.layers[0];
    uint16_t* r = u16(p.ACT[0]) + (size_t)jb * p.R * y.Npad;
    uint16_t* nrm = u16(p.ACT[1]) + (size_t)jb * p.R * y.Npad;
    GemmNT g{};
    g.A = z; g.lda = y.Kpad; g.W = u16(y.Wp); g.ldw = y.ldw; g.C = r; g.ldc = y.Npad;
    g.M = (int)p.R; g.N = y.Npad; g.K = y.ldw; g.bias = f32(y.bias_f); g.act_tanh = 2; g.ctl = c;
    g.H = p.H; g.Wd = p.Wd; g.Cpad = y.Kpad;
    launch_nt(g);
    norm_stats(r, nullptr, norm_stat_of(jb), false, c);
    NormApply a{};
    a.X = r; a.Out = nrm; a.ld = y.Npad; a.Cpad = y.Npad; a.HW = (int64_t)p.H * p.Wd; a.rows = p.R;
    a.stat = norm_stat_of(jb); a.ctl = c;
    instnorm_apply<T, false><<<norm_apply_grid(y.Npad), instnorm_apply_threads(y.Npad), 0, st>>>(a);
    GemmNT t{};
    t.A = nrm; t.lda = y.Npad; t.W = u16(y.WTp); t.ldw = 9 * y.Npad; t.C = u16(p.K) + (size_t)j * p.stage_stride; t.ldc = y.Kpad;
    t.M = (int)p.R; t.N = y.Kpad; t.K = t.ldw; t.negate = 1; t.ctl = c; t.H = p.H; t.Wd = p.Wd; t.Cpad = y.Npad;
    launch_nt(t);
  }
  // cotangent chain of stage j through the block: kbar -> dn -> du -> zbar (eq. (vjp))
  void parabolic_vjp(const uint16_t* kbar, int j, int detect) {
    const Layer& y = p.layers[0];
    const size_t so = (size_t)j * p.R * y.Npad;
    uint16_t* dn = u16(p.DELTA[0]) + so;
    uint16_t* du = u16(p.DELTA[1]) + so;
    GemmNT g{};
    g.A = kbar; g.lda = y.Kpad; g.W = u16(y.Wp); g.ldw = y.ldw; g.C = dn; g.ldc = y.Npad;
    g.M = (int)p.R; g.N = y.Npad; g.K = y.ldw; g.negate = 1; g.ctl = ctl; g.detect = detect;
    g.H = p.H; g.Wd = p.Wd; g.Cpad = y.Kpad;
    launch_nt(g);
    norm_stats(dn, u16(p.ACT[1]) + so, f32(p.nstat_vjp), true, ctl);
    NormApply a{};
    a.X = dn; a.Nrm = u16(p.ACT[1]) + so; a.Rl = u16(p.ACT[0]) + so; a.Out = du; a.ld = y.Npad; a.Cpad = y.Npad;
    a.HW = (int64_t)p.H * p.Wd; a.rows = p.R; a.stat = norm_stat_of(j); a.stat_vjp = f32(p.nstat_vjp); a.ctl = ctl;
    a.detect = detect;
    instnorm_apply<T, true><<<norm_apply_grid(y.Npad), instnorm_apply_threads(y.Npad), 0, st>>>(a);
    GemmNT t{};
    t.A = du; t.lda = y.Npad; t.W = u16(y.WTp); t.ldw = 9 * y.Npad; t.C = u16(p.ZBAR) + (size_t)j * p.stage_stride; t.ldc = y.Kpad;
    t.M = (int)p.R; t.N = y.Kpad; t.K = t.ldw; t.ctl = ctl; t.detect = detect; t.H = p.H; t.Wd = p.Wd; t.Cpad = y.Npad;
    launch_nt(t);
  }
  // piece of the piecewise-constant parameters that step i uses
  int piece_of(int i, int N) const { return (int)(((int64_t)i * p.n_intervals) / N); }

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
      if (vec8())
        stage_input_v8<T><<<stream_blocks(p.R * (p.dpad / 8)), 256, 0, st>>>(ck, p.d, u16(p.K), p.stage_stride, j, arow,
                                                                            h, z, p.dpad, p.R, c);
      else
        stage_input<T><<<blocks_for(p.R * p.dpad, 256), 256, 0, st>>>(ck, p.d, u16(p.K), p.stage_stride, j, arow, h, z,
                                                                     p.dpad, p.R, c);
      const float tau = round_low_host((float)(t_i + tab->c[j] * (double)h), low);
      if (taus_out) taus_out[j] = tau;
      const uint16_t* in = z;
      if (p.parabolic) {
        parabolic_eval(z, j, jb, c);
        continue;
      }
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
      if (p.cnf)  // dl/dt = -tr(dv/dz) into the l column of the slope
        cnf_trace_row<T><<<blocks_for(p.R, 4), 256, 0, st>>>(u16(p.ACT[0]) + (size_t)jb * p.R * p.layers[0].Npad,
                                                             p.layers[0].Npad, f32(p.cnf_c), p.R,
                                                             u16(p.K) + (size_t)j * p.stage_stride, p.dpad, p.d - 1, c);
    }
  }

  // streaming kernels: 8-wide variants when the state width allows 16-byte accesses
  bool vec8() const { return (p.d & 7) == 0; }
  static unsigned stream_blocks(int64_t groups, int64_t cap = 4096) {  // grid-stride loops
    const int64_t b = (groups + 255) / 256;
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>(b, cap));
  }

  // ------------------------------------------------ row-tile-persistent path (dense networks)
  bool use_fused = false;

  void cast_fragments(const float* theta) {
    CastArgs c{};
    c.L = p.L;
    int nfrag = 0;
    for (int l = 0; l < p.L; ++l) {
      const Layer& y = p.layers[l];
      CastLayer& d = c.layer[l];
      d.W = theta + y.theta_w;
      d.b = theta + y.theta_b;
      d.Wf = (u16x8*)(ws + y.Wf);
      d.WTf = (u16x8*)(ws + y.WTf);
      d.bias_f = f32(y.bias_f);
      d.wt_f = f32(y.wt_f);
      d.out = y.out; d.in = y.in; d.in_full = y.in_full; d.has_time = y.has_time;
      d.Npad = y.Npad; d.Kpad = y.Kpad;
      d.frag0 = nfrag;
      nfrag += (y.Kpad / 32) * (y.Npad / 16) + (y.Npad / 32) * (y.Kpad / 16);
    }
    c.nfrag = nfrag;
    if (p.wide)
      cast_dense_fragments_wide<T><<<blocks_for(nfrag, 4), 256, 0, st>>>(c);
    else
      cast_dense_fragments<T><<<blocks_for(nfrag, 4), 256, 0, st>>>(c);
  }

  // per step: h_i, then the stage times rounded to low precision
  void write_steptab(const double* tgrid, int N, const rampde_tableau* tab, rampde_dtype low) {
    std::vector<float> tabv((size_t)N * (1 + p.s));
    for (int i = 0; i < N; ++i) {
      const float h = (float)(tgrid[i + 1] - tgrid[i]);
      tabv[(size_t)i * (1 + p.s)] = h;
      for (int j = 0; j < p.s; ++j)
        tabv[(size_t)i * (1 + p.s) + 1 + j] = round_low_host((float)(tgrid[i] + tab->c[j] * (double)h), low);
    }
    for (size_t off = 0; off < tabv.size(); off += 768) {
      FloatChunk c;
      const int cnt = (int)std::min<size_t>(768, tabv.size() - off);
      memcpy(c.v, tabv.data() + off, sizeof(float) * cnt);
      write_floats<<<1, 256, 0, st>>>(c, f32(p.steptab) + off, cnt);
    }
  }

  FusedArgs fused_args(const rampde_tableau* tab, int N) const {
    FusedArgs a{};
    int boff = 0;
    for (int l = 0; l < p.L; ++l) {
      const Layer& y = p.layers[l];
      a.layer[l].Wf = (const u16x8*)(ws + y.Wf);
      a.layer[l].WTf = (const u16x8*)(ws + y.WTf);
      a.layer[l].bias = f32(y.bias_f);
      a.layer[l].wt = y.has_time ? f32(y.wt_f) : nullptr;
      a.layer[l].Kpad = y.Kpad;
      a.layer[l].Npad = y.Npad;
      a.layer[l].bias_off = boff;
      boff += y.Npad;
    }
    a.wt_off = p.wt_off;
    a.nparam = p.nparam;
    a.k_in_lds = p.k_in_lds ? 1 : 0;
    a.act_lds_off = p.act_lds_off;
    a.L = p.L;
    a.s = p.s;
    a.N = N;
    a.d = p.d;
    a.dpad = p.dpad;
    a.ldp = p.ldp;
    a.R = p.R;
    a.stage_stride = p.stage_stride;
    for (int i = 0; i < p.s; ++i) {
      a.b[i] = (float)tab->b[i];
      a.c[i] = (float)tab->c[i];
      for (int j = 0; j < p.s; ++j) {
        a.A[i * p.s + j] = (float)tab->A[i * p.s + j];
        if (j + 1 < i && tab->A[i * p.s + j] != 0.0) a.dense_tableau = 1;
      }
    }
    a.steptab = f32(p.steptab);
    a.K = u16(p.K);
    a.bsum = p.bsum ? f32(p.bsum) : nullptr;
    return a;
  }

  // hidden width for which a shape-specialised instantiation exists (all hidden layers padded
  // to the same width), or 0
  int static_hidden_width() const {
    if (p.L < 2) return 0;
    const int hp = p.layers[0].Npad;
    for (int l = 0; l + 1 < p.L; ++l)
      if (p.layers[l].Npad != hp) return 0;
    return (hp == 256 || hp == 512 || hp == 1024) ? hp : 0;
  }

  int launch_fused(bool adjoint, const FusedArgs& a) {
    FusedLaunch l{};
    l.adjoint = adjoint ? 1 : 0;
    l.waves = p.overlap_wgrad ? 4 : 8;
    if (p.MT == 1 && !adjoint) l.waves = 16;
    l.bf16 = std::is_same<T, BF16>::value ? 1 : 0;
    l.MT = p.MT;
    l.NTL = p.dpad / 64;
    l.grid = blocks_for(p.R, 16 * p.MT);
    l.lds_bytes = p.lds_bytes;
    l.stream = st;
    hipError_t e;
    if (p.wide) {
      e = wide_launch(l, a);
      if (e != hipSuccess) return hip_fail(e, "wide row-tile kernel launch");
      return RAMPDE_OK;
    }
    switch (static_hidden_width()) {
      case 256: e = fused_launch_hp256(l, a); break;
      case 512: e = fused_launch_hp512(l, a); break;
      case 1024: e = fused_launch_hp1024(l, a); break;
      default: e = fused_launch_hp0(l, a); break;
    }
    if (e != hipSuccess) return hip_fail(e, "row-tile-persistent kernel launch");
    return RAMPDE_OK;
  }

  double step_flops() const {  // one velocity evaluation of the whole batch, padded shapes
    double f = 0.0;
    for (const Layer& y : p.layers) f += 2.0 * (double)p.R * y.Npad * y.Kpad;
    return f;
  }

  int forward_fused(const float* theta, const float* y0, const double* tgrid, int N, const rampde_tableau* tab,
                    const rampde_policy* pol, uint16_t* ckpt, float* yN) {
    cast_fragments(theta);
    write_steptab(tgrid, N, tab, pol->low);
    FusedArgs a = fused_args(tab, N);
    a.y0 = y0;
    a.y = yN;
    a.ckpt = ckpt;
    a.round_incr = ((pol->flags & RAMPDE_ROUND_INCREMENT) ? 1 : 0) | ((pol->flags & RAMPDE_NAIVE_STATE) ? 2 : 0);
    int rc;
    {
      TimeScope ts(RAMPDE_K_FUSED_FORWARD, step_flops() * p.s * N, st);
      rc = launch_fused(false, a);
    }
    if (rc) return rc;
    HIP_TRY(hipGetLastError());
    return RAMPDE_OK;
  }

  int adjoint_step_fused(const FusedArgs& a) {
    int rc;
    {
      TimeScope ts(RAMPDE_K_FUSED_ADJOINT_STEP, step_flops() * p.s * (a.skip_recompute ? 1.0 : 2.0) * a.nsteps, st);
      rc = launch_fused(true, a);
    }
    if (rc) return rc;
    if (a.tpart) {
      // the launch's per-workgroup slots of the time-grid sums -> the per-step sums (steps a.step, a.step - 1, ...)
      const int grid = blocks_for(p.R, 16 * p.MT);
      if ((size_t)grid * a.nsteps > kTimeSlotPairs) return RAMPDE_EUNSUPPORTED;
      fold_time_slots<<<a.nsteps, 256, 0, st>>>(a.tpart, grid, f32(p.tpart), a.step, ctl);
    }
    return RAMPDE_OK;
  }

  int forward(const float* theta, const float* y0, const double* tgrid, int N, const rampde_tableau* tab,
              const rampde_policy* pol, uint16_t* ckpt, float* yN) {
    if (use_fused) return forward_fused(theta, y0, tgrid, N, tab, pol, ckpt, yN);
    if (p.conv) HIP_TRY(allow_conv_tile_lds());
    cast_weights(theta);
    const int naive = (pol->flags & RAMPDE_NAIVE_STATE) ? 1 : 0;
    const int incr_mode = ((pol->flags & RAMPDE_ROUND_INCREMENT) ? 1 : 0) | (naive ? 2 : 0);
    float* y = yN;
    if (p.conv) {
      y = f32(p.y_rows);
      to_rows(y0, y);
      init_state<T><<<blocks_for(p.n, 256), 256, 0, st>>>(y, y, ckpt, p.n, 0, naive);
    } else {
      init_state<T><<<blocks_for(p.n, 256), 256, 0, st>>>(y0, y, ckpt, p.n, 1, naive);
    }
    Coefs bw{};
    for (int j = 0; j < p.s; ++j) bw.v[j] = (float)tab->b[j];
    int piece = 0;
    for (int i = 0; i < N; ++i) {
      const float h = (float)(tgrid[i + 1] - tgrid[i]);
      const uint16_t* ck = ckpt + (size_t)i * p.n;
      if (p.parabolic && piece_of(i, N) != piece) {
        piece = piece_of(i, N);
        cast_weights(theta + (size_t)piece * p.Pblk);
      }
      stages(ck, tgrid[i], h, tab, pol->low, 0, nullptr, nullptr);
      // bytes per state element: read y (4) + s slopes (2 each) + write y (4) + write checkpoint (2)
      TimeScope ts(RAMPDE_K_COMBINE_STORE, (double)p.n * (10.0 + 2.0 * p.s), st);
      if (vec8())
        combine_store_v8<T><<<stream_blocks(p.n / 8), 256, 0, st>>>(y, u16(p.K), p.stage_stride, p.s, bw, h, incr_mode,
                                                                   ckpt + (size_t)(i + 1) * p.n, p.d, p.dpad, p.R);
      else
        combine_store<T><<<blocks_for(p.n, 256), 256, 0, st>>>(y, u16(p.K), p.stage_stride, p.s, bw, h, incr_mode,
                                                              ckpt + (size_t)(i + 1) * p.n, p.d, p.dpad, p.R);
    }
    if (p.conv) to_nchw(y, yN);
    HIP_TRY(hipGetLastError());
    return RAMPDE_OK;
  }

  // one step of the adjoint recursion: recompute, cotangent chain, decision, fp32 updates
  void backward_step(int i, const double* tgrid, const rampde_tableau* tab, const rampde_policy* pol,
                     const uint16_t* ckpt, float* a, const float* gys_i, float* grad_theta, int dynamic, int detect,
                     bool recompute, float* tpart_i) {
    const int s = p.s;
    const int naive = (pol->flags & RAMPDE_NAIVE_STATE) ? 1 : 0;
    const float h = (float)(tgrid[i + 1] - tgrid[i]);
    Coefs taus{};
    if (recompute) {
      stages(ckpt + (size_t)i * step_elems, tgrid[i], h, tab, pol->low, 1, taus.v, ctl);
    } else {
      for (int j = 0; j < s; ++j) taus.v[j] = round_low_host((float)(tgrid[i] + tab->c[j] * (double)h), pol->low);
    }
    // cotangent chain, stages in reverse
    for (int j = s - 1; j >= 0; --j) {
      Coefs acol{};
      for (int l = j + 1; l < s; ++l) acol.v[l] = (float)tab->A[l * s + j];
      uint16_t* kbar = u16(p.KBAR) + (size_t)j * p.stage_stride;
      if (vec8())
        stage_cotangent_v8<T><<<stream_blocks(p.R * (p.dpad / 8)), 256, 0, st>>>(
            a, p.d, u16(p.ZBAR), p.stage_stride, j, s, (float)tab->b[j], acol, h, kbar, p.dpad, p.R, ctl, detect);
      else
        stage_cotangent<T><<<blocks_for(p.R * p.dpad, 256), 256, 0, st>>>(a, p.d, u16(p.ZBAR), p.stage_stride, j, s,
                                                                         (float)tab->b[j], acol, h, kbar, p.dpad, p.R,
                                                                         ctl, detect);
      const uint16_t* delta = kbar;
      if (p.parabolic) {
        parabolic_vjp(kbar, j, detect);
        continue;
      }
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
          if (p.cnf) {
            g.tr_c = f32(p.cnf_c);
            g.tr_kl = kbar + (p.d - 1);
            g.tr_ld = p.dpad;
          }
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
    chain_decide<<<1, 1, 0, st>>>(ctl, i, detect);
    Coefs cs{};
    for (int j = 0; j < s; ++j) cs.v[j] = (float)tab->c[j];
    if (tpart_i) {
      // state-shaped terms of the time-grid gradient, with the adjoint as it is before this step's update
      Coefs bw{};
      CoefMat am{};
      for (int j = 0; j < s; ++j) {
        bw.v[j] = (float)tab->b[j];
        for (int l = 0; l < j; ++l) am.v[j * kMaxStages + l] = (float)tab->A[j * s + l];
      }
      const int tg_blocks = stream_blocks(p.n, 1024);
      time_grid_terms<T><<<tg_blocks, 256, 0, st>>>(a, p.d, u16(p.K), u16(p.ZBAR), p.stage_stride, s, bw,
                                                    am, h, p.dpad, p.R, ctl, f32(p.tslots));
      fold_time_slots<<<1, 256, 0, st>>>(f32(p.tslots), tg_blocks, tpart_i, 0, ctl);
    }
    // (the fp32 update of a comes before the parameter gradients, which do not read it: the stage
    // cotangents it streams are then still in the last-level cache)
    int nslots = 0;
    {
      // bytes per state element: read a (4) + s stage cotangents (2 each) + write a (4)
      TimeScope ts(RAMPDE_K_ADJOINT_UPDATE, (double)p.n * (8.0 + 2.0 * s), st);
      if (vec8()) {
        nslots = (int)stream_blocks(p.n / 8);  // (at most 4096: the size of the slot array)
        adjoint_update_v8<T><<<nslots, 256, 0, st>>>(a, p.d, u16(p.ZBAR), p.stage_stride, s, h, gys_i, p.dpad, p.R, ctl,
                                                     naive, (unsigned*)(ws + p.amax_slots));
      } else
        adjoint_update<T><<<blocks_for(p.n, 256), 256, 0, st>>>(a, p.d, u16(p.ZBAR), p.stage_stride, s, h, gys_i,
                                                               p.dpad, p.R, ctl, naive);
    }
    scale_grow<<<1, 256, 0, st>>>(ctl, f32(p.scale_hist), i, Low<T>::p_bits, dynamic,
                                  (pol->flags & RAMPDE_GROW_RAW_NORM) ? 1 : 0, (const unsigned*)(ws + p.amax_slots), nslots);
    param_grads(h, taus, grad_theta, cs, tpart_i);
  }

  // parameter gradient of one accepted step: contraction over all stages and rows at once,
  // scaled by h / S_step and accumulated in fp32 (paper Sec. 3, update of g)
  void param_grads(float h, const Coefs& taus, float* grad_theta, const Coefs& cs, float* tpart_i) {
    // (grad_theta: the gradient of the parameters this step used -- the step's piece when they are piecewise constant)
    const int s = p.s;
    const int64_t rows = (int64_t)s * p.R;
    // parabolic block: the one weight tensor gets two terms, pass 0: dW += du^T z (and db), pass 1:
    // dW -= n^T kbar (the slope -W^T n is linear in W with "input" kbar and "output cotangent" n)
    const int passes = p.parabolic ? 2 : p.L;
    for (int l = 0; l < passes; ++l) {
      const Layer& y = p.layers[p.parabolic ? 0 : l];
      GemmTN g{};
      g.A = (l == p.L - 1) ? u16(p.KBAR) : u16(p.DELTA[l]);
      g.lda = y.Npad;
      g.B = (l == 0) ? u16(p.Z) : u16(p.ACT[l - 1]);
      g.ldb = y.Kpad;
      if (p.parabolic) {
        g.A = l == 0 ? u16(p.DELTA[1]) : u16(p.ACT[1]);
        g.B = l == 0 ? u16(p.Z) : u16(p.KBAR);
        if (l == 1) h = -h;
      }
      g.rows = rows;
      if (conv_wgrad_tr_applies(p)) {
        ConvWgradTr c{};
        c.A = g.A; c.lda = g.lda; c.B = g.B; c.ldb = g.ldb;
        c.lines = rows / p.Wd;
        c.lines_per_split = y.cw_per;
        c.part = f32(y.cw_part);
        c.h = h; c.ctl = ctl; c.H = p.H;
        c.want_sums = l == 0;
        c.tiles_a = y.Npad / 128; c.tiles_b = y.Kpad / 128; c.splits = y.cw_splits;
        const int groups = c.tiles_a * c.splits;
        dim3 cgrid(8 * 3 * c.tiles_b * ((groups + 7) / 8));
        TimeScope ts(RAMPDE_K_WGRAD_GEMM, 2.0 * rows * (double)y.Npad * y.Kpad * 9, st);
        const size_t lds = conv_wgrad_tr_lds_bytes(p.Wd);
        if (p.Wd == 16) conv_wgrad_tr<T, 1><<<cgrid, 256, lds, st>>>(c);
        else if (p.Wd == 32) conv_wgrad_tr<T, 2><<<cgrid, 256, lds, st>>>(c);
        else conv_wgrad_tr<T, 4><<<cgrid, 256, lds, st>>>(c);
        continue;  // (bias gradient included)
      } else if (conv_wgrad_applies(p)) {
        // all 9 taps of a 64 x 64 channel block per workgroup
        ConvWgrad c{};
        c.A = g.A; c.lda = g.lda; c.B = g.B; c.ldb = g.ldb;
        c.rows = rows;
        c.rows_per_split = y.cw_per;
        c.part = f32(y.cw_part);
        c.h = h; c.ctl = ctl; c.H = p.H; c.Wd = p.Wd;
        c.want_sums = !(p.parabolic && l == 1);
        c.Na = y.out;
        c.R = p.R;
        for (int j = 0; j < kMaxStages; ++j) {
          c.taus[j] = j < s ? taus.v[j] : 0.f;
          c.cs[j] = j < s ? cs.v[j] : 0.f;
        }
        c.wt = y.has_time ? f32(y.wt_f) : nullptr;
        c.ldwt = y.Npad;
        c.tpart = tpart_i ? f32(p.tslots) : nullptr;
        dim3 cgrid(y.Npad / 64, y.Kpad / 64, y.cw_splits);
        TimeScope ts(RAMPDE_K_WGRAD_GEMM, 2.0 * rows * (double)y.Npad * y.Kpad * 9, st);
        const size_t lds = conv_wgrad_lds_bytes(p.Wd);
        const bool tsum = c.tpart && c.wt;
        if (conv_wgrad_tr64_applies(p, y)) {
          // 64 x 64 channels: the kernel built on transposing LDS reads (same private copies)
          const size_t l64 = conv_wgrad_tr64_lds_bytes(p.Wd);
          if (p.Wd == 16) {
            if (tsum) conv_wgrad_tr64<T, true, 1><<<cgrid, 256, l64, st>>>(c);
            else conv_wgrad_tr64<T, false, 1><<<cgrid, 256, l64, st>>>(c);
          } else if (p.Wd == 32) {
            if (tsum) conv_wgrad_tr64<T, true, 2><<<cgrid, 256, l64, st>>>(c);
            else conv_wgrad_tr64<T, false, 2><<<cgrid, 256, l64, st>>>(c);
          } else {
            if (tsum) conv_wgrad_tr64<T, true, 4><<<cgrid, 256, l64, st>>>(c);
            else conv_wgrad_tr64<T, false, 4><<<cgrid, 256, l64, st>>>(c);
          }
        } else if (p.Wd <= 32) {
          if (tsum) conv_wgrad<T, true, CW_MAXI_LO><<<cgrid, 256, lds, st>>>(c);
          else conv_wgrad<T, false, CW_MAXI_LO><<<cgrid, 256, lds, st>>>(c);
        } else {
          if (tsum) conv_wgrad<T, true, CW_MAXI_HI><<<cgrid, 256, lds, st>>>(c);
          else conv_wgrad<T, false, CW_MAXI_HI><<<cgrid, 256, lds, st>>>(c);
        }
        if (tsum) fold_time_slots<<<1, 256, 0, st>>>(f32(p.tslots), (int)(cgrid.x * cgrid.y * cgrid.z), tpart_i, 0, ctl);
        continue;  // (bias and time-channel gradients included)
      } else {
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
      }
      if (p.parabolic && l == 1) continue;
      // bias and time-weight gradients
      int rpb = (int)((rows + 255) / 256);
      if (rpb < 64) rpb = 64;
      dim3 cgrid(y.Npad / 64, blocks_for(rows, rpb));
      float* gb = grad_theta + y.theta_b;
      float* gwt = y.has_time ? grad_theta + y.theta_w + (p.conv ? (size_t)y.in * 9 : (size_t)y.in) : nullptr;
      float* tsl = tpart_i ? f32(p.tslots) : nullptr;
      if (p.conv)
        column_sums<T, true><<<cgrid, 256, 0, st>>>(g.A, y.Npad, p.R, s, y.out, taus, h, gb, gwt, y.in_full * 9, p.H,
                                                    p.Wd, rpb, ctl, y.has_time ? f32(y.wt_f) : nullptr, cs, tsl);
      else
        column_sums<T, false><<<cgrid, 256, 0, st>>>(g.A, y.Npad, p.R, s, y.out, taus, h, gb, gwt, y.in_full, p.H,
                                                     p.Wd, rpb, ctl, y.has_time ? f32(y.wt_f) : nullptr, cs, tsl);
      if (tsl && y.has_time) fold_time_slots<<<1, 256, 0, st>>>(tsl, (int)(cgrid.x * cgrid.y), tpart_i, 0, ctl);
    }
    if (p.cnf) {
      // the trace row's share of dW1 and dW2: s_h = sum over stages and rows of kbar_l (1 - a_h^2)
      const Layer &y0 = p.layers[0], &y1 = p.layers[1];
      fill_zero_u32<<<1, 256, 0, st>>>((uint32_t*)(ws + p.cnf_s), (size_t)y0.Npad);
      int rpb = (int)((rows + 255) / 256);
      if (rpb < 64) rpb = 64;
      dim3 sgrid(y0.Npad / 64, blocks_for(rows, rpb));
      cnf_trace_sums<T><<<sgrid, 256, 0, st>>>(u16(p.ACT[0]), y0.Npad, u16(p.KBAR), p.dpad, p.d - 1, rows, rpb, f32(p.cnf_s), ctl);
      cnf_trace_grad<T><<<blocks_for((int64_t)y0.out * y0.in, 256), 256, 0, st>>>(
          f32(p.cnf_s), u16(y0.Wp), y0.Kpad, u16(y1.Wp), y1.Kpad, y0.in, y0.out, h, ctl, grad_theta + y0.theta_w, y0.in_full,
          grad_theta + y1.theta_w, y1.in_full);
    }
  }

  // parameter gradients from the feature-major buffers of the row-tile-persistent adjoint kernel
  // nsteps = 0: the one step `step`, h and taus as given; nsteps >= 1 (groups of steps): steps step,
  // step - 1, ..., step - nsteps + 1 in one launch, h and taus from the step table
  void param_grads_fused(int step, float h, const Coefs& taus, hipStream_t stream, int nsteps = 0) {
    float* grad_theta = f32(p.gpart);  // copy 0; chunk c adds into copy c
    // (the kernels that take several steps per launch find a step's buffer set themselves)
    const size_t set = (nsteps > 0 || p.wgrad_slab) ? 0 : (size_t)(step % p.nsets) * p.fm_stride;
    WgradArgs w{};
    w.L = p.L;
    w.ksplits = p.ksplits;
    w.kchunk = p.kchunk;
    w.P = p.P;
    w.ldk = p.ldk;
    w.Rp = p.Rp;
    w.s = p.s;
    for (int j = 0; j < kMaxStages; ++j) w.taus[j] = j < p.s ? taus.v[j] : 0.f;
    w.h = h;
    w.scale_hist = f32(p.scale_hist);
    w.step = step;
    w.nsteps = nsteps;
    w.nsets = p.nsets;
    w.set_stride = (int64_t)(p.fm_stride / 2);
    w.steptab = f32(p.steptab);
    int blk = 0;
    double flops = 0.0;
    for (int l = 0; l < p.L; ++l) {
      const Layer& y = p.layers[l];
      WgradLayer& d = w.layer[l];
      d.DT = (l == p.L - 1) ? u16(p.KBART + set) : u16(p.DELTAT[l] + set);
      d.AT = (l == 0) ? u16(p.ZT + set) : u16(p.ACTT[l - 1] + set);
      d.G = grad_theta + y.theta_w;
      d.gb = grad_theta + y.theta_b;
      d.gwt = y.has_time ? grad_theta + y.theta_w + y.in : nullptr;
      d.ldg = y.in_full;
      d.Na = y.out;
      d.Nb = y.in;
      d.NaPad = y.Npad;
      d.NbPad = y.Kpad;
      d.tiles_a = (y.Npad + 127) / 128;
      d.tiles_b = (y.Kpad + 127) / 128;
      d.tile0 = blk;
      blk += d.tiles_a * d.tiles_b;
      flops += 2.0 * (double)p.ldk * y.Npad * y.Kpad * std::max(1, nsteps);
    }
    w.ntiles = blk;
    if (p.wgrad_slab) {
      SlabArgs sa{};
      sa.w = w;
      sa.w.nsteps = std::max(1, nsteps);
      blk = 0;
      for (int l = 0; l < p.L; ++l) {
        WgradLayer& d = sa.w.layer[l];
        const SlabShape sh = slab_shape(d.NaPad, d.NbPad);
        sa.shape[l] = sh;
        d.tiles_a = (d.NaPad + slab_tile_a(sh) - 1) / slab_tile_a(sh);
        d.tiles_b = (d.NbPad + slab_tile_b(sh) - 1) / slab_tile_b(sh);
        d.tile0 = blk;
        blk += d.tiles_a * d.tiles_b;
      }
      sa.w.ntiles = blk;
      const int grid = (blk * w.ksplits + 7) / 8 * 8;
      TimeScope ts(RAMPDE_K_WGRAD_GEMM, flops, stream);
      if (sa.w.nsteps > 1)
        wgrad_slab<T, true><<<grid, 256, kSlabLdsBytes, stream>>>(sa);
      else
        wgrad_slab<T, false><<<grid, 256, kSlabLdsBytes, stream>>>(sa);
      return;
    }
    const int grid = (blk * w.ksplits + 7) / 8 * 8;  // a multiple of the XCD count: see the kernel's block mapping
    TimeScope ts(RAMPDE_K_WGRAD_GEMM, flops, stream);
    if (nsteps > 0)
      wgrad_feature_major_steps<T><<<grid, 256, 0, stream>>>(w);
    else
      wgrad_feature_major<T><<<grid, 256, 0, stream>>>(w);
  }

  int backward(const float* theta, const double* tgrid, int N, const rampde_tableau* tab, const rampde_policy* pol,
               rampde_scaling scaling, const uint16_t* ckpt, const float* grad_yN, const float* grad_ys,
               float* grad_y0, float* grad_theta, float* grad_t, float* scale_hist, rampde_stats* stats) {
    const int dynamic = scaling == RAMPDE_SCALE_DYNAMIC;
    if (grad_t) fill_zero_u32<<<1, 256, 0, st>>>((uint32_t*)(ws + p.tpart), 2 * (size_t)N);
    if (grad_t) fill_zero_u32<<<256, 256, 0, st>>>((uint32_t*)(ws + p.tslots), 2 * kTimeSlotPairs);
    const int detect = dynamic || scaling == RAMPDE_SCALE_NONE_SAFE;
    const int k_max = pol->k_max > 0 ? pol->k_max : 16;
    const int HW = p.H * p.Wd;
    if (p.conv) HIP_TRY(allow_conv_tile_lds());
    if (p.wgrad_slab)  // (its ring of operand slabs takes most of a CU's LDS)
      for (const void* f : {reinterpret_cast<const void*>(&wgrad_slab<T, false>), reinterpret_cast<const void*>(&wgrad_slab<T, true>)})
        HIP_TRY(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kSlabLdsBytes));
    if (conv_wgrad_tr_applies(p)) {
      for (const void* f : {reinterpret_cast<const void*>(&conv_wgrad_tr<T, 1>), reinterpret_cast<const void*>(&conv_wgrad_tr<T, 2>),
                            reinterpret_cast<const void*>(&conv_wgrad_tr<T, 4>)})
        HIP_TRY(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)conv_wgrad_tr_lds_bytes(64)));
    } else if (conv_wgrad_applies(p)) {
      if (conv_wgrad_tr64_applies(p, p.layers[0]))
        for (const void* f : {reinterpret_cast<const void*>(&conv_wgrad_tr64<T, false, 1>), reinterpret_cast<const void*>(&conv_wgrad_tr64<T, true, 1>),
                              reinterpret_cast<const void*>(&conv_wgrad_tr64<T, false, 2>), reinterpret_cast<const void*>(&conv_wgrad_tr64<T, true, 2>),
                              reinterpret_cast<const void*>(&conv_wgrad_tr64<T, false, 4>), reinterpret_cast<const void*>(&conv_wgrad_tr64<T, true, 4>)})
          HIP_TRY(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)conv_wgrad_tr64_lds_bytes(16)));
      const int lds = (int)conv_wgrad_lds_bytes(p.Wd);
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad<T, false, CW_MAXI_LO>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds));
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad<T, true, CW_MAXI_LO>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds));
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad<T, false, CW_MAXI_HI>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds));
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad<T, true, CW_MAXI_HI>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    }
    ctl_reset<<<1, 1, 0, st>>>(ctl, f32(p.scale_hist), N);
    if (conv_wgrad_applies(p))
      for (auto& y : p.layers)
        if (y.cw_floats) fill_zero_u32<<<1024, 256, 0, st>>>((uint32_t*)(ws + y.cw_part), y.cw_floats);
    // piecewise-constant parameters: the piece whose rounded weights are in the workspace and whose
    // private gradient copies are being filled (-1: none yet)
    int piece = -1;
    auto flush_piece = [&](int q) {
      // fold the private copies into the piece's gradient, then clear them -- both skipped once a chain
      // has been rejected, so that the retry continues on the sums of the piece's accepted steps
      if (!conv_wgrad_applies(p)) return;
      const Layer& y = p.layers[0];
      float* gq = grad_theta + (size_t)q * p.Pblk;
      const int64_t n = (int64_t)y.out * y.in * 9 + (int64_t)y.out * 10;
      if (conv_wgrad_tr_applies(p))
        conv_wgrad_tr_reduce<<<blocks_for(n, 256), 256, 0, st>>>(gq + y.theta_w, y.in_full * 9, f32(y.cw_part), y.cw_splits,
                                                                 y.Npad / 128, y.Kpad / 128, y.out, y.in, gq + y.theta_b, ctl);
      else
        conv_wgrad_reduce<<<blocks_for(n, 256), 256, 0, st>>>(gq + y.theta_w, y.in_full * 9, f32(y.cw_part), y.cw_splits,
                                                              y.Npad / 64, y.Kpad / 64, y.out, y.in, gq + y.theta_b, nullptr,
                                                              y.in_full * 9, ctl);
      fill_zero_unless_poisoned<<<1024, 256, 0, st>>>((uint32_t*)(ws + y.cw_part), y.cw_floats, ctl);
    };
    if (!use_fused && !p.parabolic) cast_weights(theta);
    SideStream& side = SideStream::get();
    if (use_fused && p.overlap_wgrad) {
      int rc = side.prepare(N);
      if (rc) return rc;
    }
    // fused path: the adjoint alternates between two buffers so that a step whose chain
    // overflowed leaves its input adjoint intact; step 0 writes grad_y0
    auto a_buf = [&](int i) -> float* { return (i % 2 == 0) ? grad_y0 : f32(p.a_alt); };
    FusedArgs fa{};
    if (use_fused) {
      cast_fragments(theta);
      write_steptab(tgrid, N, tab, pol->low);
      fa = fused_args(tab, N);
      fa.ckpt = const_cast<uint16_t*>(ckpt);
      fa.ckpt_stride = step_elems;
      fa.ldk = p.ldk;
      fa.Rp = p.Rp;
      fa.ZBAR = u16(p.ZBAR);
      for (int l = 0; l + 1 < p.L; ++l) {
        fa.ACTT[l] = u16(p.ACTT[l]);
        fa.DELTAT[l] = u16(p.DELTAT[l]);
      }
      fa.ZT = u16(p.ZT);
      fa.KBART = u16(p.KBART);
      fa.nsets = p.nsets;
      fa.set_stride = (int64_t)(p.fm_stride / 2);
      fa.nsteps = 1;
      fa.tpart = grad_t ? f32(p.tslots) : nullptr;
      fa.round_incr = (pol->flags & RAMPDE_NAIVE_STATE) ? 2 : 0;
      fill_zero_u32<<<1024, 256, 0, st>>>((uint32_t*)(ws + p.gpart), (size_t)p.ksplits * p.P);
      if (p.Rp != p.R) {
        // rows R..Rp of every stage are padding of the contraction: they must read as zero
        fill_zero_u32<<<1024, 256, 0, st>>>((uint32_t*)(ws + p.ZT), (size_t)p.nsets * p.fm_stride / 4);
      }
      fa.ctl = ctl;
      fa.scale_hist = f32(p.scale_hist);
      fa.detect = detect;
      fa.dynamic = dynamic;
      fa.raw_norm = (pol->flags & RAMPDE_GROW_RAW_NORM) ? 1 : 0;
    }
    float* a = use_fused ? a_buf(N) : grad_y0;
    const int naive_low = (pol->flags & RAMPDE_NAIVE_STATE) ? (std::is_same<T, BF16>::value ? 2 : 1) : 0;
    float* gys_rows = nullptr;
    auto gys_at = [&](int i) -> const float* {
      if (!grad_ys) return nullptr;
      const float* src = grad_ys + (size_t)i * step_elems;
      if (!p.conv) return src;
      to_rows(src, gys_rows);
      return gys_rows;
    };
    if (p.conv) {
      a = f32(p.a_rows);
      gys_rows = f32(p.gys_rows);
      to_rows(grad_yN, a);
      init_adjoint<<<stream_blocks(p.n, 512), 256, 0, st>>>(a, gys_at(N), a, p.n, ctl, 0, naive_low);
    } else {
      init_adjoint<<<stream_blocks(p.n, 512), 256, 0, st>>>(grad_yN, gys_at(N), a, p.n, ctl, 1, naive_low);
    }
    scale_init<<<1, 1, 0, st>>>(ctl, f32(p.scale_hist), N, Low<T>::p_bits, dynamic, detect);

    Ctl hctl;
    memset(&hctl, 0, sizeof hctl);
    int from = N - 1;
    bool recompute_first = true;
    int status = RAMPDE_OK;
    const bool must_sync = detect || stats || scale_hist;
    for (;;) {
      if (use_fused && p.step_group > 1) {
        // groups of steps: one adjoint launch and one parameter-gradient launch per group, all on
        // the caller's stream; the adjoint ping-pongs between two buffers per launch so that the
        // last launch writes grad_y0
        const int groups = (N + p.step_group - 1) / p.step_group;
        int hi = N - 1;
        const float* cur = a_buf(N);
        for (int gi = 0; gi < groups; ++gi) {
          const int n = std::min(p.step_group, hi + 1);
          fa.step = hi;
          fa.nsteps = n;
          fa.a_in = cur;
          fa.a_out = ((groups - 1 - gi) % 2 == 0) ? grad_y0 : f32(p.a_alt);
          cur = fa.a_out;
          fa.gys = gys_at(hi);
          fa.gys_stride = step_elems;
          fa.skip_recompute = 0;
          int rc = adjoint_step_fused(fa);
          if (rc) return rc;
          param_grads_fused(hi, 0.f, Coefs{}, st, n);
          hi -= n;
        }
      }
      int pending_hi = -1, pending_n = 0;  // steps whose parameter gradients wait for their group's launch
      for (int i = (use_fused && p.step_group > 1) ? -1 : from; i >= 0; --i) {
        if (use_fused) {
          // this set was last read by the parameter-gradient kernel of step i + 2
          if (p.overlap_wgrad && i + 2 <= N - 1) HIP_TRY(hipStreamWaitEvent(st, side.wgrad_done(i + 2), 0));
          fa.step = i;
          fa.nsteps = 1;
          fa.a_in = a_buf(i + 1);
          fa.a_out = a_buf(i);
          fa.gys = gys_at(i);
          // (with the time-grid gradient the step's slopes are needed again: they are recomputed)
          fa.skip_recompute = (i == from && !recompute_first && !grad_t) ? 1 : 0;
          int rc = adjoint_step_fused(fa);
          if (rc) return rc;
          const float h = (float)(tgrid[i + 1] - tgrid[i]);
          Coefs taus{};
          for (int j = 0; j < p.s; ++j) taus.v[j] = round_low_host((float)(tgrid[i] + tab->c[j] * (double)h), pol->low);
          if (p.overlap_wgrad) {
            HIP_TRY(hipEventRecord(side.adjoint_done(i), st));
            HIP_TRY(hipStreamWaitEvent(side.stream, side.adjoint_done(i), 0));
            param_grads_fused(i, h, taus, side.stream);
            HIP_TRY(hipEventRecord(side.wgrad_done(i), side.stream));
          } else if (p.wgrad_slab) {
            // groups of steps per launch; a group ends early at step 0.  After a rejected chain the launch
            // that holds the rejected step takes the accepted steps before it, and the loop re-enters with
            // a group that starts at the rejected step.
            if (pending_n == 0) pending_hi = i;
            ++pending_n;
            if (pending_n == p.wgrad_group || i == 0) {
              param_grads_fused(pending_hi, 0.f, Coefs{}, st, pending_n);
              pending_n = 0;
            }
          } else {
            param_grads_fused(i, h, taus, st);
          }
        } else {
          float* g_i = grad_theta;
          if (p.parabolic) {
            const int q = piece_of(i, N);
            if (q != piece) {
              // (after a rejected chain the loop re-enters inside a piece whose copies are still being
              // filled: then only the weights are rounded again)
              if (piece >= 0 && i != from) flush_piece(piece);
              cast_weights(theta + (size_t)q * p.Pblk);
              piece = q;
            }
            g_i = grad_theta + (size_t)q * p.Pblk;
          }
          backward_step(i, tgrid, tab, pol, ckpt, a, gys_at(i), g_i, dynamic, detect,
                        i == from ? recompute_first : true, grad_t ? f32(p.tpart) + 2 * (size_t)i : nullptr);
        }
      }
      if (use_fused) {
        a = grad_y0;
        if (p.overlap_wgrad) HIP_TRY(hipStreamWaitEvent(st, side.wgrad_done(0), 0));  // helper stream is in order: joins all
        reduce_partial_gradients<<<blocks_for(p.P, 256), 256, 0, st>>>(grad_theta, f32(p.gpart), p.P, p.ksplits, ctl);
      }
      if (grad_t) fold_time_sums<<<blocks_for(N + 1, 256), 256, 0, st>>>(grad_t, f32(p.tpart), N, ctl);
      if (p.parabolic) {
        flush_piece(piece);
        piece = -1;  // (a retry starts by rounding the weights of its piece again)
      } else if (conv_wgrad_applies(p))
        for (auto& y : p.layers) {
          const int64_t n = (int64_t)y.out * y.in * 9 + (int64_t)y.out * 10;
          conv_wgrad_reduce<<<blocks_for(n, 256), 256, 0, st>>>(
              grad_theta + y.theta_w, y.in_full * 9, f32(y.cw_part), y.cw_splits, y.Npad / 64, y.Kpad / 64, y.out, y.in,
              grad_theta + y.theta_b, y.has_time ? grad_theta + y.theta_w + (size_t)y.in * 9 : nullptr, y.in_full * 9, ctl);
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
      if (grad_t) fill_zero_u32<<<1, 64, 0, st>>>((uint32_t*)(ws + p.tpart) + 2 * (size_t)from, 2);
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
    if (p.conv) to_nchw(a, grad_y0);
    HIP_TRY(hipGetLastError());
    std::vector<float> hist;
    if (scale_hist || stats) {
      hist.resize((size_t)N + 1);
      HIP_TRY(hipMemcpyAsync(hist.data(), f32(p.scale_hist), sizeof(float) * (size_t)(N + 1), hipMemcpyDeviceToHost, st));
    }
    if (must_sync) HIP_TRY(hipStreamSynchronize(st));
    if (scale_hist) memcpy(scale_hist, hist.data(), sizeof(float) * (size_t)(N + 1));
    if (stats) {
      stats->status = st_code;
      stats->failed_step = hctl.poison ? hctl.failed_step : -1;
      stats->retries = hctl.retries;
      stats->s_min = hctl.s_min;
      stats->s_max = hctl.s_max;
      stats->s_first = hist[N];
      stats->s_last = hist[0];
    }
    return status;
  }
};

static rampde_scaling resolve_scaling(const rampde_policy* pol) {
  if (pol->scaling != RAMPDE_SCALE_AUTO) return pol->scaling;
  return pol->low == RAMPDE_F16 ? RAMPDE_SCALE_DYNAMIC : RAMPDE_SCALE_NONE;
}

// ---------------------------------------------------------------- scratch of the entry point that allocates nothing
// rampde_odeint_fwd_static keeps what rampde_odeint_fwd keeps in the caller's workspace (rounded weight
// fragments, stage values, slopes, running sums) in this array.  Every GPU the library runs on holds its
// own copy, at its own address, until the process ends.  In host code the array's NAME is only a handle
// for hipGetSymbolAddress: the device address is looked up once per device and kept below, and only
// that address is ever handed to kernels.
constexpr size_t kStaticScratchBytes = RAMPDE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};

static int static_scratch(void** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return RAMPDE_EUNSUPPORTED;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || ((uintptr_t)ptr & 255)) return RAMPDE_EWORKSPACE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return RAMPDE_OK;
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
  if (is_backward && pol && pol->scale_group > 0 && pol->scale_group < B) {
    // the backward pass runs scale group by scale group on the same workspace: room for the largest
    // (the groups have scale_group samples, the last one the remainder)
    rampde_policy one = *pol;
    one.scale_group = 0;
    const size_t full = rampde_workspace_bytes(vel, pol->scale_group, N, tab, &one, 1);
    const int64_t tail = B % pol->scale_group;
    const size_t rest = tail ? rampde_workspace_bytes(vel, tail, N, tab, &one, 1) : 1;
    return (full && rest) ? std::max(full, rest) : 0;
  }
  Plan p = make_plan(vel, B, N, tab, pol, is_backward);
  if (!p.ok) return 0;
  size_t total = p.total;
  if (is_backward && p.wide) {
    // the backward pass with the time-grid gradient uses the other row-tile kernels: room for either
    Plan q = make_plan(vel, B, N, tab, pol, is_backward, false);
    if (q.ok) total = std::max(total, q.total);
  }
  return total;
}

int rampde_odeint_fwd(const rampde_velocity* vel, const float* theta, const float* y0, int64_t B,
                      const double* tgrid, int N, const rampde_tableau* tab, const rampde_policy* pol, void* ckpt,
                      float* yN, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(vel, tgrid, N, tab, pol);
  if (rc) return rc;
  if (!theta || !y0 || !ckpt || !yN || !workspace || B < 1) return RAMPDE_EINVAL;
  if (!aligned16(theta) || !aligned16(y0) || !aligned16(ckpt) || !aligned16(yN)) return RAMPDE_EINVAL;
  Plan p = make_plan(vel, B, N, tab, pol, 0);
  if (!p.ok) return RAMPDE_EINVAL;
  if (workspace_bytes < p.total || ((uintptr_t)workspace & 255)) return RAMPDE_EWORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool fused = p.fused;
  if (pol->low == RAMPDE_F16) {
    Runner<F16> r(p, workspace, st);
    r.use_fused = fused;
    return r.forward(theta, y0, tgrid, N, tab, pol, (uint16_t*)ckpt, yN);
  }
  Runner<BF16> r(p, workspace, st);
  r.use_fused = fused;
  return r.forward(theta, y0, tgrid, N, tab, pol, (uint16_t*)ckpt, yN);
}

int rampde_odeint_fwd_static(const rampde_velocity* vel, const float* theta, const float* y0, int64_t B,
                             const double* tgrid, int N, const rampde_tableau* tab, const rampde_policy* pol,
                             void* ckpt, float* yN, void* hip_stream) {
  // size check first, on the host: nothing is launched for a problem the array cannot hold
  int rc = check_common(vel, tgrid, N, tab, pol);
  if (rc) return rc;
  if (B < 1) return RAMPDE_EINVAL;
  const Plan p = make_plan(vel, B, N, tab, pol, 0);
  if (!p.ok) return RAMPDE_EINVAL;
  if (p.total > kStaticScratchBytes) return RAMPDE_EWORKSPACE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // the timing facility creates events: not in a call that promises to allocate nothing
  const bool timing = g_timing;
  g_timing = false;
  rc = rampde_odeint_fwd(vel, theta, y0, B, tgrid, N, tab, pol, ckpt, yN, ws, kStaticScratchBytes, hip_stream);
  g_timing = timing;
  return rc;
}

int rampde_odeint_bwd(const rampde_velocity* vel, const float* theta, int64_t B, const double* tgrid, int N,
                      const rampde_tableau* tab, const rampde_policy* pol, const void* ckpt, const float* grad_yN,
                      const float* grad_ys, float* grad_y0, float* grad_theta, float* scale_hist,
                      rampde_stats* stats, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return rampde_odeint_bwd_tgrid(vel, theta, B, tgrid, N, tab, pol, ckpt, grad_yN, grad_ys, grad_y0, grad_theta, nullptr,
                                 scale_hist, stats, workspace, workspace_bytes, hip_stream);
}

// one backward pass over rows that are the whole batch or one scale group of it
static int backward_rows(const rampde_velocity* vel, const float* theta, int64_t B, int64_t step_elems,
                         const double* tgrid, int N, const rampde_tableau* tab, const rampde_policy* pol,
                         const void* ckpt, const float* grad_yN, const float* grad_ys, float* grad_y0,
                         float* grad_theta, float* grad_t, float* scale_hist, rampde_stats* stats, void* workspace,
                         size_t workspace_bytes, hipStream_t st) {
  Plan p = make_plan(vel, B, N, tab, pol, 1, grad_t == nullptr);
  if (!p.ok) return RAMPDE_EINVAL;
  if (workspace_bytes < p.total || ((uintptr_t)workspace & 255)) return RAMPDE_EWORKSPACE;
  const rampde_scaling sc = resolve_scaling(pol);
  const bool fused = p.fused;
  if (pol->low == RAMPDE_F16) {
    Runner<F16> r(p, workspace, st);
    r.use_fused = fused;
    if (step_elems) r.step_elems = step_elems;
    return r.backward(theta, tgrid, N, tab, pol, sc, (const uint16_t*)ckpt, grad_yN, grad_ys, grad_y0, grad_theta,
                      grad_t, scale_hist, stats);
  }
  Runner<BF16> r(p, workspace, st);
  r.use_fused = fused;
  if (step_elems) r.step_elems = step_elems;
  return r.backward(theta, tgrid, N, tab, pol, sc, (const uint16_t*)ckpt, grad_yN, grad_ys, grad_y0, grad_theta,
                    grad_t, scale_hist, stats);
}

int rampde_odeint_bwd_tgrid(const rampde_velocity* vel, const float* theta, int64_t B, const double* tgrid, int N,
                            const rampde_tableau* tab, const rampde_policy* pol, const void* ckpt,
                            const float* grad_yN, const float* grad_ys, float* grad_y0, float* grad_theta,
                            float* grad_t, float* scale_hist, rampde_stats* stats, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(vel, tgrid, N, tab, pol);
  if (rc) return rc;
  if (!theta || !ckpt || !grad_yN || !grad_y0 || !grad_theta || !workspace || B < 1) return RAMPDE_EINVAL;
  if (pol->scale_group < 0) return RAMPDE_EINVAL;
  // (the parabolic block has no time input and step-wise constant parameters: no time-grid gradient is formed)
  if (grad_t && vel->kind == RAMPDE_VEL_PARABOLIC) return RAMPDE_EUNSUPPORTED;
  if (!aligned16(theta) || !aligned16(ckpt) || !aligned16(grad_yN) || !aligned16(grad_ys) || !aligned16(grad_y0) ||
      !aligned16(grad_theta))
    return RAMPDE_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t G = pol->scale_group;
  if (G == 0 || G >= B)
    return backward_rows(vel, theta, B, 0, tgrid, N, tab, pol, ckpt, grad_yN, grad_ys, grad_y0, grad_theta, grad_t,
                         scale_hist, stats, workspace, workspace_bytes, st);

  // Scale groups (the batch-size-one setting of Alg. 2 carried over to a batch: G consecutive samples
  // share one scale; each group has its own initial scale, overflow retries and growth, and its share
  // of dL/dtheta is unscaled with its own h / S before it is added to the others').  The groups are
  // independent adjoint problems that share theta: they run one after the other on the caller's
  // stream and workspace, each on its slice of the caller's buffers.
  rampde_policy one = *pol;
  one.scale_group = 0;
  Plan whole = make_plan(vel, B, N, tab, &one, 1, grad_t == nullptr);
  if (!whole.ok) return RAMPDE_EINVAL;
  const int64_t per_sample = whole.n / B;
  const int64_t step_elems = whole.n;
  if ((G * per_sample) % 8) return RAMPDE_EINVAL;  // every group's slice must start 16-byte aligned
  const size_t low_bytes = 2;
  rampde_stats all{};
  all.failed_step = -1;
  bool any_overflow = false;
  // (the unscaled-safe variant reads its outcome back in any case: no extra synchronisation)
  const bool want_stats = stats || resolve_scaling(pol) == RAMPDE_SCALE_NONE_SAFE;
  int group = 0;
  for (int64_t b0 = 0; b0 < B; b0 += G, ++group) {
    const int64_t Bg = std::min<int64_t>(G, B - b0);
    const int64_t off = b0 * per_sample;
    rampde_stats gs{};
    rc = backward_rows(vel, theta, Bg, step_elems, tgrid, N, tab, &one, (const char*)ckpt + (size_t)off * low_bytes,
                       grad_yN + off, grad_ys ? grad_ys + off : nullptr, grad_y0 + off, grad_theta, grad_t,
                       scale_hist ? scale_hist + (size_t)group * (N + 1) : nullptr, want_stats ? &gs : nullptr, workspace,
                       workspace_bytes, st);
    if (stats) {
      if (group == 0) {
        all = gs;
      } else {
        all.retries += gs.retries;
        all.s_min = std::min(all.s_min, gs.s_min);
        all.s_max = std::max(all.s_max, gs.s_max);
        if (gs.status > all.status) {
          all.status = gs.status;
          all.failed_step = gs.failed_step;
        }
      }
      *stats = all;
    }
    if (rc) return rc;
    if (want_stats && gs.status == 1) any_overflow = true;
  }
  if (any_overflow) {
    // unscaled-safe variant: an overflow anywhere leaves +inf everywhere (the group's own pass has
    // filled dL/dtheta and its own rows of dL/dy_0)
    fill_u32<<<1024, 256, 0, st>>>((uint32_t*)grad_y0, (size_t)whole.n, 0x7f800000u);
    HIP_TRY(hipGetLastError());
  }
  return RAMPDE_OK;
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
