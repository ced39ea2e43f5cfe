// Row-tile-persistent kernels for dense (MLP) velocity networks.
//
// Samples are independent in the forward recursion (paper Algorithm 1) and in the cotangent
// chain of the adjoint (paper Algorithm 2, eq. (vjp)); only the parameter gradient and the
// adjoint scale couple them.  So one workgroup owns TM = 16 * MT batch rows and carries them
//   * mlp_forward_fused : through ALL time steps, stages and layers in one launch,
//   * mlp_adjoint_step  : through one step of the adjoint: stage recomputation, the whole
//                         cotangent chain, the fp32 adjoint update and the max-norm / overflow
//                         bookkeeping of the dynamic scale (the last workgroup to finish takes
//                         the accept / grow decision, so no extra launches are needed).
//
// Where things live
//   * fp32 state (y forward, a backward): in registers, in the accumulator layout of the last
//     contraction of a stage, so the Runge-Kutta combinations are lane-local;
//   * slopes k_j / stage cotangents zbar_j: low precision, in LDS when they fit (else in the
//     global workspace); every lane only ever reads back the elements it wrote itself;
//   * activations of the current layer: LDS, two ping-pong tiles plus one tile for the stage
//     input (so the epilogue of a stage's last contraction can already write the next stage's
//     input while other wavefronts still read the ping-pong tiles);
//   * biases and time-column weights: LDS (copied once per launch);
//   * weights: streamed from L2 in a pre-swizzled "fragment-major" layout straight into MFMA
//     operand registers (each wavefront reads a disjoint slice of the output columns, so
//     staging weights in LDS would not save traffic), PD k-blocks ahead and across layer
//     boundaries.
//
// MFMA shape: v_mfma_f32_16x16x32_{f16,bf16} with the WEIGHT tile as the first operand, so a
// lane ends up with 4 consecutive output columns of one row: 8-byte stores, float4 bias loads.
#pragma once
#include "common.hpp"

namespace rampde {

// LDS pointers carry their address space in the type: a generic pointer would turn every LDS
// access into a flat instruction, whose completion order is unknown to the wait-count logic, and
// every wait in the software pipeline below would become a wait for ALL outstanding loads.
#define RAMPDE_LDS __attribute__((address_space(3)))
typedef RAMPDE_LDS uint16_t lds_u16;
typedef RAMPDE_LDS float lds_f32;
typedef RAMPDE_LDS u16x8 lds_u16x8;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint2 lds_load_u2(const lds_u16* p) {
  const u32x2 v = *(const RAMPDE_LDS u32x2*)p;
  return make_uint2(v[0], v[1]);
}
__device__ inline void lds_store_u2(lds_u16* p, uint2 q) {
  u32x2 v;
  v[0] = q.x;
  v[1] = q.y;
  *(RAMPDE_LDS u32x2*)p = v;
}
__device__ inline float4 lds_load_f4(const lds_f32* p) {
  const f32x4 v = *(const RAMPDE_LDS f32x4*)p;
  return make_float4(v[0], v[1], v[2], v[3]);
}
typedef __attribute__((address_space(1))) u16x8 glb_u16x8;  // weight fragments: always global memory

constexpr int kMaxLayers = 8;
// k-blocks (of 32) of weight fragments kept in flight per wavefront.  Four, except for hidden width
// 512, where the adjoint kernel of 32-row tiles would spill registers (two then measure faster).
template <int HP>
constexpr int kPipelineDepth = (HP == 512) ? 2 : 4;

struct FusedLayer {
  const u16x8* Wf;    // forward fragments  [Kpad/32][Npad/16][64 lanes]: lane -> W[nt*16 + lane%16][kb*32 + (lane/16)*8 + 0..7]
  const u16x8* WTf;   // transposed frags   [Npad/32][Kpad/16][64 lanes]: lane -> W[nb*32 + (lane/16)*8 + 0..7][kt*16 + lane%16]
  const float* bias;  // [Npad] fp32, already rounded to low precision
  const float* wt;    // [Npad] time-column weights (layer 1 only) or null
  int Kpad, Npad;
  int bias_off;       // offset (floats) of this layer's bias in the LDS parameter block
};

struct FusedArgs {
  FusedLayer layer[kMaxLayers];
  int L, s, N, d, dpad, ldp;
  int wt_off;            // offset (floats) of the time-column weights in the LDS parameter block
  int nparam;            // floats in the LDS parameter block (multiple of 4)
  int k_in_lds;          // slopes / stage cotangents of a step are kept in LDS
  int act_lds_off;       // adjoint kernel: > 0 = offset (16-bit elements) in LDS of a copy of the step's hidden
                         // activations [s][L - 1][TM][ldp], which the tanh' factors then read instead of HBM
  int64_t R;
  int64_t stage_stride;  // R * dpad
  float A[kMaxStages * kMaxStages];
  int dense_tableau;     // some a_jl != 0 with l < j - 1 (beyond the sub-diagonal): not Euler, Heun, classic RK4
  float b[kMaxStages];
  float c[kMaxStages];
  const float* steptab;  // [N][1 + s]: h_i, tau_{i,1..s} (tau already rounded to low precision)
  // forward
  const float* y0;
  float* y;
  uint16_t* ckpt;
  int64_t ckpt_stride;   // adjoint kernels: elements from one stored state to the next (R * d, or more when
                         // the rows of this launch are a slice of a larger batch)
  int round_incr;        // bit 0: round sum_j b_j k_j to low before the fp32 add; bit 1: naive baseline,
                         // the state (y, and the adjoint a) is itself kept in low precision
  uint16_t* K;  // [s][R][dpad] slopes (used when they do not fit in LDS)
  float* bsum;  // [R][dpad] fp32 (64-row-tile kernels): running sum over the stages of b_l k_l within a step
  // one adjoint step
  int step;
  // Everything the parameter-gradient contraction reads is stored "feature-group-major":
  // element (feature f, k) at ((f / 4) * ldk + k) * 4 + f % 4, k = stage * Rp + row.  A lane's 4
  // consecutive features of one row are one 8-byte word (stores stay as cheap as row-major ones,
  // and the same word is what the tanh' factor of the transposed passes needs), while for a fixed
  // feature group k runs contiguously, which is what the contraction over k wants.
  uint16_t* ZT;                // [dpad / 4][ldk][4] stage inputs
  uint16_t* ACTT[kMaxLayers];  // [Npad_l / 4][ldk][4] hidden activations, l = 0..L-2
  uint16_t* DELTAT[kMaxLayers];// [Npad_l / 4][ldk][4] their cotangents
  uint16_t* KBART;             // [dpad / 4][ldk][4] cotangents of the slopes
  int64_t ldk, Rp;
  uint16_t* ZBAR;              // [s][R][dpad] (used when they do not fit in LDS)
  // The kernel runs steps step, step - 1, ..., step - nsteps + 1 (nsteps > 1 only when nothing is
  // decided between steps: no overflow detection, fixed scale).  The feature-group-major buffers of
  // step i are set i % nsets; the pointers above are those of set 0, sets are set_stride elements apart.
  int nsteps, nsets;
  int64_t set_stride;
  const float* a_in;
  float* a_out;
  const float* gys;            // running-cost cotangent of step `step` or null; step i - 1 lies gys_stride before step i
  int64_t gys_stride;
  Ctl* ctl;
  float* scale_hist;
  int detect, dynamic, raw_norm, skip_recompute;
  // time-grid gradient (paper Sec. 3, update lines of t'): null, or [N][2] fp32 per-step sums
  //   tpart[i][0] = (h/S)(dt - dh) - Phi^T a_{i+1},   tpart[i][1] = (h/S) dh + Phi^T a_{i+1}
  // (here: the launch's table of per-workgroup slots, [step of the launch][workgroup][2], folded into the per-step
  // sums by fold_time_slots after the launch)
  // added to by every workgroup; folded into dL/dt once the steps are accepted
  float* tpart;
};

// theta (fp32) -> fragment-major low-precision copies of all dense layers (see FusedLayer) and the
// rounded biases / time-column weights (kept as fp32 for the epilogues), in one launch.
struct CastLayer {
  const float* W;   // [out][in_full]
  const float* b;   // [out]
  u16x8* Wf;
  u16x8* WTf;
  float* bias_f;    // [Npad]
  float* wt_f;      // [Npad]
  int out, in, in_full, has_time, Npad, Kpad;
  int frag0;        // index of the layer's first fragment among all layers' fragments
};
struct CastArgs {
  CastLayer layer[kMaxLayers];
  int L, nfrag;
};

template <class T>
__global__ void cast_dense_fragments(CastArgs c) {
  const int lane = threadIdx.x & 63;
  int frag = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (frag >= c.nfrag) return;
  CastLayer y = c.layer[0];
#pragma unroll
  for (int q = 1; q < kMaxLayers; ++q)
    if (q < c.L && frag >= c.layer[q].frag0) y = c.layer[q];
  frag -= y.frag0;
  const int nfw = (y.Kpad / 32) * (y.Npad / 16);
  if (frag < nfw) {
    const int kb = frag / (y.Npad / 16), nt = frag % (y.Npad / 16);
    const int n = nt * 16 + (lane & 15), k0 = kb * 32 + (lane >> 4) * 8;
    u16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = k0 + e;
      v[e] = (n < y.out && k < y.in) ? Low<T>::from_f32(y.W[(size_t)n * y.in_full + k]) : (uint16_t)0;
    }
    y.Wf[(size_t)frag * 64 + lane] = v;
    if (kb == 0 && lane < 16) {
      y.bias_f[n] = (n < y.out) ? Low<T>::to_f32(Low<T>::from_f32(y.b[n])) : 0.f;
      y.wt_f[n] = (n < y.out && y.has_time) ? Low<T>::to_f32(Low<T>::from_f32(y.W[(size_t)n * y.in_full + y.in])) : 0.f;
    }
  } else {
    const int f = frag - nfw;
    const int nb = f / (y.Kpad / 16), kt = f % (y.Kpad / 16);
    const int k = kt * 16 + (lane & 15), n0 = nb * 32 + (lane >> 4) * 8;
    u16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int n = n0 + e;
      v[e] = (n < y.out && k < y.in) ? Low<T>::from_f32(y.W[(size_t)n * y.in_full + k]) : (uint16_t)0;
    }
    y.WTf[(size_t)f * 64 + lane] = v;
  }
}

// tanh of an fp32 pre-activation:  1 - 2 / (exp(2x) + 1)  with the hardware exp2 and reciprocal
// (exact limits +-1 for large |x|).  Absolute error about 1.5e-7 everywhere, i.e. a few fp32 ulp for
// |x| > 0.1 and a relative error that grows like 1.5e-7 / |x| towards zero: still 50 times below the
// half-spacing of fp16 (2^-12 relative) at |x| = 1e-3.  The result is rounded to 16 bits by the caller.
__device__ inline float tanh_fast(float x) {
  const float e = __builtin_amdgcn_exp2f(2.885390081777927f * x);
  return fmaf(-2.f, __builtin_amdgcn_rcpf(e + 1.f), 1.f);
}

template <class T>
__device__ inline uint2 pack4(const float (&v)[4]) {
  uint2 p;
  p.x = Low<T>::pack2(v[0], v[1]);
  p.y = Low<T>::pack2(v[2], v[3]);
  return p;
}
template <class T>
__device__ inline void unpack4(uint2 p, float (&v)[4]) {
  v[0] = Low<T>::to_f32((uint16_t)p.x);
  v[1] = Low<T>::to_f32((uint16_t)(p.x >> 16));
  v[2] = Low<T>::to_f32((uint16_t)p.y);
  v[3] = Low<T>::to_f32((uint16_t)(p.y >> 16));
}
template <class T>
__device__ inline bool any_nonfinite4(uint2 p) {
  return Low<T>::nonfinite((uint16_t)p.x) || Low<T>::nonfinite((uint16_t)(p.x >> 16)) ||
         Low<T>::nonfinite((uint16_t)p.y) || Low<T>::nonfinite((uint16_t)(p.y >> 16));
}

// 4 consecutive fp32 / 16-bit state elements of row `row`, columns c..c+3 of a [R][d] array;
// columns >= d and rows >= R read as zero and are not written.  d % 4 == 0 takes the vector path.
__device__ inline void load4f(const float* p, int64_t row, int64_t R, int c, int d, float (&v)[4]) {
  v[0] = v[1] = v[2] = v[3] = 0.f;
  if (row >= R) return;
  if ((d & 3) == 0) {
    if (c < d) {
      const float4 t = *reinterpret_cast<const float4*>(&p[(size_t)row * d + c]);
      v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (c + r < d) v[r] = p[(size_t)row * d + c + r];
  }
}
__device__ inline void store4f(float* p, int64_t row, int64_t R, int c, int d, const float (&v)[4]) {
  if (row >= R) return;
  if ((d & 3) == 0) {
    if (c < d) *reinterpret_cast<float4*>(&p[(size_t)row * d + c]) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (c + r < d) p[(size_t)row * d + c + r] = v[r];
  }
}
__device__ inline uint2 load4h(const uint16_t* p, int64_t row, int64_t R, int c, int d) {
  uint2 q = make_uint2(0u, 0u);
  if (row >= R) return q;
  if ((d & 3) == 0) {
    if (c < d) q = *reinterpret_cast<const uint2*>(&p[(size_t)row * d + c]);
  } else {
    uint32_t e[4] = {0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (c + r < d) e[r] = p[(size_t)row * d + c + r];
    q.x = e[0] | (e[1] << 16);
    q.y = e[2] | (e[3] << 16);
  }
  return q;
}
__device__ inline void store4h(uint16_t* p, int64_t row, int64_t R, int c, int d, uint2 q) {
  if (row >= R) return;
  if ((d & 3) == 0) {
    if (c < d) *reinterpret_cast<uint2*>(&p[(size_t)row * d + c]) = q;
  } else {
    const uint16_t e[4] = {(uint16_t)q.x, (uint16_t)(q.x >> 16), (uint16_t)q.y, (uint16_t)(q.y >> 16)};
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (c + r < d) p[(size_t)row * d + c + r] = e[r];
  }
}

// 4 consecutive features n..n+3 (n % 4 == 0) of contraction index k in a feature-group-major array
__device__ inline uint2* group4(uint16_t* XT, int64_t ldk, int64_t k, int n) {
  return reinterpret_cast<uint2*>(XT + ((size_t)(n >> 2) * ldk + k) * 4);
}
#define RAMPDE_STORE_G4(ptr, val) (*(ptr) = (val))

// One contraction pass of a row tile: out[TM][Ncols] = in[TM][32*KB] * Wfrag^T for the
// calling wavefront's slice of output-column tiles.
struct PassDesc {
  const glb_u16x8* Wf;
  int KB;    // k-blocks of 32
  int NT16;  // column tiles of 16 in total; a wavefront owns NT16/4 consecutive ones
};

// The weight stream of a pass is software-pipelined PD k-blocks deep.  Both functions are
// branch-free (out-of-range k-blocks are clamped to the last one and masked out of the MFMA
// by a zero activation operand) so that the number of loads in flight is known statically
// and every wait is for exactly the fragment that is consumed next.
// KBC / NTC > 0: the pass's k-blocks and column tiles are compile-time constants (kernels
// specialised for a network shape): the whole pipeline unrolls into straight-line code with
// immediate offsets.  KBC = 0: both are taken from the descriptor at run time.
template <int PD, int NTG, int RW, int KBC, int NTC>
__device__ inline void ring_preload(u16x8 (&ring)[PD][RW], const PassDesc& p, int nt0, int lane) {
  const glb_u16x8* base = p.Wf + (size_t)nt0 * 64 + lane;
  if constexpr (KBC > 0) {
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      if (u < KBC) {
#pragma unroll
        for (int nt = 0; nt < NTG; ++nt) ring[u][nt] = base[(size_t)u * NTC * 64 + nt * 64];
      }
    }
  } else {
    const size_t kstride = (size_t)p.NT16 * 64;
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      const int kb = min(u, p.KB - 1);
#pragma unroll
      for (int nt = 0; nt < NTG; ++nt) ring[u][nt] = base[kb * kstride + nt * 64];
    }
  }
}

template <class T, int PD, int MT, int NTG, int RW, int KBC, int NTC>
__device__ inline void tile_mma(f32x4 (&acc)[RW][MT], u16x8 (&ring)[PD][RW], const PassDesc& p, int nt0,
                                const lds_u16* in, int ldp, int lane) {
  static_assert(PD % 2 == 0, "activation fragments are double-buffered by k-block parity");
  const int lm = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int nt = 0; nt < NTG; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const glb_u16x8* wbase = p.Wf + (size_t)nt0 * 64 + lane;
  const lds_u16* abase = in + lm * ldp + lq * 8;
  u16x8 a[2][MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) a[0][mt] = *(const lds_u16x8*)(abase + mt * 16 * ldp);

  if constexpr (KBC > 0 && KBC <= 2 * PD) {
    // short contraction: fully unrolled
#pragma unroll
    for (int kb = 0; kb < KBC; ++kb) {
      const int u = kb % PD;
      if (kb + 1 < KBC) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          a[(kb + 1) & 1][mt] = *(const lds_u16x8*)(abase + mt * 16 * ldp + (kb + 1) * 32);
      }
#pragma unroll
      for (int nt = 0; nt < NTG; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = Low<T>::mfma16(ring[u][nt], a[kb & 1][mt], acc[nt][mt]);
      if (kb + PD < KBC) {
#pragma unroll
        for (int nt = 0; nt < NTG; ++nt) ring[u][nt] = wbase[(size_t)(kb + PD) * NTC * 64 + nt * 64];
      }
    }
  } else if constexpr (KBC > 0) {
    // long contraction (KBC a multiple of PD): a rolled steady-state loop that always refills,
    // then the last PD k-blocks without refills; no clamps, no masks
    static_assert(KBC % PD == 0 || KBC <= 2 * PD, "compile-time contraction lengths are multiples of the pipeline depth");
#pragma unroll 1
    for (int kb0 = 0; kb0 < KBC - PD; kb0 += PD) {
      const glb_u16x8* wnext = wbase + (size_t)(kb0 + PD) * NTC * 64;
      const lds_u16* an = abase + (kb0 + 1) * 32;
#pragma unroll
      for (int u = 0; u < PD; ++u) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[(u + 1) & 1][mt] = *(const lds_u16x8*)(an + mt * 16 * ldp + u * 32);
#pragma unroll
        for (int nt = 0; nt < NTG; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = Low<T>::mfma16(ring[u][nt], a[u & 1][mt], acc[nt][mt]);
#pragma unroll
        for (int nt = 0; nt < NTG; ++nt) ring[u][nt] = wnext[(size_t)u * NTC * 64 + nt * 64];
      }
    }
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      if (u + 1 < PD) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          a[(u + 1) & 1][mt] = *(const lds_u16x8*)(abase + mt * 16 * ldp + (KBC - PD + u + 1) * 32);
      }
#pragma unroll
      for (int nt = 0; nt < NTG; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = Low<T>::mfma16(ring[u][nt], a[u & 1][mt], acc[nt][mt]);
    }
  } else {
    const int kstride = p.NT16 * 64;
    const int KB = p.KB;
    const int kb_tail = ((KB + PD - 1) / PD - 1) * PD;  // first k-block of the last group of PD
    // steady state: fetch the next activation fragment, consume ring[u], refill it PD k-blocks ahead
    for (int kb0 = 0; kb0 < kb_tail; kb0 += PD) {
      const glb_u16x8* wnext = wbase + (size_t)(kb0 + PD) * kstride;
#pragma unroll
      for (int u = 0; u < PD; ++u) {
        const int kb = kb0 + u;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          a[(u + 1) & 1][mt] = *(const lds_u16x8*)(abase + mt * 16 * ldp + (kb + 1) * 32);
#pragma unroll
        for (int nt = 0; nt < NTG; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = Low<T>::mfma16(ring[u][nt], a[u & 1][mt], acc[nt][mt]);
        const int ku = min(u, KB - 1 - kb0 - PD);  // clamp to the last k-block (only in the last main group)
#pragma unroll
        for (int nt = 0; nt < NTG; ++nt) ring[u][nt] = wnext[ku * kstride + nt * 64];
      }
    }
    // drain: the last group of PD k-blocks, no refills; k-blocks past the end contribute zero
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      const int kb = kb_tail + u;
      const int ka = min(kb + 1, KB - 1);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        a[(u + 1) & 1][mt] = *(const lds_u16x8*)(abase + mt * 16 * ldp + ka * 32);
      const bool valid = kb < KB;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const u16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
        const u16x8 a_use = valid ? a[u & 1][mt] : zero;
#pragma unroll
        for (int nt = 0; nt < NTG; ++nt) acc[nt][mt] = Low<T>::mfma16(ring[u][nt], a_use, acc[nt][mt]);
      }
    }
  }
}

// Software pipeline of weight fragments + the pass drivers.  A pass calls, per owned 16x16 tile,
//   pre(n, m)                 -> uint2   before the contraction (early global loads the epilogue needs)
//   epi(acc, pf, nt, mt, n, m)           after it (nt is the tile's index within the group)
// with n = first of the lane's 4 columns and m = the lane's row within the tile of TM rows, and
//   nxt()                                between contraction and epilogue: it must preload the
//                                        first PD k-blocks of whatever pass runs next.
// The sequence of passes is static in the kernels, so there is no run-time bookkeeping of what
// the ring holds: every pass finds its first fragments already requested by its predecessor.
//
// A workgroup has NW wavefronts (4 or 8; 8 = two per SIMD, which hides the LDS / MFMA / barrier
// latencies of a single row tile).  Hidden widths are padded to multiples of 256 by the host, so
// in a hidden pass every wavefront owns a multiple of NTH = 16 / NW column tiles.  A state-shaped
// pass has 4 * NTL column tiles (NTL = dpad / 64): the first ACTIVE wavefronts own NTS each.
// HP > 0: all hidden layers have (padded) width HP, known at compile time; HP = 0: run-time widths.
template <int NTL, int NW, int HP>
struct Shape {
  static constexpr int NTH = 16 / NW;
  static constexpr int NTS = (4 * NTL >= NW) ? (4 * NTL) / NW : 1;
  static constexpr int ACTIVE = (4 * NTL >= NW) ? NW : 4 * NTL;
  static constexpr int RW = NTH > NTS ? NTH : NTS;
  // k-blocks of a contraction over the state width / over a hidden width; column tiles of a
  // hidden-shaped / state-shaped output (0 = not known at compile time)
  static constexpr int KB_S = HP > 0 ? 2 * NTL : 0;
  static constexpr int KB_H = HP / 32;
  static constexpr int NT_H = HP / 16;
  static constexpr int NT_S = HP > 0 ? 4 * NTL : 0;
};

template <class T, int MT, int NTL, int NW, int HP>
struct TileEngine {
  using Sh = Shape<NTL, NW, HP>;
  static constexpr int NTH = Sh::NTH, NTS = Sh::NTS, ACTIVE = Sh::ACTIVE, RW = Sh::RW;
  static constexpr int PD = kPipelineDepth<HP>;
  u16x8 ring[PD][RW];
  int lane, wave;

  __device__ inline bool state_wave() const { return ACTIVE == NW || wave < ACTIVE; }
  __device__ inline int state_col(int nt, int lq) const { return (wave * NTS + nt) * 16 + lq * 4; }

  // request the first PD k-blocks of group g of a hidden pass / of a state-shaped pass.
  // FROM_STATE: the pass contracts over the state width (first layer, or first transposed layer).
  template <bool FROM_STATE>
  __device__ inline void preload_hidden(const PassDesc& p, int g) {
    constexpr int KBC = FROM_STATE ? Sh::KB_S : Sh::KB_H;
    const int ntw = HP > 0 ? Sh::NT_H / NW : p.NT16 / NW;
    ring_preload<PD, NTH, RW, KBC, Sh::NT_H>(ring, p, wave * ntw + g * NTH, lane);
  }
  template <bool FROM_STATE>
  __device__ inline void preload_state(const PassDesc& p) {
    constexpr int KBC = FROM_STATE ? Sh::KB_S : Sh::KB_H;
    if (state_wave()) ring_preload<PD, NTS, RW, KBC, Sh::NT_S>(ring, p, wave * NTS, lane);
  }

  template <int NTG, int KBC, int NTC, class Pre, class Epi, class Nxt>
  __device__ inline void group(const PassDesc& p, int nt0, const lds_u16* in, int ld_in, bool sync_before_epi,
                               Pre& pre, Epi& epi, Nxt& nxt) {
    const int lm = lane & 15, lq = lane >> 4;
    uint2 pf[NTG][MT];
#pragma unroll
    for (int nt = 0; nt < NTG; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) pf[nt][mt] = pre((nt0 + nt) * 16 + lq * 4, mt * 16 + lm);
    f32x4 acc[RW][MT];
    tile_mma<T, PD, MT, NTG, RW, KBC, NTC>(acc, ring, p, nt0, in, ld_in, lane);
    nxt();
    if (sync_before_epi) __syncthreads();
#pragma unroll
    for (int nt = 0; nt < NTG; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) epi(acc[nt][mt], pf[nt][mt], nt, mt, (nt0 + nt) * 16 + lq * 4, mt * 16 + lm);
  }

  // hidden pass: groups of NTH column tiles per wavefront.  Ends with a barrier.
  template <bool FROM_STATE, class Pre, class Epi, class Nxt>
  __device__ inline void run_hidden(const PassDesc& p, const lds_u16* in, int ld_in, Pre pre, Epi epi, Nxt nxt) {
    constexpr int KBC = FROM_STATE ? Sh::KB_S : Sh::KB_H;
    const int ntw = HP > 0 ? Sh::NT_H / NW : p.NT16 / NW;
    const int groups = ntw / NTH;
#pragma unroll
    for (int g = 0; g < groups; ++g) {
      auto nx = [&]() {
        if (g + 1 < groups) preload_hidden<FROM_STATE>(p, g + 1);
        else nxt();
      };
      group<NTH, KBC, Sh::NT_H>(p, wave * ntw + g * NTH, in, ld_in, false, pre, epi, nx);
    }
    __syncthreads();
  }

  // state-shaped pass (the contraction that ends a stage): one group of NTS tiles on the ACTIVE
  // wavefronts, compile-time tile indices so that per-tile state registers can be addressed; the
  // other wavefronts only request their next fragments.  Ends with a barrier.
  template <bool FROM_STATE, class Pre, class Epi, class Nxt>
  __device__ inline void run_state(const PassDesc& p, const lds_u16* in, int ld_in, bool sync_before_epi, Pre pre,
                                   Epi epi, Nxt nxt) {
    constexpr int KBC = FROM_STATE ? Sh::KB_S : Sh::KB_H;
    if (state_wave()) {
      group<NTS, KBC, Sh::NT_S>(p, wave * NTS, in, ld_in, sync_before_epi, pre, epi, nxt);
    } else {
      nxt();
      if (sync_before_epi) __syncthreads();
    }
    __syncthreads();
  }
};

__device__ __forceinline__ PassDesc fwd_pass(const FusedArgs& g, int l) {
  return PassDesc{(const glb_u16x8*)g.layer[l].Wf, g.layer[l].Kpad / 32, g.layer[l].Npad / 16};
}
__device__ __forceinline__ PassDesc bwd_pass(const FusedArgs& g, int l) {
  return PassDesc{(const glb_u16x8*)g.layer[l].WTf, g.layer[l].Npad / 32, g.layer[l].Kpad / 16};
}

// LDS carve-up shared by both kernels.
template <int MT>
struct TileLds {
  static constexpr int TM = 16 * MT;
  lds_f32* param;   // [nparam] biases of all layers, then time-column weights
  lds_u16* zbuf;    // [TM][ldz]  stage input / stage cotangent tile
  lds_u16* buf0;    // [TM][ldp]
  lds_u16* buf1;    // [TM][ldp]
  lds_u16* kl;      // [s][TM][dpad] slopes or stage cotangents (when k_in_lds)
  lds_u16* act;     // [s][L - 1][TM][ldp] hidden activations of the step (adjoint kernel, when they fit) or null
  int ldz, ldp;
  __device__ __forceinline__ TileLds(lds_u16* smem, const FusedArgs& g) {
    param = (lds_f32*)smem;
    ldz = g.dpad + 8;
    ldp = g.ldp;
    zbuf = smem + 2 * g.nparam;
    buf0 = zbuf + TM * ldz;
    buf1 = buf0 + TM * ldp;
    kl = buf1 + TM * ldp;
    act = g.act_lds_off > 0 ? smem + g.act_lds_off : nullptr;
  }
  __device__ inline lds_u16* act_tile(int j, int l, int L) const { return act + (size_t)(j * (L - 1) + l) * TM * ldp; }
  // tile that layer / transposed pass number q (0 = first of its chain) reads and writes
  __device__ inline const lds_u16* in(int q) const { return q == 0 ? zbuf : (((q - 1) & 1) ? buf1 : buf0); }
  __device__ inline int ld_in(int q) const { return q == 0 ? ldz : ldp; }
  __device__ inline lds_u16* out(int q) const { return (q & 1) ? buf1 : buf0; }
};

// (every function that takes the kernel argument block by reference is force-inlined: an
// out-of-line call would make the compiler copy the whole block to scratch memory)
__device__ __forceinline__ void load_params(lds_f32* param, const FusedArgs& g) {
  for (int l = 0; l < g.L; ++l)
    for (int i = threadIdx.x; i < g.layer[l].Npad; i += blockDim.x) param[g.layer[l].bias_off + i] = g.layer[l].bias[i];
  for (int i = threadIdx.x; i < g.layer[0].Npad; i += blockDim.x) param[g.wt_off + i] = g.layer[0].wt ? g.layer[0].wt[i] : 0.f;
}

// Low-precision per-stage vectors of a tile (slopes, stage cotangents): LDS or global.
template <int MT>
struct StageStore {
  lds_u16* lds;    // used when in_lds
  bool in_lds;
  uint16_t* glob;
  int dpad;
  int64_t stage_stride, row0, R;
  __device__ inline void put(int j, int m, int n, uint2 q) const {
    if (in_lds) lds_store_u2(&lds[(j * 16 * MT + m) * (dpad + 8) + n], q);  // row pitch padded: no bank conflicts
    else if (row0 + m < R) *reinterpret_cast<uint2*>(&glob[(size_t)j * stage_stride + (size_t)(row0 + m) * dpad + n]) = q;
  }
  __device__ inline uint2 get(int j, int m, int n) const {
    if (in_lds) return lds_load_u2(&lds[(j * 16 * MT + m) * (dpad + 8) + n]);
    if (row0 + m < R) return *reinterpret_cast<const uint2*>(&glob[(size_t)j * stage_stride + (size_t)(row0 + m) * dpad + n]);
    return make_uint2(0u, 0u);
  }
};

// Hidden layers of one velocity evaluation (all but the last layer) for stage j.  The ring must
// hold the first fragments of layer 0 (if L > 1); on return it holds those of the last layer.
template <class T, int MT, int NTL, int NW, int HP, bool KEEP>
__device__ __forceinline__ void hidden_layers(TileEngine<T, MT, NTL, NW, HP>& eng, const TileLds<MT>& lds, const FusedArgs& g,
                                     int j, float tau, int64_t row0, int64_t set_off = 0) {
  for (int l = 0; l + 1 < g.L; ++l) {
    const PassDesc p = fwd_pass(g, l);
    const PassDesc nx = fwd_pass(g, l + 1);
    const bool next_is_last = (l + 2 == g.L);
    const lds_f32* bias = lds.param + g.layer[l].bias_off;
    const lds_f32* wt = lds.param + g.wt_off;
    const bool has_wt = (l == 0);
    lds_u16* out = lds.out(l);
    const int ldp = lds.ldp;
    uint16_t* goutT = KEEP ? g.ACTT[l] + set_off : nullptr;
    const int64_t kj = (int64_t)j * g.Rp + row0;
    auto pre = [](int, int) { return make_uint2(0u, 0u); };
    auto epi = [&](const f32x4& acc, uint2, int, int, int n, int m) {
      const float4 bv = lds_load_f4(&bias[n]);
      float v[4] = {acc[0] + bv.x, acc[1] + bv.y, acc[2] + bv.z, acc[3] + bv.w};
      if (has_wt) {
        const float4 tv = lds_load_f4(&wt[n]);
        v[0] = fmaf(tv.x, tau, v[0]); v[1] = fmaf(tv.y, tau, v[1]);
        v[2] = fmaf(tv.z, tau, v[2]); v[3] = fmaf(tv.w, tau, v[3]);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = tanh_fast(v[r]);
      const uint2 q = pack4<T>(v);
      lds_store_u2(&out[m * ldp + n], q);
      if (KEEP && lds.act) lds_store_u2(&lds.act_tile(j, l, g.L)[m * ldp + n], q);
      if (KEEP && row0 + m < g.R) RAMPDE_STORE_G4(group4(goutT, g.ldk, kj + m, n), q);
    };
    auto nxt = [&]() {
      if (next_is_last) eng.template preload_state<false>(nx);
      else eng.template preload_hidden<false>(nx, 0);
    };
    if (l == 0) eng.template run_hidden<true>(p, lds.in(l), lds.ld_in(l), pre, epi, nxt);
    else eng.template run_hidden<false>(p, lds.in(l), lds.ld_in(l), pre, epi, nxt);
  }
}

// fp32 pre-activation of the last layer for the lane's 4 columns
__device__ __forceinline__ void last_layer_values(const f32x4& acc, const lds_f32* param, const FusedArgs& g, float tau, int n,
                                         float (&v)[4]) {
  const float4 bv = lds_load_f4(&param[g.layer[g.L - 1].bias_off + n]);
  v[0] = acc[0] + bv.x; v[1] = acc[1] + bv.y; v[2] = acc[2] + bv.z; v[3] = acc[3] + bv.w;
  if (g.L == 1) {  // the only layer also carries the time column
    const float4 tv = lds_load_f4(&param[g.wt_off + n]);
    v[0] = fmaf(tv.x, tau, v[0]); v[1] = fmaf(tv.y, tau, v[1]);
    v[2] = fmaf(tv.z, tau, v[2]); v[3] = fmaf(tv.w, tau, v[3]);
  }
}

// ---------------------------------------------------------------------------------------
// Forward pass, all steps in one launch (paper Algorithm 1).  NTL = dpad / 64: column tiles of
// the state that one wavefront owns.
template <class T, int MT, int NTL, int NW, int HP>
__global__ __launch_bounds__(64 * NW) void mlp_forward_fused(FusedArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int TM = 16 * MT;
  const TileLds<MT> lds((lds_u16*)smem, g);
  const int tid = threadIdx.x;
  TileEngine<T, MT, NTL, NW, HP> eng;
  constexpr int NTS = Shape<NTL, NW, HP>::NTS;
  eng.lane = tid & 63;
  eng.wave = tid >> 6;
  const int lm = eng.lane & 15, lq = eng.lane >> 4;
  const int64_t row0 = (int64_t)blockIdx.x * TM;
  const int64_t n_state = g.R * g.d;
  const int L = g.L, s = g.s;
  StageStore<MT> ks{lds.kl, g.k_in_lds != 0, g.K, g.dpad, g.stage_stride, row0, g.R};

  load_params(lds.param, g);
  // y <- y0 (registers), first stored state, first stage input
  float yv[NTS][MT][4];
  if (eng.state_wave()) {
#pragma unroll
    for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int n = eng.state_col(nt, lq), m = mt * 16 + lm;
        load4f(g.y0, row0 + m, g.R, n, g.d, yv[nt][mt]);
        const uint2 q = pack4<T>(yv[nt][mt]);
        if (g.round_incr & 2) unpack4<T>(q, yv[nt][mt]);
        store4h(g.ckpt, row0 + m, g.R, n, g.d, q);
        lds_store_u2(&lds.zbuf[m * lds.ldz + n], q);
      }
  }
  __syncthreads();

  const PassDesc first = fwd_pass(g, 0);
  const PassDesc last = fwd_pass(g, L - 1);
  auto preload_first = [&]() {  // first pass of a velocity evaluation
    if (L > 1) eng.template preload_hidden<true>(first, 0);
    else eng.template preload_state<true>(first);
  };
  preload_first();
  for (int i = 0; i < g.N; ++i) {
    const float* st = g.steptab + (size_t)i * (1 + s);
    const float h = st[0];
    uint16_t* ck_next = g.ckpt + (size_t)(i + 1) * n_state;
    for (int j = 0; j < s; ++j) {
      const float tau = st[1 + j];
      hidden_layers<T, MT, NTL, NW, HP, false>(eng, lds, g, j, tau, row0);
      const bool more = (j + 1 < s) || (i + 1 < g.N);
      auto pre0 = [](int, int) { return make_uint2(0u, 0u); };
      auto epi_last = [&](const f32x4& acc, uint2, int nt, int mt, int n, int m) {
            float v[4];
            last_layer_values(acc, lds.param, g, tau, n, v);
            const uint2 kq = pack4<T>(v);
            float kf[4];
            unpack4<T>(kq, kf);
            float (&y)[4] = yv[nt][mt];
            float incr[4] = {0.f, 0.f, 0.f, 0.f};
            uint2 zq;
            if (j + 1 < s) {
              // next stage input  z = Q(yhat + h * sum_l a_{j+1,l} k_l)
              ks.put(j, m, n, kq);
              for (int l = 0; l < j; ++l) {
                const float a = g.A[(j + 1) * s + l];
                if (a != 0.f) {
                  float kl[4];
                  unpack4<T>(ks.get(l, m, n), kl);
#pragma unroll
                  for (int r = 0; r < 4; ++r) incr[r] = fmaf(a, kl[r], incr[r]);
                }
              }
              const float aj = g.A[(j + 1) * s + j];
              float z[4];
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                incr[r] = fmaf(aj, kf[r], incr[r]);
                z[r] = fmaf(h, incr[r], Low<T>::to_f32(Low<T>::from_f32(y[r])));
              }
              zq = pack4<T>(z);
            } else {
              // y <- y + h * sum_l b_l k_l (fp32); next stored state; first stage input of the next step
              for (int l = 0; l < j; ++l) {
                float kl[4];
                unpack4<T>(ks.get(l, m, n), kl);
#pragma unroll
                for (int r = 0; r < 4; ++r) incr[r] = fmaf(g.b[l], kl[r], incr[r]);
              }
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                incr[r] = fmaf(g.b[j], kf[r], incr[r]);
                if (g.round_incr & 1) incr[r] = Low<T>::to_f32(Low<T>::from_f32(incr[r]));
                y[r] = fmaf(h, incr[r], y[r]);
              }
              zq = pack4<T>(y);
              if (g.round_incr & 2) unpack4<T>(zq, y);
              store4h(ck_next, row0 + m, g.R, n, g.d, zq);
            }
            lds_store_u2(&lds.zbuf[m * lds.ldz + n], zq);
          };
      auto nxt_last = [&]() {
        if (more) preload_first();
      };
      if (L == 1) eng.template run_state<true>(last, lds.in(0), lds.ld_in(0), true, pre0, epi_last, nxt_last);
      else eng.template run_state<false>(last, lds.in(L - 1), lds.ld_in(L - 1), false, pre0, epi_last, nxt_last);
    }
  }
  if (eng.state_wave()) {
#pragma unroll
    for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        store4f(g.y, row0 + mt * 16 + lm, g.R, eng.state_col(nt, lq), g.d, yv[nt][mt]);
  }
}

// ---------------------------------------------------------------------------------------
// One step of the adjoint for a row tile (paper Algorithm 2, the body of the loop over steps).
// TG: also collect the per-step sums of the time-grid gradient (g.tpart).
template <class T, int MT, int NTL, int NW, int HP, bool MULTI, bool TG>
__global__ __launch_bounds__(64 * NW) void mlp_adjoint_step(FusedArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  if (g.ctl->poison) return;
  constexpr int TM = 16 * MT;
  const TileLds<MT> lds((lds_u16*)smem, g);
  const int tid = threadIdx.x;
  TileEngine<T, MT, NTL, NW, HP> eng;
  constexpr int NTS = Shape<NTL, NW, HP>::NTS;
  eng.lane = tid & 63;
  eng.wave = tid >> 6;
  const int lm = eng.lane & 15, lq = eng.lane >> 4;
  const int64_t row0 = (int64_t)blockIdx.x * TM;
  const int L = g.L, s = g.s, D = g.dpad;
  const float S = g.ctl->S;
  StageStore<MT> ks{lds.kl, g.k_in_lds != 0, g.K, D, g.stage_stride, row0, g.R};
  StageStore<MT> zs{lds.kl, g.k_in_lds != 0, g.ZBAR, D, g.stage_stride, row0, g.R};

  load_params(lds.param, g);
  // lane-resident state: the adjoint a (fp32), carried in registers from step to step
  float av[NTS][MT][4];
  bool bad = false;
  unsigned bits = 0;
#pragma unroll
  for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      load4f(g.a_in, row0 + mt * 16 + lm, g.R, eng.state_col(nt, lq), g.d, av[nt][mt]);

  // (MULTI = false: exactly one step, and the loop below folds away)
  const int nsteps = MULTI ? g.nsteps : 1;
#pragma unroll 1
  for (int it = 0; it < nsteps; ++it) {
    const int step = g.step - it;
    const float* st = g.steptab + (size_t)step * (1 + s);
    const float h = st[0];
    const int64_t set_off = (int64_t)(step % g.nsets) * g.set_stride;
    uint16_t* const ZT = g.ZT + set_off;
    uint16_t* const KBART = g.KBART + set_off;
    // per-lane parts of this step's time-grid sums: Phi^T a_{i+1}, dt and dh of eq. (vjp)
    constexpr bool want_t = TG;
    float t_phia = 0.f, t_dt = 0.f, t_dh = 0.f;
    // lambda = Q(S a); yhat = stored state
    uint2 lamq[NTS][MT], yhat[NTS][MT];
#pragma unroll
    for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int n = eng.state_col(nt, lq), m = mt * 16 + lm;
        float sa[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) sa[r] = S * av[nt][mt][r];
        lamq[nt][mt] = pack4<T>(sa);
        bad = bad || any_nonfinite4<T>(lamq[nt][mt]);
        yhat[nt][mt] = load4h(g.ckpt + (size_t)step * g.ckpt_stride, row0 + m, g.R, n, g.d);
      }

    // cotangent of the slope of stage j:  kbar_j = Q( b_j lambda + h sum_{l>j} a_lj zbar_l ),
    // with zbar_{j+1} still in registers (zn) and the later ones read back from the stage store
    auto make_kbar = [&](int j, int nt, int mt, int m, int n, const float* zn) -> uint2 {
      float lam[4], acc[4] = {0.f, 0.f, 0.f, 0.f}, v[4];
      unpack4<T>(lamq[nt][mt], lam);
      for (int l = s - 1; l > j + 1; --l) {
        const float a = g.A[l * s + j];
        if (a != 0.f) {
          float zl[4];
          unpack4<T>(zs.get(l, m, n), zl);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[r] = fmaf(a, zl[r], acc[r]);
        }
      }
      if (zn) {
        const float a = g.A[(j + 1) * s + j];
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] = fmaf(a, zn[r], acc[r]);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = fmaf(h, acc[r], g.b[j] * lam[r]);
      const uint2 q = pack4<T>(v);
      bad = bad || any_nonfinite4<T>(q);
      if (want_t && g.L == 1) {
        // single-layer network: the slope cotangent is the layer-1 cotangent
        // (g.L, not the local copy L: capturing that local here made the compiler keep the whole
        // argument block and the closures in scratch memory)
        float kb[4];
        unpack4<T>(q, kb);
        const float4 tv = lds_load_f4(&(lds.param + g.wt_off)[n]);
        const float tb = kb[0] * tv.x + kb[1] * tv.y + kb[2] * tv.z + kb[3] * tv.w;
        t_dt += tb;
        t_dh = fmaf(g.c[j], tb, t_dh);
      }
      lds_store_u2(&lds.zbuf[m * lds.ldz + n], q);
      if (row0 + m < g.R) RAMPDE_STORE_G4(group4(KBART, g.ldk, (int64_t)j * g.Rp + row0 + m, n), q);
      return q;
    };

    const PassDesc firstf = fwd_pass(g, 0);
    const PassDesc lastf = fwd_pass(g, L - 1);
    const PassDesc firstb = bwd_pass(g, L - 1);
    const PassDesc lastb = bwd_pass(g, 0);

    auto preload_first_f = [&]() {
      if (L > 1) eng.template preload_hidden<true>(firstf, 0);
      else eng.template preload_state<true>(firstf);
    };
    auto preload_first_b = [&]() {
      if (L > 1) eng.template preload_hidden<true>(firstb, 0);
      else eng.template preload_state<true>(firstb);
    };

    if (!g.skip_recompute) {
      // ---- stage recomputation from the stored state, keeping inputs and activations
      preload_first_f();
      if (eng.state_wave()) {
#pragma unroll
        for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const int n = eng.state_col(nt, lq), m = mt * 16 + lm;
            lds_store_u2(&lds.zbuf[m * lds.ldz + n], yhat[nt][mt]);
            if (row0 + m < g.R) RAMPDE_STORE_G4(group4(ZT, g.ldk, row0 + m, n), yhat[nt][mt]);
          }
      }
      __syncthreads();
      for (int j = 0; j < s; ++j) {
        const float tau = st[1 + j];
        hidden_layers<T, MT, NTL, NW, HP, true>(eng, lds, g, j, tau, row0, set_off);
        const bool more = j + 1 < s;
        auto pre0 = [](int, int) { return make_uint2(0u, 0u); };
        auto epi_last = [&](const f32x4& acc, uint2, int nt, int mt, int n, int m) {
              float v[4];
              last_layer_values(acc, lds.param, g, tau, n, v);
              const uint2 kq = pack4<T>(v);
              float kf[4];
              unpack4<T>(kq, kf);
              if (want_t) {
#pragma unroll
                for (int r = 0; r < 4; ++r) t_phia = fmaf(g.b[j] * kf[r], av[nt][mt][r], t_phia);
              }
              if (j + 1 < s) {
                float incr[4] = {0.f, 0.f, 0.f, 0.f}, yh[4], z[4];
                unpack4<T>(yhat[nt][mt], yh);
                ks.put(j, m, n, kq);
                for (int l = 0; l < j; ++l) {
                  const float a = g.A[(j + 1) * s + l];
                  if (a != 0.f) {
                    float kl[4];
                    unpack4<T>(ks.get(l, m, n), kl);
#pragma unroll
                    for (int r = 0; r < 4; ++r) incr[r] = fmaf(a, kl[r], incr[r]);
                  }
                }
                const float aj = g.A[(j + 1) * s + j];
#pragma unroll
                for (int r = 0; r < 4; ++r) z[r] = fmaf(h, fmaf(aj, kf[r], incr[r]), yh[r]);
                const uint2 zq = pack4<T>(z);
                lds_store_u2(&lds.zbuf[m * lds.ldz + n], zq);
                if (row0 + m < g.R) RAMPDE_STORE_G4(group4(ZT, g.ldk, (int64_t)(j + 1) * g.Rp + row0 + m, n), zq);
              } else {
                make_kbar(s - 1, nt, mt, m, n, nullptr);  // the slope of the last stage is not needed again
              }
            };
        auto nxt_last = [&]() {
          if (more) preload_first_f();
          else preload_first_b();
        };
        if (L == 1) eng.template run_state<true>(lastf, lds.in(0), lds.ld_in(0), true, pre0, epi_last, nxt_last);
        else eng.template run_state<false>(lastf, lds.in(L - 1), lds.ld_in(L - 1), false, pre0, epi_last, nxt_last);
      }
    } else {
      preload_first_b();
      if (eng.state_wave()) {
#pragma unroll
        for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            make_kbar(s - 1, nt, mt, mt * 16 + lm, eng.state_col(nt, lq), nullptr);
      }
      __syncthreads();
    }

    // ---- cotangent chain, stages in reverse (eq. (vjp) pushed through the stage recursion)
    float da[NTS][MT][4];
#pragma unroll
    for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) da[nt][mt][r] = 0.f;

    for (int j = s - 1; j >= 0; --j) {
      for (int l = L - 1; l >= 1; --l) {
        const int q = L - 1 - l;
        const PassDesc p = bwd_pass(g, l);
        const PassDesc nx = bwd_pass(g, l - 1);
        const bool next_is_last = (l == 1);
        uint16_t* actT = g.ACTT[l - 1] + set_off;
        uint16_t* goutT = g.DELTAT[l - 1] + set_off;
        const int64_t kj = (int64_t)j * g.Rp + row0;
        lds_u16* out = lds.out(q);
        const int ldp = lds.ldp;
        // (a retry launch that skips the recomputation has no LDS copy: it reads the stored one)
        const lds_u16* act_lds = (lds.act && !g.skip_recompute) ? lds.act_tile(j, l - 1, g.L) : nullptr;
        auto pre_act = [&](int n, int m) {
                  if (act_lds) return lds_load_u2(&act_lds[m * ldp + n]);
                  return (row0 + m < g.R) ? *group4(actT, g.ldk, kj + m, n) : make_uint2(0u, 0u);
                };
        auto epi_delta = [&](const f32x4& acc, uint2 pf, int, int, int n, int m) {
                  float a[4], v[4];
                  unpack4<T>(pf, a);
#pragma unroll
                  for (int r = 0; r < 4; ++r) v[r] = acc[r] * (1.f - a[r] * a[r]);
                  const uint2 dq = pack4<T>(v);
                  if (want_t && l == 1) {
                    // layer-1 cotangent times the time column: this stage's part of dt and dh
                    float dv[4];
                    unpack4<T>(dq, dv);
                    const float4 tv = lds_load_f4(&(lds.param + g.wt_off)[n]);
                    const float tb = dv[0] * tv.x + dv[1] * tv.y + dv[2] * tv.z + dv[3] * tv.w;
                    t_dt += tb;
                    t_dh = fmaf(g.c[j], tb, t_dh);
                  }
                  lds_store_u2(&out[m * ldp + n], dq);
                  if (row0 + m < g.R) {
                    RAMPDE_STORE_G4(group4(goutT, g.ldk, kj + m, n), dq);
                    bad = bad || any_nonfinite4<T>(dq);
                  }
                };
        auto nxt_b = [&]() {
          if (next_is_last) eng.template preload_state<false>(nx);
          else eng.template preload_hidden<false>(nx, 0);
        };
        if (q == 0) eng.template run_hidden<true>(p, lds.in(q), lds.ld_in(q), pre_act, epi_delta, nxt_b);
        else eng.template run_hidden<false>(p, lds.in(q), lds.ld_in(q), pre_act, epi_delta, nxt_b);
      }
      const int q = L - 1;
      auto pre0 = [](int, int) { return make_uint2(0u, 0u); };
      auto epi_zbar = [&](const f32x4& acc, uint2, int nt, int mt, int n, int m) {
            const float v[4] = {acc[0], acc[1], acc[2], acc[3]};
            const uint2 zq = pack4<T>(v);
            if (row0 + m < g.R) bad = bad || any_nonfinite4<T>(zq);
            float zf[4];
            unpack4<T>(zq, zf);
#pragma unroll
            for (int r = 0; r < 4; ++r) da[nt][mt][r] += zf[r];
            if (want_t) {
              for (int l = 0; l < j; ++l) {
                const float a = g.A[j * s + l];
                if (a != 0.f) {
                  float kl[4];
                  unpack4<T>(ks.get(l, m, n), kl);
#pragma unroll
                  for (int r = 0; r < 4; ++r) t_dh = fmaf(a * kl[r], zf[r], t_dh);
                }
              }
            }
            if (j > 0) {
              zs.put(j, m, n, zq);
              make_kbar(j - 1, nt, mt, m, n, zf);
            }
          };
      auto nxt_z = [&]() {
        if (j > 0) preload_first_b();
      };
      if (L == 1) eng.template run_state<true>(lastb, lds.in(0), lds.ld_in(0), true, pre0, epi_zbar, nxt_z);
      else eng.template run_state<false>(lastb, lds.in(q), lds.ld_in(q), false, pre0, epi_zbar, nxt_z);
    }
    // ---- a <- a + (h / S) sum_j zbar_j (+ running-cost cotangent), fp32; max |a| after the last step
    bits = 0;
    const float hs = h / S;
    if (want_t) block_sum2(fmaf(hs, t_dt - t_dh, -t_phia), fmaf(hs, t_dh, t_phia), g.tpart + 2 * ((size_t)it * gridDim.x + blockIdx.x));
#pragma unroll
    for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int n = eng.state_col(nt, lq), m = mt * 16 + lm;
        float gy[4] = {0.f, 0.f, 0.f, 0.f};
        if (g.gys) load4f(g.gys - (int64_t)it * g.gys_stride, row0 + m, g.R, n, g.d, gy);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          av[nt][mt][r] = fmaf(hs, da[nt][mt][r], av[nt][mt][r]) + gy[r];
          if (g.round_incr & 2) av[nt][mt][r] = Low<T>::to_f32(Low<T>::from_f32(av[nt][mt][r]));
          const unsigned bb = __builtin_bit_cast(unsigned, fabsf(av[nt][mt][r]));
          if (row0 + m < g.R && n + r < g.d) bits = bb > bits ? bb : bits;
        }
      }
  }  // steps of this launch

  if (g.detect) raise_if_any(bad, g.ctl);
#pragma unroll
  for (int nt = 0; nt < NTS; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      store4f(g.a_out, row0 + mt * 16 + lm, g.R, eng.state_col(nt, lq), g.d, av[nt][mt]);
  block_amax(bits, &g.ctl->amax_bits);

  // ---- the last workgroup to get here takes the decision of this step (accept / grow, or poison)
  // (the flags and the max-norm travel by device-scope atomics; one fence per workgroup orders
  // them before the arrival counter)
  __shared__ int is_last;
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    is_last = (atomicAdd(&g.ctl->done, 1) == (int)gridDim.x - 1);
  }
  __syncthreads();
  if (is_last && tid == 0) {
    __threadfence();
    Ctl* c = g.ctl;
    const unsigned nonfinite = atomicOr(&c->nonfinite, 0u);
    const unsigned amax_bits = atomicMax(&c->amax_bits, 0u);
    if (g.detect && nonfinite) {
      c->poison = 1;
      c->failed_step = g.step;
    } else {
      for (int it = 0; it < nsteps; ++it) g.scale_hist[g.step - it] = S;
      c->S_step = S;
      c->s_min = fminf(c->s_min, S);
      c->s_max = fmaxf(c->s_max, S);
      if (g.dynamic && c->attempt == 1) {
        const float amax = __builtin_bit_cast(float, amax_bits);
        const float test = g.raw_norm ? amax : S * amax;
        if (test <= ldexpf(1.f, Low<T>::p_bits - 1) && S < ldexpf(1.f, 126)) c->S = 2.f * S;
      }
      c->attempt = 1;
      c->amax_bits = 0;
      c->nonfinite = 0;
    }
    c->done = 0;
  }
}

}  // namespace rampde
