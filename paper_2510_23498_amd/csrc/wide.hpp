// Row-tile kernels for WIDE dense velocity networks (hidden width 512): the same work split as
// fused.hpp -- a workgroup owns a tile of batch rows and carries it through whole passes of the
// method (paper Algorithm 1: all steps of the forward pass; Algorithm 2: one adjoint step with
// recomputation, cotangent chain, detector, fp32 update and the scale decision) -- rebuilt around
// what bounds a 64-row tile on a gfx950 compute unit:
//
//   * v_mfma_f32_32x32x16 with a 64 x 64 output tile per wavefront (64 hidden columns x 64 batch
//     rows, four accumulators).  Per contraction step of 16 a wavefront then fetches two weight
//     fragments and two activation fragments for FOUR matrix instructions: half the LDS reads per
//     flop of 16 x 16 x 32 tiles, and the 32-row fragment read (32 rows x 2 chunks of 16 bytes, row
//     pitch = 1 chunk modulo 16) is free of bank conflicts, which the 16-row x 4-chunk read is not.
//   * nothing per-tile lives in registers between passes: the fp32 state (y forward, a backward),
//     the stored state, the slopes and the stage cotangents are re-read from global memory (a
//     tile's 32 KB stay in L2) by the epilogues of the state-shaped passes, which are the only
//     places that need them.  The register file goes to the accumulators (64), the weight ring
//     (64) and the activation fragments (16): 64-row tiles for the adjoint step too, which halves
//     the weight traffic per row from L2 against 32-row tiles.
//   * weights stream from L2 in a fragment-major layout (1 KB per wavefront load), 8 contraction
//     steps ahead, across pass boundaries (every pass requests the first fragments of its
//     successor before its own epilogue).
//
// Layouts.  Weight fragments of a layer W[n][k] (n = output feature, k = input feature):
//   forward    Wf  [Kpad / 16][Npad / 32][64 lanes] x 16 B: lane -> W[ct * 32 + lane % 32][ks * 16 + (lane / 32) * 8 + 0..7]
//   transposed WTf [Npad / 16][Kpad / 32][64 lanes] x 16 B: lane -> W[ns * 16 + (lane / 32) * 8 + 0..7][kt * 32 + lane % 32]
// The weight tile is the FIRST operand of the matrix instruction, the activations the second: a lane
// ends with batch row lane % 32 and four runs of 4 consecutive output features (8-byte stores).
// Everything handed to the parameter-gradient kernel is feature-group-major as in fused.hpp.
#pragma once
#include "fused.hpp"

namespace rampde {

// A value the optimiser must treat as new at this point.  The epilogues derive every address from
// laundered lane coordinates: otherwise all their (loop-invariant) 64-bit addresses are computed
// once at kernel entry and kept alive -- or spilled -- across the contraction loops.
__device__ __forceinline__ int fresh(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

constexpr int kWideWaves = 8;
constexpr int kWidePD = 8;  // contraction steps (of 16) of weight fragments in flight per wavefront

// theta (fp32) -> the two fragment-major copies above + rounded biases / time column (fp32)
template <class T>
__global__ void cast_dense_fragments_wide(CastArgs c) {
  const int lane = threadIdx.x & 63;
  int frag = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (frag >= c.nfrag) return;
  CastLayer y = c.layer[0];
#pragma unroll
  for (int q = 1; q < kMaxLayers; ++q)
    if (q < c.L && frag >= c.layer[q].frag0) y = c.layer[q];
  frag -= y.frag0;
  const int nfw = (y.Kpad / 16) * (y.Npad / 32);
  if (frag < nfw) {
    const int ks = frag / (y.Npad / 32), ct = frag % (y.Npad / 32);
    const int n = ct * 32 + (lane & 31), k0 = ks * 16 + (lane >> 5) * 8;
    u16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = k0 + e;
      v[e] = (n < y.out && k < y.in) ? Low<T>::from_f32(y.W[(size_t)n * y.in_full + k]) : (uint16_t)0;
    }
    y.Wf[(size_t)frag * 64 + lane] = v;
    if (ks == 0 && lane < 32) {
      y.bias_f[n] = (n < y.out) ? Low<T>::to_f32(Low<T>::from_f32(y.b[n])) : 0.f;
      y.wt_f[n] = (n < y.out && y.has_time) ? Low<T>::to_f32(Low<T>::from_f32(y.W[(size_t)n * y.in_full + y.in])) : 0.f;
    }
  } else {
    const int f = frag - nfw;
    const int ns = f / (y.Kpad / 32), kt = f % (y.Kpad / 32);
    const int k = kt * 32 + (lane & 31), n0 = ns * 16 + (lane >> 5) * 8;
    u16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int n = n0 + e;
      v[e] = (n < y.out && k < y.in) ? Low<T>::from_f32(y.W[(size_t)n * y.in_full + k]) : (uint16_t)0;
    }
    y.WTf[(size_t)f * 64 + lane] = v;
  }
}

// One contraction pass of a wavefront: acc[ct][rt] (32 x 32 each) += W-tile(ct) * act-tile(rt)^T over
// KS steps of 16.  `wb` points at the calling lane's 16 bytes of fragment (step 0, first owned
// column tile); consecutive column tiles are 64 fragments-of-16-bytes apart, steps CT * 64 apart.
// `ab` is the lane's LDS address in row tile 0: row lane % 32, element (lane / 32) * 8.
// On entry ring[u] holds steps u < min(PD, KS) (requested by the previous pass).
template <int NCT, int PD>
__device__ __forceinline__ void wide_preload(u16x8 (&ring)[PD][2], const glb_u16x8* wb, int KS, int CT) {
#pragma unroll
  for (int u = 0; u < PD; ++u) {
    const int ks = u < KS ? u : KS - 1;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) ring[u][ct] = wb[(size_t)ks * CT * 64 + ct * 64];
  }
}

template <class T, int NCT, int NRT, int KS, int CT, int PD>
__device__ __forceinline__ void wide_mma(f32x16 (&acc)[NCT][NRT], u16x8 (&ring)[PD][2], const glb_u16x8* wb,
                                         const lds_u16* ab, int ld) {
  static_assert(PD % 2 == 0 && (KS <= PD || KS % PD == 0), "pipeline depth");
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[ct][rt][q] = 0.f;
  u16x8 b[2][NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) b[0][rt] = *(const lds_u16x8*)(ab + rt * 32 * ld);
  constexpr int MAIN = KS > PD ? KS - PD : 0;
#pragma unroll 1
  for (int ks0 = 0; ks0 < MAIN; ks0 += PD) {
    const glb_u16x8* wn = wb + (size_t)(ks0 + PD) * CT * 64;
    const lds_u16* an = ab + (ks0 + 1) * 16;
#pragma unroll
    for (int u = 0; u < PD; ++u) {
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) b[(u + 1) & 1][rt] = *(const lds_u16x8*)(an + rt * 32 * ld + u * 16);
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) acc[ct][rt] = Low<T>::mfma32(ring[u][ct], b[u & 1][rt], acc[ct][rt]);
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct) ring[u][ct] = wn[(size_t)u * CT * 64 + ct * 64];
      // issue order within the step: the next step's activation fragments first (their latency hides
      // behind this step's matrix instructions), then the matrix instructions, then the refill of
      // this ring slot -- which must issue here, a full PD steps ahead of its use, and not drift to
      // the end of the unrolled group
      __builtin_amdgcn_sched_group_barrier(0x100, NRT, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, NCT * NRT, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, NCT, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  constexpr int TAIL = KS < PD ? KS : PD;
#pragma unroll
  for (int u = 0; u < TAIL; ++u) {
    if (u + 1 < TAIL) {
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) b[(u + 1) & 1][rt] = *(const lds_u16x8*)(ab + rt * 32 * ld + (MAIN + u + 1) * 16);
    }
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) acc[ct][rt] = Low<T>::mfma32(ring[u][ct], b[u & 1][rt], acc[ct][rt]);
  }
}

// Shapes of a network with state width D and hidden width HP on a 64-row tile, 8 wavefronts.
//   hidden-shaped output: wavefront w owns column tiles 2w, 2w + 1 (of 32) per group of 512
//   columns, both row tiles;
//   state-shaped output: D / 32 column tiles x 2 row tiles over 8 wavefronts.
template <int HP, int D>
struct WideShape {
  static_assert(HP == 512, "hidden width");
  static_assert(D == 128 || D == 256, "state width");
  static constexpr int TM = 64;
  static constexpr int KS_S = D / 16, KS_H = HP / 16;
  static constexpr int CT_H = HP / 32, CT_S = D / 32;
  static constexpr int S_NRT = (D == 128) ? 1 : 2;  // row tiles a wavefront owns in a state-shaped pass
  static constexpr int ldz = D + 8, ldp = HP + 8;
  __device__ static inline int s_ct(int wave) { return D == 128 ? (wave & 3) : wave; }
  __device__ static inline int s_rt0(int wave) { return D == 128 ? (wave >> 2) : 0; }
};

template <int HP, int D>
struct WideLds {
  using Sh = WideShape<HP, D>;
  lds_f32* param;
  lds_u16* zbuf;  // [64][D + 8]
  lds_u16* x0;    // [64][HP + 8]
  lds_u16* x1;
  __device__ __forceinline__ WideLds(lds_u16* smem, const FusedArgs& g) {
    param = (lds_f32*)smem;
    zbuf = smem + 2 * g.nparam;
    x0 = zbuf + Sh::TM * Sh::ldz;
    x1 = x0 + Sh::TM * Sh::ldp;
  }
  __device__ inline lds_u16* x(int q) const { return (q & 1) ? x1 : x0; }
};
template <int HP, int D>
constexpr size_t wide_lds_bytes(int nparam) {
  return (size_t)nparam * 4 + 64 * (size_t)(D + 8) * 2 + 2 * 64 * (size_t)(HP + 8) * 2;
}

// The per-wavefront engine: lane coordinates, the weight ring, and the pass drivers.
template <class T, int HP, int D>
struct WideEngine {
  using Sh = WideShape<HP, D>;
  static constexpr int PD = kWidePD;
  u16x8 ring[PD][2];
  int lane, wave, lr, lh;  // lr = lane % 32 (batch row within a row tile), lh = lane / 32

  __device__ inline const glb_u16x8* frag_base(const u16x8* W, int ct0) const {
    return (const glb_u16x8*)W + (size_t)ct0 * 64 + lane;
  }
  // request the first fragments of a hidden-shaped pass (contraction over the state: KS_S, else KS_H)
  template <bool FROM_STATE>
  __device__ __forceinline__ void preload_hidden(const u16x8* W) {
    wide_preload<2, PD>(ring, frag_base(W, 2 * wave), FROM_STATE ? Sh::KS_S : Sh::KS_H, Sh::CT_H);
  }
  __device__ __forceinline__ void preload_state(const u16x8* W) {
    wide_preload<1, PD>(ring, frag_base(W, Sh::s_ct(wave)), Sh::KS_H, Sh::CT_S);
  }

  // hidden-shaped pass: epi(acc16, n0 of the tile, row tile); nxt() requests the successor's fragments
  template <bool FROM_STATE, class Epi, class Nxt>
  __device__ __forceinline__ void run_hidden(const u16x8* W, const lds_u16* in, Epi epi, Nxt nxt) {
    constexpr int KS = FROM_STATE ? Sh::KS_S : Sh::KS_H;
    constexpr int ld = FROM_STATE ? Sh::ldz : Sh::ldp;
    f32x16 acc[2][2];
    wide_mma<T, 2, 2, KS, Sh::CT_H, PD>(acc, ring, frag_base(W, 2 * wave), in + lr * ld + lh * 8, ld);
    nxt();
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) epi(acc[ct][rt], (2 * wave + ct) * 32, rt);
    __syncthreads();
  }
  // state-shaped pass (contraction over the hidden width)
  template <class Epi, class Nxt>
  __device__ __forceinline__ void run_state(const u16x8* W, const lds_u16* in, Epi epi, Nxt nxt) {
    f32x16 acc[1][Sh::S_NRT];
    const int rt0 = Sh::s_rt0(wave);
    wide_mma<T, 1, Sh::S_NRT, Sh::KS_H, Sh::CT_S, PD>(acc, ring, frag_base(W, Sh::s_ct(wave)),
                                                      in + (rt0 * 32 + lr) * Sh::ldp + lh * 8, Sh::ldp);
    nxt();
#pragma unroll
    for (int rt = 0; rt < Sh::S_NRT; ++rt) epi(acc[0][rt], Sh::s_ct(wave) * 32, rt0 + rt);
    __syncthreads();
  }
  // the state elements of this lane, as the state-shaped passes see them: f(n, m) for every
  // (first feature n of a run of 4, row m of the tile)
  template <class F>
  __device__ __forceinline__ void for_state(F f) const {
    const int r = fresh(lr), c = Sh::s_ct(wave) * 32 + 4 * fresh(lh);
#pragma unroll
    for (int rt = 0; rt < Sh::S_NRT; ++rt)
#pragma unroll
      for (int q = 0; q < 4; ++q) f(c + 8 * q, (Sh::s_rt0(wave) + rt) * 32 + r);
  }
};

// hidden layers of one velocity evaluation (all layers but the last), stage j.  KEEP: the
// activations also go to the feature-group-major buffers (adjoint recomputation).
template <class T, int HP, int D, bool KEEP>
__device__ __forceinline__ void wide_hidden_layers(WideEngine<T, HP, D>& eng, const WideLds<HP, D>& lds, const FusedArgs& g,
                                                   int j, float tau, int64_t row0, int64_t set_off) {
  using Sh = WideShape<HP, D>;
  for (int l = 0; l + 1 < g.L; ++l) {
    const lds_f32* bias = lds.param + g.layer[l].bias_off;
    const lds_f32* wt = lds.param + g.wt_off;
    const bool has_wt = (l == 0);
    lds_u16* out = lds.x(l);
    uint16_t* goutT = KEEP ? g.ACTT[l] + set_off : nullptr;
    const int64_t kj = (int64_t)j * g.Rp + row0;
    const u16x8* Wnext = g.layer[l + 1].Wf;
    const bool next_is_last = (l + 2 == g.L);
    auto epi = [&](const f32x16& acc, int n_tile, int rt) {
      const int m = rt * 32 + fresh(eng.lr), lh4 = 4 * fresh(eng.lh);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n_tile + 8 * q + lh4;
        const float4 bv = lds_load_f4(&bias[n]);
        float v[4] = {acc[4 * q] + bv.x, acc[4 * q + 1] + bv.y, acc[4 * q + 2] + bv.z, acc[4 * q + 3] + bv.w};
        if (has_wt) {
          const float4 tv = lds_load_f4(&wt[n]);
          v[0] = fmaf(tv.x, tau, v[0]); v[1] = fmaf(tv.y, tau, v[1]);
          v[2] = fmaf(tv.z, tau, v[2]); v[3] = fmaf(tv.w, tau, v[3]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = tanh_fast(v[r]);
        const uint2 pq = pack4<T>(v);
        lds_store_u2(&out[m * Sh::ldp + n], pq);
        if (KEEP && row0 + m < g.R) *group4(goutT, g.ldk, kj + m, n) = pq;
      }
    };
    auto nxt = [&]() {
      if (next_is_last) eng.preload_state(Wnext);
      else eng.template preload_hidden<false>(Wnext);
    };
    if (l == 0) eng.template run_hidden<true>(g.layer[0].Wf, lds.zbuf, epi, nxt);
    else eng.template run_hidden<false>(g.layer[l].Wf, lds.x(l - 1), epi, nxt);
  }
}

// ---------------------------------------------------------------------------------------
// Forward pass, all steps in one launch (paper Algorithm 1).
template <class T, int HP, int D>
__global__ __launch_bounds__(64 * kWideWaves) void mlp_forward_wide(FusedArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  using Sh = WideShape<HP, D>;
  const WideLds<HP, D> lds((lds_u16*)smem, g);
  WideEngine<T, HP, D> eng;
  eng.lane = threadIdx.x & 63;
  eng.wave = threadIdx.x >> 6;
  eng.lr = eng.lane & 31;
  eng.lh = eng.lane >> 5;
  const int64_t row0 = (int64_t)blockIdx.x * Sh::TM;
  const int64_t n_state = g.R * D;
  const int L = g.L, s = g.s;

  load_params(lds.param, g);
  // y <- y0 (kept in the output buffer), first stored state, first stage input
  eng.for_state([&](int n, int m) {
    float v[4];
    load4f(g.y0, row0 + m, g.R, n, D, v);
    const uint2 q = pack4<T>(v);
    if (g.round_incr & 2) unpack4<T>(q, v);
    store4f(g.y, row0 + m, g.R, n, D, v);
    store4h(g.ckpt, row0 + m, g.R, n, D, q);
    lds_store_u2(&lds.zbuf[m * Sh::ldz + n], q);
  });
  __syncthreads();

  eng.template preload_hidden<true>(g.layer[0].Wf);
  for (int i = 0; i < g.N; ++i) {
    const float* st = g.steptab + (size_t)i * (1 + s);
    const float h = st[0];
    const uint16_t* ck = g.ckpt + (size_t)i * n_state;
    uint16_t* ck_next = g.ckpt + (size_t)(i + 1) * n_state;
    for (int j = 0; j < s; ++j) {
      const float tau = st[1 + j];
      wide_hidden_layers<T, HP, D, false>(eng, lds, g, j, tau, row0, 0);
      const bool more = (j + 1 < s) || (i + 1 < g.N);
      const lds_f32* bias = lds.param + g.layer[L - 1].bias_off;
      auto epi_last = [&](const f32x16& acc, int n_tile, int rt) {
        const int m = rt * 32 + fresh(eng.lr), lh4 = 4 * fresh(eng.lh);
        const int64_t row = row0 + m;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n_tile + 8 * q + lh4;
          const float4 bv = lds_load_f4(&bias[n]);
          const float v[4] = {acc[4 * q] + bv.x, acc[4 * q + 1] + bv.y, acc[4 * q + 2] + bv.z, acc[4 * q + 3] + bv.w};
          const uint2 kq = pack4<T>(v);
          float kf[4], incr[4] = {0.f, 0.f, 0.f, 0.f};
          unpack4<T>(kq, kf);
          uint2 zq;
          if (j + 1 < s) {
            // next stage input  z = Q(yhat + h * sum_l a_{j+1,l} k_l)
            store4h(g.K + (size_t)j * g.stage_stride, row, g.R, n, D, kq);
            for (int l = 0; l < j; ++l) {
              const float a = g.A[(j + 1) * s + l];
              if (a != 0.f) {
                float kl[4];
                unpack4<T>(load4h(g.K + (size_t)l * g.stage_stride, row, g.R, n, D), kl);
#pragma unroll
                for (int r = 0; r < 4; ++r) incr[r] = fmaf(a, kl[r], incr[r]);
              }
            }
            const float aj = g.A[(j + 1) * s + j];
            float yh[4], z[4];
            unpack4<T>(load4h(ck, row, g.R, n, D), yh);
#pragma unroll
            for (int r = 0; r < 4; ++r) z[r] = fmaf(h, fmaf(aj, kf[r], incr[r]), yh[r]);
            zq = pack4<T>(z);
          } else {
            // y <- y + h * sum_l b_l k_l (fp32); next stored state = first stage input of the next step
            for (int l = 0; l < j; ++l) {
              float kl[4];
              unpack4<T>(load4h(g.K + (size_t)l * g.stage_stride, row, g.R, n, D), kl);
#pragma unroll
              for (int r = 0; r < 4; ++r) incr[r] = fmaf(g.b[l], kl[r], incr[r]);
            }
            float y[4];
            load4f(g.y, row, g.R, n, D, y);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              incr[r] = fmaf(g.b[j], kf[r], incr[r]);
              if (g.round_incr & 1) incr[r] = Low<T>::to_f32(Low<T>::from_f32(incr[r]));
              y[r] = fmaf(h, incr[r], y[r]);
            }
            zq = pack4<T>(y);
            if (g.round_incr & 2) unpack4<T>(zq, y);
            store4f(g.y, row, g.R, n, D, y);
            store4h(ck_next, row, g.R, n, D, zq);
          }
          lds_store_u2(&lds.zbuf[m * Sh::ldz + n], zq);
        }
      };
      auto nxt_last = [&]() {
        if (more) eng.template preload_hidden<true>(g.layer[0].Wf);
      };
      eng.run_state(g.layer[L - 1].Wf, lds.x(L - 2), epi_last, nxt_last);
    }
  }
}

// ---------------------------------------------------------------------------------------
// One step of the adjoint for a 64-row tile (paper Algorithm 2, the body of the loop over steps).
template <class T, int HP, int D>
__global__ __launch_bounds__(64 * kWideWaves) void mlp_adjoint_wide(FusedArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  if (g.ctl->poison) return;
  using Sh = WideShape<HP, D>;
  const WideLds<HP, D> lds((lds_u16*)smem, g);
  WideEngine<T, HP, D> eng;
  const int tid = threadIdx.x;
  eng.lane = tid & 63;
  eng.wave = tid >> 6;
  eng.lr = eng.lane & 31;
  eng.lh = eng.lane >> 5;
  const int64_t row0 = (int64_t)blockIdx.x * Sh::TM;
  const int64_t n_state = g.R * D;
  const int L = g.L, s = g.s;
  const float S = g.ctl->S;
  const int step = g.step;
  const float* st = g.steptab + (size_t)step * (1 + s);
  const float h = st[0];
  const int64_t set_off = (int64_t)(step % g.nsets) * g.set_stride;
  uint16_t* const ZT = g.ZT + set_off;
  uint16_t* const KBART = g.KBART + set_off;
  const uint16_t* ck = g.ckpt + (size_t)step * n_state;
  bool bad = false;

  load_params(lds.param, g);

  // cotangent of the slope of stage j:  kbar_j = Q( b_j lambda + h sum_{l>j} a_lj zbar_l ),  lambda = Q(S a);
  // zbar_{j+1} may still be in registers (zn), the later ones are read back from the workspace
  auto make_kbar = [&](int j, int m, int n, const float* zn) {
    const int64_t row = row0 + m;
    float a[4], lam[4], acc[4] = {0.f, 0.f, 0.f, 0.f}, v[4];
    load4f(g.a_in, row, g.R, n, D, a);
#pragma unroll
    for (int r = 0; r < 4; ++r) a[r] *= S;
    const uint2 lq = pack4<T>(a);
    bad = bad || any_nonfinite4<T>(lq);
    unpack4<T>(lq, lam);
    for (int l = s - 1; l > j + (zn ? 1 : 0); --l) {
      const float c = g.A[l * s + j];
      if (c != 0.f) {
        float zl[4];
        unpack4<T>(load4h(g.ZBAR + (size_t)l * g.stage_stride, row, g.R, n, D), zl);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] = fmaf(c, zl[r], acc[r]);
      }
    }
    if (zn) {
      const float c = g.A[(j + 1) * s + j];
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[r] = fmaf(c, zn[r], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = fmaf(h, acc[r], g.b[j] * lam[r]);
    const uint2 q = pack4<T>(v);
    bad = bad || any_nonfinite4<T>(q);
    lds_store_u2(&lds.zbuf[m * Sh::ldz + n], q);
    if (row < g.R) *group4(KBART, g.ldk, (int64_t)j * g.Rp + row, n) = q;
  };

  if (!g.skip_recompute) {
    // ---- stage recomputation from the stored state, keeping inputs and activations
    eng.template preload_hidden<true>(g.layer[0].Wf);
    eng.for_state([&](int n, int m) {
      const uint2 q = load4h(ck, row0 + m, g.R, n, D);
      lds_store_u2(&lds.zbuf[m * Sh::ldz + n], q);
      if (row0 + m < g.R) *group4(ZT, g.ldk, row0 + m, n) = q;
    });
    __syncthreads();
    for (int j = 0; j < s; ++j) {
      const float tau = st[1 + j];
      wide_hidden_layers<T, HP, D, true>(eng, lds, g, j, tau, row0, set_off);
      const lds_f32* bias = lds.param + g.layer[L - 1].bias_off;
      auto epi_last = [&](const f32x16& acc, int n_tile, int rt) {
        const int m = rt * 32 + fresh(eng.lr), lh4 = 4 * fresh(eng.lh);
        const int64_t row = row0 + m;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n_tile + 8 * q + lh4;
          if (j + 1 < s) {
            const float4 bv = lds_load_f4(&bias[n]);
            const float v[4] = {acc[4 * q] + bv.x, acc[4 * q + 1] + bv.y, acc[4 * q + 2] + bv.z, acc[4 * q + 3] + bv.w};
            const uint2 kq = pack4<T>(v);
            float kf[4], incr[4] = {0.f, 0.f, 0.f, 0.f}, yh[4], z[4];
            unpack4<T>(kq, kf);
            store4h(g.K + (size_t)j * g.stage_stride, row, g.R, n, D, kq);
            for (int l = 0; l < j; ++l) {
              const float a = g.A[(j + 1) * s + l];
              if (a != 0.f) {
                float kl[4];
                unpack4<T>(load4h(g.K + (size_t)l * g.stage_stride, row, g.R, n, D), kl);
#pragma unroll
                for (int r = 0; r < 4; ++r) incr[r] = fmaf(a, kl[r], incr[r]);
              }
            }
            const float aj = g.A[(j + 1) * s + j];
            unpack4<T>(load4h(ck, row, g.R, n, D), yh);
#pragma unroll
            for (int r = 0; r < 4; ++r) z[r] = fmaf(h, fmaf(aj, kf[r], incr[r]), yh[r]);
            const uint2 zq = pack4<T>(z);
            lds_store_u2(&lds.zbuf[m * Sh::ldz + n], zq);
            if (row < g.R) *group4(ZT, g.ldk, (int64_t)(j + 1) * g.Rp + row, n) = zq;
          } else {
            make_kbar(s - 1, m, n, nullptr);  // the slope of the last stage is not needed again
          }
        }
      };
      auto nxt_last = [&]() {
        if (j + 1 < s) eng.template preload_hidden<true>(g.layer[0].Wf);
        else eng.template preload_hidden<true>(g.layer[L - 1].WTf);
      };
      eng.run_state(g.layer[L - 1].Wf, lds.x(L - 2), epi_last, nxt_last);
    }
  } else {
    eng.template preload_hidden<true>(g.layer[L - 1].WTf);
    eng.for_state([&](int n, int m) { make_kbar(s - 1, m, n, nullptr); });
    __syncthreads();
  }

  // ---- cotangent chain, stages in reverse (eq. (vjp) pushed through the stage recursion)
  for (int j = s - 1; j >= 0; --j) {
    const int64_t kj = (int64_t)j * g.Rp + row0;
    for (int l = L - 1; l >= 1; --l) {
      const int q = L - 1 - l;  // number of this transposed pass within the chain
      const uint16_t* actT = g.ACTT[l - 1] + set_off;
      uint16_t* goutT = g.DELTAT[l - 1] + set_off;
      lds_u16* out = lds.x(q);
      const u16x8* Wnext = g.layer[l - 1].WTf;
      const bool next_is_last = (l == 1);
      auto epi_delta = [&](const f32x16& acc, int n_tile, int rt) {
        const int m = rt * 32 + fresh(eng.lr), lh4 = 4 * fresh(eng.lh);
        const bool live = row0 + m < g.R;
        uint2 aq[4];
#pragma unroll
        for (int qd = 0; qd < 4; ++qd)
          aq[qd] = live ? *group4(const_cast<uint16_t*>(actT), g.ldk, kj + m, n_tile + 8 * qd + lh4) : make_uint2(0u, 0u);
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const int n = n_tile + 8 * qd + lh4;
          float a[4], v[4];
          unpack4<T>(aq[qd], a);
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[4 * qd + r] * (1.f - a[r] * a[r]);
          const uint2 dq = pack4<T>(v);
          lds_store_u2(&out[m * Sh::ldp + n], dq);
          if (live) {
            *group4(goutT, g.ldk, kj + m, n) = dq;
            bad = bad || any_nonfinite4<T>(dq);
          }
        }
      };
      auto nxt_b = [&]() {
        if (next_is_last) eng.preload_state(Wnext);
        else eng.template preload_hidden<false>(Wnext);
      };
      if (q == 0) eng.template run_hidden<true>(g.layer[l].WTf, lds.zbuf, epi_delta, nxt_b);
      else eng.template run_hidden<false>(g.layer[l].WTf, lds.x(q - 1), epi_delta, nxt_b);
    }
    auto epi_zbar = [&](const f32x16& acc, int n_tile, int rt) {
      const int m = rt * 32 + fresh(eng.lr), lh4 = 4 * fresh(eng.lh);
      const int64_t row = row0 + m;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n_tile + 8 * q + lh4;
        const float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        const uint2 zq = pack4<T>(v);
        if (row < g.R) bad = bad || any_nonfinite4<T>(zq);
        store4h(g.ZBAR + (size_t)j * g.stage_stride, row, g.R, n, D, zq);
        if (j > 0) {
          float zf[4];
          unpack4<T>(zq, zf);
          make_kbar(j - 1, m, n, zf);
        }
      }
    };
    auto nxt_z = [&]() {
      if (j > 0) eng.template preload_hidden<true>(g.layer[L - 1].WTf);
    };
    eng.run_state(g.layer[0].WTf, lds.x(L - 2), epi_zbar, nxt_z);
  }

  // ---- a <- a + (h / S) sum_j zbar_j (+ running-cost cotangent), fp32; max |a|
  // (every lane reads back exactly the stage cotangents it wrote itself)
  unsigned bits = 0;
  const float hs = h / S;
  eng.for_state([&](int n, int m) {
    const int64_t row = row0 + m;
    float a[4], da[4] = {0.f, 0.f, 0.f, 0.f}, gy[4] = {0.f, 0.f, 0.f, 0.f};
    load4f(g.a_in, row, g.R, n, D, a);
    for (int j = s - 1; j >= 0; --j) {
      float zf[4];
      unpack4<T>(load4h(g.ZBAR + (size_t)j * g.stage_stride, row, g.R, n, D), zf);
#pragma unroll
      for (int r = 0; r < 4; ++r) da[r] += zf[r];
    }
    if (g.gys) load4f(g.gys, row, g.R, n, D, gy);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      a[r] = fmaf(hs, da[r], a[r]) + gy[r];
      if (g.round_incr & 2) a[r] = Low<T>::to_f32(Low<T>::from_f32(a[r]));
      const unsigned bb = __builtin_bit_cast(unsigned, fabsf(a[r]));
      if (row < g.R) bits = bb > bits ? bb : bits;
    }
    store4f(g.a_out, row, g.R, n, D, a);
  });

  if (g.detect) raise_if_any(bad, g.ctl);
  block_amax(bits, &g.ctl->amax_bits);

  // ---- the last workgroup to get here takes the decision of this step (accept / grow, or poison)
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
      g.scale_hist[g.step] = S;
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
