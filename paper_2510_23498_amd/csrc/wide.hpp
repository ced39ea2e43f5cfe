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


// A value the optimiser must treat as new at this point.  The epilogues derive every per-lane address
// offset from laundered lane coordinates: otherwise all their (loop-invariant) addresses are computed
// once at kernel entry and kept alive -- or spilled -- across the contraction loops.
__device__ __forceinline__ int fresh(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

// Forces a wave-uniform value into scalar registers HERE (the kernel arguments live in memory: without
// this the tableau coefficients are fetched, and waited for, inside every unrolled piece of an epilogue).
__device__ __forceinline__ float pinned(float x) {
  asm volatile("" : "+s"(x));
  return x;
}
__device__ __forceinline__ int pinned(int x) {
  asm volatile("" : "+s"(x));
  return x;
}

// Marks a point at which loaded values must have arrived.  Used right after a contraction, when no
// younger load is outstanding, and BEFORE the next pass's weight fragments are requested: the load
// counter completes in order, so a wait placed after that request (and in branchy code the compiler
// places a full one) would also wait for the fragments.
__device__ __forceinline__ void arrived(const float4& v) { asm volatile("" ::"v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w)); }
__device__ __forceinline__ void arrived(const uint2& v) { asm volatile("" ::"v"(v.x), "v"(v.y)); }

constexpr int kWideWaves = 8;
constexpr int kWidePD = 8;  // contraction steps (of 16) of weight fragments in flight per wavefront

// Exponent fields of the two 16-bit values packed in a word: all ones = inf or NaN.  (w & mask) + carry
// sets bit 15 / bit 31 exactly for such a half (no carry crosses the halves), so overflow detection is
// one and-add-or per PAIR of values, accumulated over an epilogue and tested once.
template <class T> struct LowPair;
template <> struct LowPair<F16> { static constexpr uint32_t mask = 0x7C007C00u, carry = 0x04000400u; };
template <> struct LowPair<BF16> { static constexpr uint32_t mask = 0x7F807F80u, carry = 0x00800080u; };
template <class T>
__device__ __forceinline__ void note_nonfinite(uint32_t& nf, uint2 q) {
  nf |= (q.x & LowPair<T>::mask) + LowPair<T>::carry;
  nf |= (q.y & LowPair<T>::mask) + LowPair<T>::carry;
}
__device__ __forceinline__ bool saw_nonfinite(uint32_t nf) { return (nf & 0x80008000u) != 0u; }

// tanh of an fp32 pre-activation (see tanh_fast), as the hidden epilogues use it
__device__ __forceinline__ float wide_tanh(float x) {
  const float e = __builtin_amdgcn_exp2f(2.885390081777927f * x);
  return fmaf(-2.f, __builtin_amdgcn_rcpf(e + 1.f), 1.f);
}

// Addresses = wave-uniform part (scalar registers) + a 32-bit per-lane byte offset.
//   feature-group-major arrays: the 8-byte word of features n_u + 4 * lh .. + 3 at contraction index
//   k_u + m is at  XT + ((n_u / 4) * ldk + k_u) * 4 elements  +  (lh * ldk + m) * 8 bytes;
//   row-major state arrays [R][D]: features n_u + 4 * lh .. of row row0 + m at
//   P + (row0 * D + n_u) elements  +  (m * D + 4 * lh) * sizeof(element) bytes.
__device__ __forceinline__ uint2* fm_word(uint16_t* XT, int64_t ldk, int64_t k_u, int n_u, uint32_t lane_off) {
  return reinterpret_cast<uint2*>(reinterpret_cast<char*>(XT + ((size_t)(n_u >> 2) * ldk + k_u) * 4) + lane_off);
}
template <class E>
__device__ __forceinline__ E* st_word(E* P, int64_t row0, int D, int n_u, uint32_t lane_off) {
  return (E*)((const char*)(P + (size_t)row0 * D + n_u) + lane_off);
}
__device__ __forceinline__ uint2 ld_h4(const uint16_t* p) { return *reinterpret_cast<const uint2*>(p); }
__device__ __forceinline__ void st_h4(uint16_t* p, uint2 q) { *reinterpret_cast<uint2*>(p) = q; }
__device__ __forceinline__ float4 ld_f4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st_f4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }

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
// KS steps of 16.  Weight fragments are addressed as a wave-uniform fragment index (scalar registers:
// step * CT + column tile, 1 KB each) plus the lane's 16 bytes, so that no load needs an address
// register of its own.  `ab` is the lane's LDS address in row tile 0: row lane % 32, element
// (lane / 32) * 8.  On entry ring[u] holds steps u < min(PD, KS) (requested by the previous pass) and
// acc its initial value (the bias of a forward layer, zero for a transposed one).
// (buffer loads: resource descriptor in scalar registers = base + size of one layer's fragments, so
// a fragment outside it would read as zero; scalar byte offset of the fragment; the lane's 16 bytes)
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
struct WideW {
  __amdgpu_buffer_rsrc_t rsrc;
};
__device__ __forceinline__ WideW wide_weights(const u16x8* W, int Kpad, int Npad) {
  WideW w;
  w.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<u16x8*>(W), 0, Kpad * Npad * 2, 0x00020000);
  return w;
}
__device__ __forceinline__ u16x8 wide_frag(const WideW& W, int frag, uint32_t lane16) {
  return __builtin_bit_cast(u16x8, __builtin_amdgcn_raw_buffer_load_b128(W.rsrc, (int)lane16, frag * 1024, 0));
}

template <int NCT, int PD>
__device__ __forceinline__ void wide_preload(u16x8 (&ring)[PD][2], const WideW& W, int ct0, uint32_t lane16, int KS, int CT) {
#pragma unroll
  for (int u = 0; u < PD; ++u) {
    const int ks = u < KS ? u : KS - 1;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) ring[u][ct] = wide_frag(W, ks * CT + ct0 + ct, lane16);
  }
}

// BD: contraction steps by which the activation fragments (LDS) are read ahead of their matrix
// instructions: 1 when a step has 4 matrix instructions to hide the read behind, more when it has 1.
// hook(): global loads whose results are only needed after the contraction.  The load counter of a
// wavefront completes in order, so a long-latency load issued BEFORE the loop would stall the first
// wait for a refilled ring slot (step PD) until it has returned; issued after the first PD steps it
// is younger than their refills and only has to be back by step 2 PD (long contractions), or by the
// epilogue (contractions of at most PD steps, which have no refills at all).
template <class T, int NCT, int NRT, int KS, int CT, int PD, int BD, class Hook>
__device__ __forceinline__ void wide_mma(f32x16 (&acc)[NCT][NRT], u16x8 (&ring)[PD][2], const WideW& W, int ct0,
                                         uint32_t lane16, const lds_u16* ab, int rt_stride, Hook hook) {
  // (rt_stride: elements between the LDS rows of consecutive row tiles)
  static_assert(PD % 2 == 0 && (KS <= PD || KS % PD == 0), "pipeline depth");
  constexpr int NB = BD == 1 ? 2 : 4;  // activation fragment buffers (a power of two dividing PD)
  static_assert(BD < NB && PD % NB == 0 && KS >= BD, "activation lookahead");
  u16x8 b[NB][NRT];
#pragma unroll
  for (int u = 0; u < BD; ++u)
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) b[u][rt] = *(const lds_u16x8*)(ab + rt * rt_stride + u * 16);
  constexpr int MAIN = KS > PD ? KS - PD : 0;
  if constexpr (MAIN == 0) hook();
#pragma unroll 1
  for (int ks0 = 0; ks0 < MAIN; ks0 += PD) {
    if (ks0 == PD || (MAIN == PD && ks0 == 0)) hook();
    const lds_u16* an = ab + (ks0 + BD) * 16;
#pragma unroll
    for (int u = 0; u < PD; ++u) {
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) b[(u + BD) % NB][rt] = *(const lds_u16x8*)(an + rt * rt_stride + u * 16);
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) acc[ct][rt] = Low<T>::mfma32(ring[u][ct], b[u % NB][rt], acc[ct][rt]);
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct) ring[u][ct] = wide_frag(W, (ks0 + PD + u) * CT + ct0 + ct, lane16);
      // issue order within the step: the activation fragments of a later step first (their latency
      // hides behind matrix instructions), then this step's matrix instructions, then the refill of
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
    if (u + BD < TAIL) {
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) b[(u + BD) % NB][rt] = *(const lds_u16x8*)(ab + rt * rt_stride + (MAIN + u + BD) * 16);
    }
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) acc[ct][rt] = Low<T>::mfma32(ring[u][ct], b[u % NB][rt], acc[ct][rt]);
  }
}

// Shapes of a network with state width D and hidden width HP on a 64-row tile, 8 wavefronts.
//   hidden-shaped output: wavefront w owns column tiles 2w, 2w + 1 (of 32), both row tiles;
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

// The per-wavefront engine: lane coordinates, the weight ring, and the pass drivers.  A pass is
//   init(n) -> float4   initial accumulator values of output features n .. n + 3 (a forward layer's
//                       bias -- the matrix instructions then add the products on top, so the
//                       epilogue has no bias to fetch -- or zero),
//   pre()               issues the global loads the epilogue will need, BEFORE the contraction, so
//                       that their latency hides behind it,
//   the contraction,
//   nxt()               requests the first weight fragments of the next pass,
//   epi(acc, n_tile, ct, rt) per 32 x 32 output tile (ct, rt: the tile's index within the wavefront's
//                       tiles, compile-time constants after unrolling),
//   a workgroup barrier.
template <class T, int HP, int D>
struct WideEngine {
  using Sh = WideShape<HP, D>;
  static constexpr int PD = kWidePD;
  u16x8 ring[PD][2];
  int lane, wave, lr, lh;  // wave: wave-uniform; lr = lane % 32 (batch row within a row tile), lh = lane / 32
  uint32_t lane16;         // the lane's byte offset within a 1 KB weight fragment

  __device__ __forceinline__ void setup() {
    lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    lr = lane & 31;
    lh = lane >> 5;
    lane16 = (uint32_t)lane * 16u;
  }
  // request the first fragments of a hidden-shaped pass (contraction over the state: KS_S, else KS_H)
  // A pass whose whole contraction fits the ring (over a state of 128: 8 steps; the split state-shaped
  // pass: 16 single fragments) is requested in two parts: 5 of 8 steps (12 of 16 fragments) ahead, during
  // the previous pass's epilogue, and the rest by the pass itself before its first matrix instruction
  // -- the epilogue's own values and a full ring together are more registers than a wavefront has, and
  // a fragment that is spilled has to be waited for right where it was requested (with these counts
  // neither kernel spills).
  static constexpr int KS_S_AHEAD = (Sh::KS_S <= PD) ? (5 * Sh::KS_S) / 8 : PD;
  template <bool FROM_STATE>
  __device__ __forceinline__ void preload_hidden(const WideW& W) {
    if constexpr (FROM_STATE && Sh::KS_S <= PD) {
#pragma unroll
      for (int u = 0; u < KS_S_AHEAD; ++u)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) ring[u][ct] = wide_frag(W, u * Sh::CT_H + 2 * wave + ct, lane16);
    } else {
      wide_preload<2, PD>(ring, W, 2 * wave, lane16, FROM_STATE ? Sh::KS_S : Sh::KS_H, Sh::CT_H);
    }
  }
  template <bool FROM_STATE>
  __device__ __forceinline__ void preload_hidden_rest(const WideW& W) {
    if constexpr (FROM_STATE && Sh::KS_S <= PD) {
#pragma unroll
      for (int u = KS_S_AHEAD; u < Sh::KS_S; ++u)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) ring[u][ct] = wide_frag(W, u * Sh::CT_H + 2 * wave + ct, lane16);
    }
  }
  // State-shaped passes.  D = 256: wavefront w owns column tile w and both row tiles.  D = 128 has
  // only 4 column tiles: wavefronts w and w + 4 share column tile w % 4 and SPLIT THE CONTRACTION
  // (k-steps [16 (w / 4), + 16)) over both row tiles -- so that every weight fragment is fetched once,
  // not by two wavefronts --, then hand each other the partial sums of the row tile the other one
  // finishes (row tile w / 4) through LDS.
  static constexpr bool kSplitK = (D == 128);
  static constexpr int KS_ST = kSplitK ? Sh::KS_H / 2 : Sh::KS_H;
  __device__ __forceinline__ int state_frag0() const { return kSplitK ? (wave >> 2) * KS_ST * Sh::CT_S + (wave & 3) : wave; }
  // (split contraction: a wavefront's 16 fragments fill the ring, slot u at ring[u % PD][u / PD], so the
  // pass has no refills and nothing in it waits for loads issued after this request)
  static constexpr int KS_ST_AHEAD = kSplitK ? (3 * KS_ST) / 4 : PD;
  __device__ __forceinline__ void preload_state_rest(const WideW& W) {
    if constexpr (kSplitK) {
#pragma unroll
      for (int u = KS_ST_AHEAD; u < KS_ST; ++u) ring[u % PD][u / PD] = wide_frag(W, state_frag0() + u * Sh::CT_S, lane16);
    }
  }
  __device__ __forceinline__ void preload_state(const WideW& W) {
    if constexpr (kSplitK) {
      static_assert(KS_ST == 2 * PD, "the ring holds a state-shaped pass");
#pragma unroll
      for (int u = 0; u < KS_ST_AHEAD; ++u) ring[u % PD][u / PD] = wide_frag(W, state_frag0() + u * Sh::CT_S, lane16);
    } else {
      wide_preload<1, PD>(ring, W, state_frag0(), lane16, KS_ST, Sh::CT_S);
    }
  }

  // What a hidden-shaped pass requests for the pass after it: a state-shaped pass (state_next) or
  // another hidden-shaped one over the hidden width.  ONE sequence of loads with selected fragment
  // numbers -- two branches that fill different ring slots make the compiler keep ring slots in memory.
  __device__ __forceinline__ void preload_after_hidden(const WideW& W, bool state_next) {
    if constexpr (kSplitK) {
      const int st0 = state_frag0();
#pragma unroll
      for (int u = 0; u < PD; ++u)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          const int v = ct * PD + u;  // the state-shaped pass's step held by ring[u][ct]
          const int frag = state_next ? st0 + v * Sh::CT_S : u * Sh::CT_H + 2 * wave + ct;
          if (v < KS_ST_AHEAD) ring[u][ct] = wide_frag(W, frag, lane16);
          else if (!state_next) ring[u][ct] = wide_frag(W, frag, lane16);
        }
    } else {
      if (state_next) preload_state(W);
      else preload_hidden<false>(W);
    }
  }

  template <bool FROM_STATE, class Init, class Pre, class Arr, class Epi, class Nxt, class Tail>
  __device__ __forceinline__ void run_hidden(const WideW& W, const lds_u16* in, Init init, Pre pre, Arr arr, Epi epi, Nxt nxt,
                                             Tail tail) {
    constexpr int KS = FROM_STATE ? Sh::KS_S : Sh::KS_H;
    constexpr int ld = FROM_STATE ? Sh::ldz : Sh::ldp;
    preload_hidden_rest<FROM_STATE>(W);
    f32x16 acc[2][2];
    {
      const int lh4 = 4 * fresh(lh);
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 v = init((2 * wave + ct) * 32 + 8 * q + lh4);
#pragma unroll
          for (int rt = 0; rt < 2; ++rt) {
            acc[ct][rt][4 * q] = v.x; acc[ct][rt][4 * q + 1] = v.y;
            acc[ct][rt][4 * q + 2] = v.z; acc[ct][rt][4 * q + 3] = v.w;
          }
        }
    }
    wide_mma<T, 2, 2, KS, Sh::CT_H, PD, 1>(acc, ring, W, 2 * wave, lane16, in + lr * ld + lh * 8, 32 * ld, pre);
    arr();
    nxt();
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) epi(acc[ct][rt], (2 * wave + ct) * 32, ct, rt);
    tail();
    __syncthreads();
  }
  // state-shaped pass (contraction over the hidden width); epi's rt counts the wavefront's own row
  // tiles; xchg: 32 KB of LDS that nothing else uses during the pass (the partial sums of D = 128 travel
  // through it): the activation buffer the pass does not read
  template <class Init, class Pre, class Epi, class Nxt>
  __device__ __forceinline__ void run_state(const WideW& W, const lds_u16* in, lds_u16* xchg, Init init, Pre pre, Epi epi,
                                            Nxt nxt) {
    // pre(): the pass's global loads were issued at the end of the previous epilogue; this marks the point
    // (after the contraction) where they must be back
    preload_state_rest(W);
    const int lh4 = 4 * fresh(lh);
    if constexpr (kSplitK) {
      const int kh = wave >> 2, ct = wave & 3;
      f32x16 acc[1][2];  // [0][0]: the row tile this wavefront finishes (kh), [0][1]: the other one
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 v = init(ct * 32 + 8 * q + lh4);
        if (kh != 0) v = make_float4(0.f, 0.f, 0.f, 0.f);  // the bias enters once
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          acc[0][rt][4 * q] = v.x; acc[0][rt][4 * q + 1] = v.y;
          acc[0][rt][4 * q + 2] = v.z; acc[0][rt][4 * q + 3] = v.w;
        }
      }
      {
        const lds_u16* ab = in + (kh * 32 + lr) * Sh::ldp + kh * KS_ST * 16 + lh * 8;
        const int rt_stride = kh ? -32 * Sh::ldp : 32 * Sh::ldp;
        u16x8 b[4][2];
#pragma unroll
        for (int u = 0; u < 3; ++u)
#pragma unroll
          for (int rt = 0; rt < 2; ++rt) b[u][rt] = *(const lds_u16x8*)(ab + rt * rt_stride + u * 16);
#pragma unroll
        for (int u = 0; u < KS_ST; ++u) {
          if (u + 3 < KS_ST) {
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) b[(u + 3) % 4][rt] = *(const lds_u16x8*)(ab + rt * rt_stride + (u + 3) * 16);
          }
#pragma unroll
          for (int rt = 0; rt < 2; ++rt) acc[0][rt] = Low<T>::mfma32(ring[u % PD][u / PD], b[u % 4][rt], acc[0][rt]);
        }
      }
      pre();
      nxt();
      // partial sums of the other row tile -> LDS, [wavefront][4][lane] x 16 B
      // (indexed by the lane's fragment byte offset, the one per-lane value that is live in every pass)
      RAMPDE_LDS f32x4* xq = (RAMPDE_LDS f32x4*)((RAMPDE_LDS char*)xchg + lane16);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        xq[(wave * 4 + q) * 64] = f32x4{acc[0][1][4 * q], acc[0][1][4 * q + 1], acc[0][1][4 * q + 2], acc[0][1][4 * q + 3]};
      __syncthreads();
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 o = xq[((wave ^ 4) * 4 + q) * 64];
        acc[0][0][4 * q] += o[0]; acc[0][0][4 * q + 1] += o[1];
        acc[0][0][4 * q + 2] += o[2]; acc[0][0][4 * q + 3] += o[3];
      }
      epi(acc[0][0], ct * 32, 0);
    } else {
      f32x16 acc[1][2];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = init(wave * 32 + 8 * q + lh4);
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          acc[0][rt][4 * q] = v.x; acc[0][rt][4 * q + 1] = v.y;
          acc[0][rt][4 * q + 2] = v.z; acc[0][rt][4 * q + 3] = v.w;
        }
      }
      wide_mma<T, 1, 2, KS_ST, Sh::CT_S, PD, 2>(acc, ring, W, state_frag0(), lane16, in + lr * Sh::ldp + lh * 8, 32 * Sh::ldp,
                                                []() {});
      pre();
      nxt();
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) epi(acc[0][rt], wave * 32, rt);
    }
    __syncthreads();
  }
  // The state elements of this lane, as the state-shaped passes see them: for its row tile(s) rt and the
  // four runs q of 4 features, f(rt, q, n_u, m) with n_u the wave-uniform first feature of the run of
  // lane half 0 (the lane's own run starts at n_u + 4 * lh) and m the row within the tile.
  template <class F>
  __device__ __forceinline__ void for_state(F f) const {
    const int r = fresh(lr);
#pragma unroll
    for (int rt = 0; rt < Sh::S_NRT; ++rt)
#pragma unroll
      for (int q = 0; q < 4; ++q) f(rt, q, Sh::s_ct(wave) * 32 + 8 * q, (Sh::s_rt0(wave) + rt) * 32 + r);
  }
  // per-lane byte offsets of the addressing helpers, for row m of the tile
  __device__ __forceinline__ uint32_t fm_off(int64_t ldk, int m) const { return ((uint32_t)fresh(lh) * (uint32_t)ldk + (uint32_t)m) * 8u; }
  template <class E>
  __device__ __forceinline__ uint32_t st_off(int m) const { return ((uint32_t)m * D + 4u * (uint32_t)fresh(lh)) * (uint32_t)sizeof(E); }
};

__device__ __forceinline__ float4 zero4(int) { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ WideW fwd_weights(const FusedArgs& g, int l) {
  return wide_weights(g.layer[l].Wf, g.layer[l].Kpad, g.layer[l].Npad);
}
__device__ __forceinline__ WideW bwd_weights(const FusedArgs& g, int l) {
  return wide_weights(g.layer[l].WTf, g.layer[l].Kpad, g.layer[l].Npad);
}

// hidden layers of one velocity evaluation (all layers but the last), stage j.  KEEP: the
// activations also go to the feature-group-major buffers (adjoint recomputation).
// state_loads(): issued at the end of the LAST hidden layer's epilogue: the global loads of the
// state-shaped pass that follows (they are back by the time its short contraction is done).
template <class T, int HP, int D, bool KEEP, class StateLoads>
__device__ __forceinline__ void wide_hidden_layers(WideEngine<T, HP, D>& eng, const WideLds<HP, D>& lds, const FusedArgs& g,
                                                   int j, float tau, int64_t row0, int64_t set_off, StateLoads state_loads) {
  using Sh = WideShape<HP, D>;
  for (int l = 0; l + 1 < g.L; ++l) {
    const lds_f32* bias = lds.param + g.layer[l].bias_off;
    const lds_f32* wt = lds.param + g.wt_off;
    const bool has_wt = (l == 0);
    lds_u16* out = lds.x(l);
    uint16_t* goutT = KEEP ? g.ACTT[l] + set_off : nullptr;
    const int64_t kj = (int64_t)j * g.Rp + row0;
    const WideW Wnext = fwd_weights(g, l + 1), Wthis = fwd_weights(g, l);
    const bool next_is_last = (l + 2 == g.L);
    // pre-activation = bias (+ time column * tau) + products: the first two are the accumulator's start
    auto init = [&](int n) {
      float4 v = lds_load_f4(&bias[n]);
      if (has_wt) {
        const float4 tv = lds_load_f4(&wt[n]);
        v.x = fmaf(tv.x, tau, v.x); v.y = fmaf(tv.y, tau, v.y);
        v.z = fmaf(tv.z, tau, v.z); v.w = fmaf(tv.w, tau, v.w);
      }
      return v;
    };
    auto pre = []() {};
    auto epi = [&](const f32x16& acc, int n_tile, int, int rt) {
      const int m = rt * 32 + fresh(eng.lr), lh4 = 4 * fresh(eng.lh);
      const bool live = KEEP && row0 + m < g.R;
      const uint32_t goff = KEEP ? eng.fm_off(g.ldk, m) : 0u;
      lds_u16* orow = out + m * Sh::ldp + n_tile + lh4;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = wide_tanh(acc[4 * q + r]);
        const uint2 pq = pack4<T>(v);
        lds_store_u2(orow + 8 * q, pq);
        // (rows past the batch exist in the feature-group-major buffers and must hold zeros; storing
        // without a branch keeps the 16 runs of this tile in one block for the scheduler)
        if (KEEP) *fm_word(goutT, g.ldk, kj, n_tile + 8 * q, goff) = live ? pq : make_uint2(0u, 0u);
      }
    };
    auto nxt = [&]() { eng.preload_after_hidden(Wnext, next_is_last); };
    auto tail = [&]() {
      if (next_is_last) state_loads();
    };
    if (l == 0) eng.template run_hidden<true>(Wthis, lds.zbuf, init, pre, pre, epi, nxt, tail);
    else eng.template run_hidden<false>(Wthis, lds.x(l - 1), init, pre, pre, epi, nxt, tail);
  }
}

// The stage arithmetic both kernels share, for one run of 4 state elements:
//   increment of the next stage input from earlier slopes other than k_j (only tableaux with
//   a_{j+1,l} != 0 for some l < j pay for these loads: not Euler, Heun or classic RK4)
template <class T, int D>
__device__ __forceinline__ void earlier_slopes(const FusedArgs& g, int dense, int j, int64_t row0, int n_u, uint32_t hoff,
                                               float (&incr)[4]) {
  if (!dense) return;
  for (int l = 0; l < j; ++l) {
    const float a = g.A[(j + 1) * g.s + l];
    if (a != 0.f) {
      float kl[4];
      unpack4<T>(ld_h4(st_word(g.K + (size_t)l * g.stage_stride, row0, D, n_u, hoff)), kl);
#pragma unroll
      for (int r = 0; r < 4; ++r) incr[r] = fmaf(a, kl[r], incr[r]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Forward pass, all steps in one launch (paper Algorithm 1).
// g.bsum ([R][D] fp32) carries the running sum  sum_{l <= j} b_l k_l  of the step from stage to stage
// (same order of fp32 operations as summing at the end), so that the last stage needs one load, not s - 1.
template <class T, int HP, int D>
__global__ __launch_bounds__(64 * kWideWaves) void mlp_forward_wide(FusedArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  using Sh = WideShape<HP, D>;
  const WideLds<HP, D> lds((lds_u16*)smem, g);
  WideEngine<T, HP, D> eng;
  eng.setup();
  const int64_t row0 = (int64_t)blockIdx.x * Sh::TM;
  const int64_t n_state = g.R * D;
  const int L = g.L, s = g.s;
  const int dense = pinned(g.dense_tableau);

  load_params(lds.param, g);
  // y <- y0 (kept in the output buffer), first stored state, first stage input
  eng.for_state([&](int, int, int n_u, int m) {
    const bool live = row0 + m < g.R;
    const uint32_t foff = eng.template st_off<float>(m), hoff = eng.template st_off<uint16_t>(m);
    float4 y4 = live ? ld_f4(st_word(g.y0, row0, D, n_u, foff)) : make_float4(0.f, 0.f, 0.f, 0.f);
    float v[4] = {y4.x, y4.y, y4.z, y4.w};
    const uint2 q = pack4<T>(v);
    if (g.round_incr & 2) unpack4<T>(q, v);
    if (live) {
      st_f4(st_word(g.y, row0, D, n_u, foff), make_float4(v[0], v[1], v[2], v[3]));
      st_h4(st_word(g.ckpt, row0, D, n_u, hoff), q);
    }
    lds_store_u2(&lds.zbuf[m * Sh::ldz + n_u + 4 * eng.lh], q);
  });
  __syncthreads();

  eng.template preload_hidden<true>(fwd_weights(g, 0));
  for (int i = 0; i < g.N; ++i) {
    const float* st = g.steptab + (size_t)i * (1 + s);
    const float h = st[0];
    const uint16_t* ck = g.ckpt + (size_t)i * n_state;
    uint16_t* ck_next = g.ckpt + (size_t)(i + 1) * n_state;
    for (int j = 0; j < s; ++j) {
      const float tau = st[1 + j];
      const bool more = (j + 1 < s) || (i + 1 < g.N);
      const bool last_stage = (j + 1 == s);
      const float bj = pinned(g.b[j]), aj = pinned(last_stage ? 0.f : g.A[(j + 1) * s + j]);
      const lds_f32* bias = lds.param + g.layer[L - 1].bias_off;
      // what the last layer's epilogue reads back: the stored state (next stage input) or the fp32
      // state (update), and the running b-weighted sum of the slopes
      // (yv: the fp32 state at the last stage; otherwise .x/.y carry the bits of the stored state)
      float4 yv[Sh::S_NRT][4], bs[Sh::S_NRT][4];
      auto state_loads = [&]() {
        eng.for_state([&](int rt, int q, int n_u, int m) {
          const bool live = row0 + m < g.R;
          const uint32_t foff = eng.template st_off<float>(m), hoff = eng.template st_off<uint16_t>(m);
          yv[rt][q] = bs[rt][q] = make_float4(0.f, 0.f, 0.f, 0.f);
          if (live) {
            if (last_stage) {
              yv[rt][q] = ld_f4(st_word(g.y, row0, D, n_u, foff));
            } else {
              const uint2 w = ld_h4(st_word(ck, row0, D, n_u, hoff));
              yv[rt][q].x = __builtin_bit_cast(float, w.x);
              yv[rt][q].y = __builtin_bit_cast(float, w.y);
            }
            if (j > 0) bs[rt][q] = ld_f4(st_word(g.bsum, row0, D, n_u, foff));
          }
        });
      };
      wide_hidden_layers<T, HP, D, false>(eng, lds, g, j, tau, row0, 0, state_loads);
      auto init = [&](int n) { return lds_load_f4(&bias[n]); };
      auto pre = [&]() {
#pragma unroll
        for (int rt = 0; rt < Sh::S_NRT; ++rt)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            arrived(yv[rt][q]);
            arrived(bs[rt][q]);
          }
      };
      auto epi_last = [&](const f32x16& acc, int n_tile, int rt) {
        const int m = (Sh::s_rt0(eng.wave) + rt) * 32 + fresh(eng.lr);
        const bool live = row0 + m < g.R;
        const uint32_t foff = eng.template st_off<float>(m), hoff = eng.template st_off<uint16_t>(m);
        lds_u16* zrow = lds.zbuf + m * Sh::ldz + n_tile + 4 * fresh(eng.lh);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n_u = n_tile + 8 * q;
          const float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
          const uint2 kq = pack4<T>(v);
          float kf[4];
          unpack4<T>(kq, kf);
          float sum[4] = {bs[rt][q].x, bs[rt][q].y, bs[rt][q].z, bs[rt][q].w};
#pragma unroll
          for (int r = 0; r < 4; ++r) sum[r] = fmaf(bj, kf[r], sum[r]);
          uint2 zq;
          if (!last_stage) {
            // next stage input  z = Q(yhat + h * sum_l a_{j+1,l} k_l)
            float incr[4] = {0.f, 0.f, 0.f, 0.f}, yhf[4], z[4];
            if (live) {
              if (dense) st_h4(st_word(g.K + (size_t)j * g.stage_stride, row0, D, n_u, hoff), kq);
              st_f4(st_word(g.bsum, row0, D, n_u, foff), make_float4(sum[0], sum[1], sum[2], sum[3]));
              earlier_slopes<T, D>(g, dense, j, row0, n_u, hoff, incr);
            }
            unpack4<T>(make_uint2(__builtin_bit_cast(uint32_t, yv[rt][q].x), __builtin_bit_cast(uint32_t, yv[rt][q].y)), yhf);
#pragma unroll
            for (int r = 0; r < 4; ++r) z[r] = fmaf(h, fmaf(aj, kf[r], incr[r]), yhf[r]);
            zq = pack4<T>(z);
          } else {
            // y <- y + h * sum_l b_l k_l (fp32); next stored state = first stage input of the next step
            float y[4] = {yv[rt][q].x, yv[rt][q].y, yv[rt][q].z, yv[rt][q].w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              if (g.round_incr & 1) sum[r] = Low<T>::to_f32(Low<T>::from_f32(sum[r]));
              y[r] = fmaf(h, sum[r], y[r]);
            }
            zq = pack4<T>(y);
            if (g.round_incr & 2) unpack4<T>(zq, y);
            if (live) {
              st_f4(st_word(g.y, row0, D, n_u, foff), make_float4(y[0], y[1], y[2], y[3]));
              st_h4(st_word(ck_next, row0, D, n_u, hoff), zq);
            }
          }
          lds_store_u2(zrow + 8 * q, zq);
        }
      };
      auto nxt_last = [&]() {
        if (more) eng.template preload_hidden<true>(fwd_weights(g, 0));
      };
      eng.run_state(fwd_weights(g, L - 1), lds.x(L - 2), lds.x(L - 1), init, pre, epi_last, nxt_last);
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
  eng.setup();
  const int tid = threadIdx.x;
  const int64_t row0 = (int64_t)blockIdx.x * Sh::TM;
  const int L = g.L, s = g.s;
  const float S = g.ctl->S;
  const int step = g.step;
  const float* st = g.steptab + (size_t)step * (1 + s);
  const float h = st[0];
  const int64_t set_off = (int64_t)(step % g.nsets) * g.set_stride;
  uint16_t* const ZT = g.ZT + set_off;
  uint16_t* const KBART = g.KBART + set_off;
  const uint16_t* ck = g.ckpt + (size_t)step * g.ckpt_stride;
  const int dense = pinned(g.dense_tableau);
  uint32_t nf = 0;  // exponent-field carries of every low-precision cotangent this lane formed

  load_params(lds.param, g);

  // cotangent of the slope of stage j from the fp32 adjoint a4 of the lane's run of 4:
  //   kbar_j = Q( b_j lambda + h sum_{l>j} a_lj zbar_l ),  lambda = Q(S a);
  // zbar_{j+1} is still in registers (zn, or null for the last stage); later ones are read back (only
  // tableaux with a_lj != 0 for some l > j + 1 pay for these loads)
  // (bj = b_j and cj = a_{j+1,j}: fetched by the caller once per pass, not once per run of 4)
  auto make_kbar = [&](int j, float bj, float cj, float4 a4, const float* zn, int n_u, int m, bool live, uint32_t hoff,
                       uint32_t goff, lds_u16* zrow_q) {
    float a[4] = {S * a4.x, S * a4.y, S * a4.z, S * a4.w}, lam[4], acc[4] = {0.f, 0.f, 0.f, 0.f}, v[4];
    const uint2 lq = pack4<T>(a);
    note_nonfinite<T>(nf, lq);
    unpack4<T>(lq, lam);
    if (live && dense) {
      for (int l = s - 1; l > j + 1; --l) {
        const float c = g.A[l * s + j];
        if (c != 0.f) {
          float zl[4];
          unpack4<T>(ld_h4(st_word(g.ZBAR + (size_t)l * g.stage_stride, row0, D, n_u, hoff)), zl);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[r] = fmaf(c, zl[r], acc[r]);
        }
      }
    }
    if (zn) {
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[r] = fmaf(cj, zn[r], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = fmaf(h, acc[r], bj * lam[r]);
    const uint2 q = pack4<T>(v);
    note_nonfinite<T>(nf, q);
    lds_store_u2(zrow_q, q);
    if (live) *fm_word(KBART, g.ldk, (int64_t)j * g.Rp + row0, n_u, goff) = q;
  };
  // the lane's adjoint values, fetched ahead of the passes whose epilogues form a slope cotangent
  float4 av[Sh::S_NRT][4];
  auto load_adjoint = [&]() {
    eng.for_state([&](int rt, int q, int n_u, int m) {
      av[rt][q] = (row0 + m < g.R) ? ld_f4(st_word(g.a_in, row0, D, n_u, eng.template st_off<float>(m)))
                                   : make_float4(0.f, 0.f, 0.f, 0.f);
    });
  };

  if (!g.skip_recompute) {
    // ---- stage recomputation from the stored state, keeping inputs and activations
    eng.template preload_hidden<true>(fwd_weights(g, 0));
    eng.for_state([&](int, int, int n_u, int m) {
      const bool live = row0 + m < g.R;
      const uint2 q = live ? ld_h4(st_word(ck, row0, D, n_u, eng.template st_off<uint16_t>(m))) : make_uint2(0u, 0u);
      lds_store_u2(&lds.zbuf[m * Sh::ldz + n_u + 4 * eng.lh], q);
      if (live) *fm_word(ZT, g.ldk, row0, n_u, eng.fm_off(g.ldk, m)) = q;
    });
    __syncthreads();
    for (int j = 0; j < s; ++j) {
      const float tau = st[1 + j];
      const bool last_stage = (j + 1 == s);
      const float aj = pinned(last_stage ? 0.f : g.A[(j + 1) * s + j]), b_last = pinned(g.b[s - 1]);
      const lds_f32* bias = lds.param + g.layer[L - 1].bias_off;
      uint2 yh[Sh::S_NRT][4];
      auto state_loads = [&]() {
        if (last_stage) {
          load_adjoint();
        } else {
          eng.for_state([&](int rt, int q, int n_u, int m) {
            yh[rt][q] = (row0 + m < g.R) ? ld_h4(st_word(ck, row0, D, n_u, eng.template st_off<uint16_t>(m)))
                                         : make_uint2(0u, 0u);
          });
        }
      };
      wide_hidden_layers<T, HP, D, true>(eng, lds, g, j, tau, row0, set_off, state_loads);
      auto init = [&](int n) { return lds_load_f4(&bias[n]); };
      auto pre = [&]() {
#pragma unroll
        for (int rt = 0; rt < Sh::S_NRT; ++rt)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (last_stage) arrived(av[rt][q]);
            else arrived(yh[rt][q]);
          }
      };
      auto epi_last = [&](const f32x16& acc, int n_tile, int rt) {
        const int m = (Sh::s_rt0(eng.wave) + rt) * 32 + fresh(eng.lr);
        const bool live = row0 + m < g.R;
        const uint32_t hoff = eng.template st_off<uint16_t>(m), goff = eng.fm_off(g.ldk, m);
        lds_u16* zrow = lds.zbuf + m * Sh::ldz + n_tile + 4 * fresh(eng.lh);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n_u = n_tile + 8 * q;
          if (!last_stage) {
            const float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
            const uint2 kq = pack4<T>(v);
            float kf[4], incr[4] = {0.f, 0.f, 0.f, 0.f}, yhf[4], z[4];
            unpack4<T>(kq, kf);
            if (live && dense) {
              st_h4(st_word(g.K + (size_t)j * g.stage_stride, row0, D, n_u, hoff), kq);
              earlier_slopes<T, D>(g, dense, j, row0, n_u, hoff, incr);
            }
            unpack4<T>(yh[rt][q], yhf);
#pragma unroll
            for (int r = 0; r < 4; ++r) z[r] = fmaf(h, fmaf(aj, kf[r], incr[r]), yhf[r]);
            const uint2 zq = pack4<T>(z);
            lds_store_u2(zrow + 8 * q, zq);
            if (live) *fm_word(ZT, g.ldk, (int64_t)(j + 1) * g.Rp + row0, n_u, goff) = zq;
          } else {
            // (the slope of the last stage is not needed again)
            make_kbar(s - 1, b_last, 0.f, av[rt][q], nullptr, n_u, m, live, hoff, goff, zrow + 8 * q);
          }
        }
      };
      auto nxt_last = [&]() {
        if (!last_stage) eng.template preload_hidden<true>(fwd_weights(g, 0));
        else eng.template preload_hidden<true>(bwd_weights(g, L - 1));
      };
      eng.run_state(fwd_weights(g, L - 1), lds.x(L - 2), lds.x(L - 1), init, pre, epi_last, nxt_last);
    }
  } else {
    eng.template preload_hidden<true>(bwd_weights(g, L - 1));
    load_adjoint();
    const float b_last = pinned(g.b[s - 1]);
    eng.for_state([&](int rt, int q, int n_u, int m) {
      make_kbar(s - 1, b_last, 0.f, av[rt][q], nullptr, n_u, m, row0 + m < g.R, eng.template st_off<uint16_t>(m), eng.fm_off(g.ldk, m),
                lds.zbuf + m * Sh::ldz + n_u + 4 * eng.lh);
    });
    __syncthreads();
  }

  // ---- cotangent chain, stages in reverse (eq. (vjp) pushed through the stage recursion)
  for (int j = s - 1; j >= 0; --j) {
    const int64_t kj = (int64_t)j * g.Rp + row0;
    const float b_prev = pinned(j > 0 ? g.b[j - 1] : 0.f), c_prev = pinned(j > 0 ? g.A[j * s + (j - 1)] : 0.f);
    for (int l = L - 1; l >= 1; --l) {
      const int qp = L - 1 - l;  // number of this transposed pass within the chain
      uint16_t* actT = g.ACTT[l - 1] + set_off;
      uint16_t* goutT = g.DELTAT[l - 1] + set_off;
      lds_u16* out = lds.x(qp);
      const WideW Wnext = bwd_weights(g, l - 1), Wthis = bwd_weights(g, l);
      const bool next_is_last = (l == 1);
      // the stored activations of the lane's 64 outputs (tanh' = 1 - act^2), requested before the contraction
      uint2 pf[2][2][4];
      auto pre = [&]() {
        const int lrr = fresh(eng.lr);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int rt = 0; rt < 2; ++rt) {
            const int m = rt * 32 + lrr;
            const uint32_t goff = eng.fm_off(g.ldk, m);
            // (rows past the batch hold zeros in these buffers)
#pragma unroll
            for (int q = 0; q < 4; ++q) pf[ct][rt][q] = *fm_word(actT, g.ldk, kj, (2 * eng.wave + ct) * 32 + 8 * q, goff);
          }
      };
      auto epi_delta = [&](const f32x16& acc, int n_tile, int ct, int rt) {
        const int m = rt * 32 + fresh(eng.lr);
        const bool live = row0 + m < g.R;
        const uint32_t goff = eng.fm_off(g.ldk, m);
        lds_u16* orow = out + m * Sh::ldp + n_tile + 4 * fresh(eng.lh);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float a[4], v[4];
          unpack4<T>(pf[ct][rt][q], a);
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[4 * q + r] * fmaf(-a[r], a[r], 1.f);
          const uint2 dq = pack4<T>(v);
          note_nonfinite<T>(nf, dq);
          lds_store_u2(orow + 8 * q, dq);
          *fm_word(goutT, g.ldk, kj, n_tile + 8 * q, goff) = live ? dq : make_uint2(0u, 0u);
        }
      };
      auto nxt_b = [&]() { eng.preload_after_hidden(Wnext, next_is_last); };
      // (the last transposed hidden pass also fetches the adjoint for the slope cotangent that the
      // state-shaped pass after it forms)
      auto tail_b = [&]() {
        if (next_is_last && j > 0) load_adjoint();
      };
      auto arr = [&]() {
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int q = 0; q < 4; ++q) arrived(pf[ct][rt][q]);
      };
      if (qp == 0) eng.template run_hidden<true>(Wthis, lds.zbuf, zero4, pre, arr, epi_delta, nxt_b, tail_b);
      else eng.template run_hidden<false>(Wthis, lds.x(qp - 1), zero4, pre, arr, epi_delta, nxt_b, tail_b);
    }
    auto pre_z = [&]() {
      if (j > 0) {
#pragma unroll
        for (int rt = 0; rt < Sh::S_NRT; ++rt)
#pragma unroll
          for (int q = 0; q < 4; ++q) arrived(av[rt][q]);
      }
    };
    auto epi_zbar = [&](const f32x16& acc, int n_tile, int rt) {
      const int m = (Sh::s_rt0(eng.wave) + rt) * 32 + fresh(eng.lr);
      const bool live = row0 + m < g.R;
      const uint32_t hoff = eng.template st_off<uint16_t>(m), goff = eng.fm_off(g.ldk, m);
      lds_u16* zrow = lds.zbuf + m * Sh::ldz + n_tile + 4 * fresh(eng.lh);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n_u = n_tile + 8 * q;
        const float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        const uint2 zq = pack4<T>(v);
        note_nonfinite<T>(nf, zq);
        if (live) st_h4(st_word(g.ZBAR + (size_t)j * g.stage_stride, row0, D, n_u, hoff), zq);
        if (j > 0) {
          float zf[4];
          unpack4<T>(zq, zf);
          make_kbar(j - 1, b_prev, c_prev, av[rt][q], zf, n_u, m, live, hoff, goff, zrow + 8 * q);
        }
      }
    };
    auto nxt_z = [&]() {
      if (j > 0) eng.template preload_hidden<true>(bwd_weights(g, L - 1));
    };
    eng.run_state(bwd_weights(g, 0), lds.x(L - 2), lds.x(L - 1), zero4, pre_z, epi_zbar, nxt_z);
  }

  // ---- a <- a + (h / S) sum_j zbar_j (+ running-cost cotangent), fp32; max |a|
  // (every lane reads back exactly the stage cotangents it wrote itself)
  unsigned bits = 0;
  const float hs = h / S;
  eng.for_state([&](int, int, int n_u, int m) {
    const bool live = row0 + m < g.R;
    if (!live) return;
    const uint32_t foff = eng.template st_off<float>(m), hoff = eng.template st_off<uint16_t>(m);
    const float4 a4 = ld_f4(st_word(g.a_in, row0, D, n_u, foff));
    const float4 gy4 = g.gys ? ld_f4(st_word(g.gys, row0, D, n_u, foff)) : make_float4(0.f, 0.f, 0.f, 0.f);
    float a[4] = {a4.x, a4.y, a4.z, a4.w}, da[4] = {0.f, 0.f, 0.f, 0.f};
    const float gy[4] = {gy4.x, gy4.y, gy4.z, gy4.w};
    for (int jt = s - 1; jt >= 0; jt -= 4) {
      uint2 z[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        z[u] = (jt - u >= 0) ? ld_h4(st_word(g.ZBAR + (size_t)(jt - u) * g.stage_stride, row0, D, n_u, hoff)) : make_uint2(0u, 0u);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float zf[4];
        unpack4<T>(z[u], zf);
#pragma unroll
        for (int r = 0; r < 4; ++r) da[r] += zf[r];
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      a[r] = fmaf(hs, da[r], a[r]) + gy[r];
      if (g.round_incr & 2) a[r] = Low<T>::to_f32(Low<T>::from_f32(a[r]));
      const unsigned bb = __builtin_bit_cast(unsigned, fabsf(a[r]));
      bits = bb > bits ? bb : bits;
    }
    st_f4(st_word(g.a_out, row0, D, n_u, foff), make_float4(a[0], a[1], a[2], a[3]));
  });

  if (g.detect) raise_if_any(saw_nonfinite(nf), g.ctl);
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
