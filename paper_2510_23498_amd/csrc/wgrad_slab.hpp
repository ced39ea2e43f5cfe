// Parameter gradients of one adjoint step for dense networks from the feature-group-major buffers of the
// row-tile adjoint kernels (paper Sec. 3, update of g;  dW_l = delta_l^T act_{l-1}, fp32 sums), for
// contractions long enough to be bound by the operand stream (every operand byte is read once per
// launch from memory that the adjoint kernel has just written).
//
// A wavefront owns a 128 x 128 block of dW_l (256 accumulator registers); a workgroup is four of them,
// arranged 2 x 2, 4 x 1 or 1 x 4 over the layer's (outputs x inputs), and owns one K-chunk of the batch
// contraction.  Per k-step of 16 the workgroup's operand slabs (128 features x 16 k = 4 KB each) are
// brought into a ring of LDS slots by direct global->LDS loads: no registers, no LDS store instructions,
// every 128-byte line of a feature group fetched by 8 consecutive lanes.  A lane's 64 bytes of a slab
// (8 k x 4 features of feature group g = lane % 32, k-octet o = lane / 32) are, after a byte
// permutation, the operand fragments of FOUR 32x32x16 matrix instructions: instruction m takes feature
// 4 g + m as its row g.  So a wavefront reads 2 x 4 KB from LDS per 16 matrix instructions, and the
// workgroup fetches (2 + 2) x 4 KB from L2 for 64 of them: half the bytes per flop of a 128 x 128
// workgroup tile.  One barrier per k-step; the reads and permutations of k-step i + 1 are issued in the
// shadow of the matrix instructions of k-step i.
// Results go to the K-chunk's private copy of the gradient vector as in wgrad_feature_major (no atomics,
// fixed summation order; the copies are summed once at the end of the backward pass).
#pragma once
#include "gemm.hpp"

namespace rampde {

constexpr int kSlabBytes = 4096;          // 128 features x 16 k, 16-bit
constexpr int64_t kSlabMinK = 8192;       // shorter contractions (stages x padded batch) keep the 128 x 128-workgroup kernel
constexpr int slab_stages(int nslab) { return nslab <= 4 ? 9 : 7; }  // ring of k-steps in LDS: 144 KB / 140 KB
typedef __attribute__((address_space(3))) uint8_t lds_u8;

// One workgroup tile: WA x WB wavefronts of 128 x 128 over one K-chunk.  SUMS: the tile also forms the sums
// over k of its cotangent slabs (bias and time-column gradients).  MULTI: the launch may cover several adjoint
// steps (the running sums are rescaled between them); otherwise the one step's factor is applied at the end.
template <class T, int WA, int WB, bool SUMS, bool MULTI>
__device__ __forceinline__ void wgs_body(const WgradArgs& g, const WgradLayer& y, int a0, int b0, int64_t k_begin, int64_t k_end,
                                         int split, int nsteps, lds_u8* ring) {
  constexpr int NSLAB = WA + WB;
  constexpr int NS = slab_stages(NSLAB);
  constexpr int kSlabSlot = NSLAB * kSlabBytes;
  constexpr int NINSTR = NSLAB * 4;           // 1 KB wave-loads per k-step
  constexpr int PERW = (NINSTR + 3) / 4;      // per wavefront
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  static_assert(WA * WB == 4 && NINSTR % 4 == 0, "four wavefronts, each with the same number of wave-loads per k-step");
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = lane & 31, oct = lane >> 5;
  const int wa = wave / WB, wb = wave % WB;
  const int nk = (int)((k_end - k_begin) >> 4);  // k-steps of 16 per adjoint step

  // ---- loader role: wave-load number q = wave + 4 i covers groups 8 (q % 4) .. + 7 of slab q / 4;
  // lane -> (group, 16-byte piece) with the pieces of a line permuted so that the fragment reads
  // below are free of bank conflicts
  // A wave-load's address = uniform base (tensor, buffer set, k-step) + a 32-bit per-lane byte offset that never
  // changes: the per-lane registers are written once, before the first load is in flight.
  const uint16_t* lbase[PERW];
  uint32_t lvoff[PERW];
  int lds_off[PERW];
#pragma unroll
  for (int i = 0; i < PERW; ++i) {
    const int q = wave + 4 * i;
    const int slab = q >> 2, part = q & 3;
    const int gamma = part * 8 + (lane >> 3);
    const int piece = (lane & 7) ^ ((gamma >> 1) & 7);
    const bool isA = slab < WA;
    const int f0 = isA ? a0 + slab * 128 : b0 + (slab - WA) * 128;
    const int pad = isA ? y.NaPad : y.NbPad;
    const int gidx = (f0 + gamma * 4 < pad) ? f0 / 4 + gamma : 0;  // beyond the padded extent: group 0, masked later
    lbase[i] = (isA ? y.DT : y.AT) + (size_t)k_begin * 4;
    lvoff[i] = (uint32_t)(((size_t)gidx * g.ldk + 2 * piece) * 8);   // (a tensor of a buffer set is < 4 GB: checked by the host)
    lds_off[i] = slab * kSlabBytes + part * 1024;
  }
  int wslot = 0;  // ring slot of the next k-step to load
  // position of the next k-step to load: (number ld_it of the step within the launch, k-step ld_kk, buffer set)
  int ld_it = 0, ld_kk = 0, ld_set = g.step % g.nsets;
  auto issue = [&]() {
    lds_u8* slot = ring + wslot * kSlabSlot;
    wslot = (wslot + 1 == NS) ? 0 : wslot + 1;
    const size_t off = (size_t)ld_set * (size_t)g.set_stride + (size_t)ld_kk * 64;
#pragma unroll
    for (int i = 0; i < PERW; ++i)
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint8_t*>(lbase[i] + off) + lvoff[i],
                                       (__attribute__((address_space(3))) void*)(slot + lds_off[i]), 16, 0, 0);
    // advance, staying on the last k-step once it is reached (the extra loads of the pipeline tail stay in bounds)
    const bool last = (ld_it == nsteps - 1) && (ld_kk == nk - 1);
    const bool wrap = (ld_kk == nk - 1);
    ld_kk = last ? ld_kk : (wrap ? 0 : ld_kk + 1);
    ld_it = (last || !wrap) ? ld_it : ld_it + 1;
    ld_set = (last || !wrap) ? ld_set : (ld_set == 0 ? g.nsets - 1 : ld_set - 1);
  };
  // ---- consumer role
  const int swz = (grp >> 1) & 7;
  int rd[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) rd[i] = (grp * 8 + ((4 * oct + i) ^ swz)) * 16;
  int rslot = 0;  // ring slot of the next k-step to consume
  auto read_raw = [&](u32x4 (&qa)[4], u32x4 (&qb)[4]) {
    const lds_u8* slot = ring + rslot * kSlabSlot;
    rslot = (rslot + 1 == NS) ? 0 : rslot + 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qa[i] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(slot + wa * kSlabBytes + rd[i]);
      qb[i] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(slot + (WA + wb) * kSlabBytes + rd[i]);
    }
  };
  auto regroup = [&](const u32x4 (&w)[4], u16x8 (&f)[4]) {
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int d = m >> 1;
      const uint32_t sel = (m & 1) ? 0x07060302u : 0x05040100u;
      u32x4 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = __builtin_amdgcn_perm(w[i][d + 2], w[i][d], sel);
      f[m] = __builtin_bit_cast(u16x8, o);
    }
  };
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.f;
  // sums over k of the cotangent fragments (bias and time-column gradients), fp32
  float sum_b[4] = {0.f, 0.f, 0.f, 0.f}, sum_t[4] = {0.f, 0.f, 0.f, 0.f};
  // stage of a k-step: stage boundaries in units of k-steps from the chunk's start (the padded batch and a
  // chunk's start are multiples of 64 k)
  const int j_first = __builtin_amdgcn_readfirstlane((int)(k_begin / g.Rp));
  const int rp16 = __builtin_amdgcn_readfirstlane((int)(g.Rp >> 4));
  const int stage_kk0 = __builtin_amdgcn_readfirstlane((int)(((int64_t)(j_first + 1) * g.Rp - k_begin) >> 4));
  int jst = j_first, stage_kk = stage_kk0;
  int it = 0, kk = 0;  // position of the k-step being multiplied
  // (the step table and the scale history are not written while this kernel runs: read through the constant
  // address space, uniform addresses become scalar loads, which no direct load in flight delays)
  typedef const __attribute__((address_space(4))) float cfloat;
  cfloat* const steptab = (cfloat*)g.steptab;
  cfloat* const hist = (cfloat*)g.scale_hist;
  cfloat* tau_row = steptab + 1;  // stage times of the adjoint step `it`

  auto wait_vm = [&](auto cnt) {
    constexpr int c = decltype(cnt)::value;
    static_assert(c < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (c & 15) | ((c >> 4) << 14));  // vmcnt only
  };
  auto sums = [&](const u16x8 (&fa)[4]) {
    if constexpr (SUMS) {
      // (uniform, branch-free: the stage of this k-step and its time)
      const bool adv = kk >= stage_kk;   // (32-bit scalar arithmetic throughout: the time's address stays uniform)
      jst += adv ? 1 : 0;
      stage_kk += adv ? rp16 : 0;
      const float tau = tau_row[jst];
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) part += Low<T>::to_f32(fa[m][e]);
        sum_b[m] += part;
        sum_t[m] = fmaf(tau, part, sum_t[m]);
      }
    }
  };
  auto mma = [&](auto half, const u16x8 (&fa)[4], const u16x8 (&fb)[4]) {
    constexpr int a0h = decltype(half)::value * 2;
#pragma unroll
    for (int a = a0h; a < a0h + 2; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        acc[a][b] = Low<T>::mfma32(fa[a], fb[b], acc[a][b]);
      }
  };
  // Pipeline: k-steps st + 1 .. st + NS - 2 are in LDS or on their way while k-step st is multiplied; the
  // fragments of k-step st + 1 are read and permuted in the shadow of the matrix instructions of st.
  u16x8 fa[2][4], fb[2][4];
#pragma unroll
  for (int u = 0; u < NS - 1; ++u) issue();
  wait_vm(std::integral_constant<int, (NS - 2) * PERW>{});
  __builtin_amdgcn_s_barrier();
  {
    u32x4 qa[4], qb[4];
    read_raw(qa, qb);
    regroup(qa, fa[0]);
    regroup(qb, fb[0]);
  }
  auto k_step = [&](u16x8 (&ca)[4], u16x8 (&cb)[4], u16x8 (&na)[4], u16x8 (&nb)[4]) {
    // own loads of k-step st + 1 have landed when at most those of the NS - 3 later k-steps are outstanding
    wait_vm(std::integral_constant<int, (NS - 3) * PERW>{});
    __builtin_amdgcn_s_barrier();  // everyone's part of k-step st + 1 is in LDS; everyone is done reading k-step st
    __builtin_amdgcn_sched_barrier(0);
    issue();
    __builtin_amdgcn_sched_barrier(0);
    u32x4 qa[4], qb[4];
    read_raw(qa, qb);   // k-step st + 1 (past the end: a clamped copy of the last one, never multiplied)
    __builtin_amdgcn_sched_barrier(0);
    mma(std::integral_constant<int, 0>{}, ca, cb);   // (covers the latency of the LDS reads)
    sums(ca);
    if constexpr (SUMS) {
      // one matrix instruction, then a ninth of the sums' vector instructions, eight times over
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    regroup(qa, na);
    regroup(qb, nb);
    mma(std::integral_constant<int, 1>{}, ca, cb);
    // one matrix instruction, then four permutations, eight times over
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    ++kk;
  };
  // (a chunk's k extent is a multiple of 64: the k-steps of an adjoint step pair up, and every adjoint step
  // starts on fragment set 0)
  float fin = 1.f;  // factor still to be applied to the sums at the end
  for (it = 0; it < (MULTI ? nsteps : 1); ++it) {
    kk = 0;
    jst = j_first;
    stage_kk = stage_kk0;
    // the step's row of the step table (h_i, tau_i1 .. tau_is) and its factor c_i = h_i / S_i, by scalar loads
    const int step = g.step - it;
    cfloat* row = steptab + (size_t)step * (1 + g.s);
    tau_row = row + 1;
    const float c = row[0] / hist[step];
    const float cn = (it + 1 < nsteps) ? steptab[(size_t)(step - 1) * (1 + g.s)] / hist[step - 1] : 1.f;
    for (int st = 0; st < nk; st += 2) {
      k_step(fa[0], fb[0], fa[1], fb[1]);
      k_step(fa[1], fb[1], fa[0], fb[0]);
    }
    // the adjoint step's partial sums are complete: s_scale[it] = c_it / c_{it+1} with c_i = h_i / S_i (the
    // last: c_it itself), so that the running sums end as  sum_i c_i * (partial sum of step i)
    const float sc = c / cn;
    fin = c;
    if constexpr (MULTI) {
      fin = 1.f;
      if (sc != 1.f) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[a][b][q] *= sc;
        if constexpr (SUMS) {
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            sum_b[m] *= sc;
            sum_t[m] *= sc;
          }
        }
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tail's extra loads

  // ---- every wavefront owns its 128 x 128 block of the chunk's private gradient copy
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const int ta0 = a0 + wa * 128, tb0 = b0 + wb * 128;
  // Two rounds, each with all its loads first and then the updates: two memory round trips, not one per
  // row.  Rows of a weight block with a time column have an odd pitch: the 16-byte accesses are then only
  // 4-byte aligned, which global memory accesses allow.
  typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
  float* const Gc = y.G + (size_t)split * g.P;
  int nb = tb0 + 4 * grp;
  // (opaque to the compiler: otherwise the 64 row addresses below are formed before the contraction and held
  // in registers throughout it)
  asm volatile("" : "+v"(nb));
  if (y.Nb % 4 == 0) {  // (uniform) a lane's 4 columns are all inside or all outside
#pragma unroll
    for (int ah = 0; ah < 2; ++ah) {
      f32x4 o[2][16];
#pragma unroll
      for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int na = ta0 + 4 * (8 * (q >> 2) + 4 * oct + (q & 3)) + ah * 2 + a2;
          const bool in = na < y.Na && nb < y.Nb;
          o[a2][q] = in ? *reinterpret_cast<const f32x4u*>(Gc + (size_t)na * y.ldg + nb) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
      for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int na = ta0 + 4 * (8 * (q >> 2) + 4 * oct + (q & 3)) + ah * 2 + a2;
          if (na < y.Na && nb < y.Nb) {
            f32x4 v = o[a2][q];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = fmaf(fin, acc[ah * 2 + a2][e][q], v[e]);
            *reinterpret_cast<f32x4u*>(Gc + (size_t)na * y.ldg + nb) = v;
          }
        }
    }
  } else {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float o[8][4];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int qq = h * 8 + q;
          const int na = ta0 + 4 * (8 * (qq >> 2) + 4 * oct + (qq & 3)) + a;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[q][e] = (na < y.Na && nb + e < y.Nb) ? Gc[(size_t)na * y.ldg + nb + e] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int qq = h * 8 + q;
          const int na = ta0 + 4 * (8 * (qq >> 2) + 4 * oct + (qq & 3)) + a;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (na < y.Na && nb + e < y.Nb) Gc[(size_t)na * y.ldg + nb + e] = fmaf(fin, acc[a][e][qq], o[q][e]);
        }
      }
    }
  }
  if constexpr (SUMS) {
    if (wb == 0) {
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        sum_b[m] += __shfl_xor(sum_b[m], 32);
        sum_t[m] += __shfl_xor(sum_t[m], 32);
      }
      if (oct == 0) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int na = ta0 + grp * 4 + m;
          if (na < y.Na) {
            float* db = y.gb + (size_t)split * g.P + na;
            *db = fmaf(fin, sum_b[m], *db);
            if (y.gwt) {
              float* dt = y.gwt + (size_t)split * g.P + (size_t)na * y.ldg;
              *dt = fmaf(fin, sum_t[m], *dt);
            }
          }
        }
      }
    }
  }
}

// Arrangement of the four wavefronts per layer.  WgradLayer::tiles_a / tiles_b count workgroup tiles of
// that arrangement.
enum SlabShape { SLAB_2x2 = 0, SLAB_4x1 = 1, SLAB_1x4 = 2 };
inline SlabShape slab_shape(int NaPad, int NbPad) {
  if (NbPad <= 128) return SLAB_4x1;
  if (NaPad <= 128) return SLAB_1x4;
  return SLAB_2x2;  // (extents between 128 and 256 are covered by masking)
}
inline int slab_tile_a(SlabShape s) { return s == SLAB_2x2 ? 256 : (s == SLAB_4x1 ? 512 : 128); }
inline int slab_tile_b(SlabShape s) { return s == SLAB_2x2 ? 256 : (s == SLAB_4x1 ? 128 : 512); }
constexpr int kSlabLdsBytes = 9 * 4 * kSlabBytes;  // the larger of the two rings (2 x 2: 9 slots of 4 slabs)
struct SlabArgs {
  WgradArgs w;
  int shape[8];
};

// One launch covers steps g.step, g.step - 1, ..., g.step - nsteps + 1 (nsteps = 0 or 1: the one step), of which the
// accepted ones at the head of the range are taken; the buffers of step i are set i % nsets; row i of steptab =
// (h_i, tau_i1 .. tau_is).
template <class T, bool MULTI>
__global__ __launch_bounds__(256, 1) void wgrad_slab(SlabArgs sa) {
  const WgradArgs& g = sa.w;
  const int per_xcd = (int)gridDim.x >> 3;
  const int gp = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (gp >= g.ntiles * g.ksplits) return;
  const int split = gp / g.ntiles;
  const int t = gp - split * g.ntiles;
  int li = 0;
#pragma unroll
  for (int q = 1; q < 8; ++q)
    if (q < g.L && t >= g.layer[q].tile0) li = q;
  const WgradLayer y = g.layer[li];
  const int shape = sa.shape[li];
  const int r = t - y.tile0;
  const int ta = r % y.tiles_a, tb = r / y.tiles_a;
  const int64_t k_begin = (int64_t)split * g.kchunk;
  int64_t k_end = k_begin + g.kchunk;
  if (k_end > g.ldk) k_end = g.ldk;
  if (k_begin >= k_end) return;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  lds_u8* ring = (lds_u8*)smem;
  // Steps whose cotangent chain was rejected (or that never ran because an earlier one was) have no recorded
  // scale: the launch covers the accepted steps at the head of its range only.
  const int want = MULTI ? g.nsteps : 1;
  int nsteps = 0;
  while (nsteps < want && g.scale_hist[g.step - nsteps] != 0.f) ++nsteps;  // (uniform: scalar loads)
  if (nsteps == 0) return;
  const bool sums = (tb == 0);
  if (shape == SLAB_2x2) {
    if (sums) wgs_body<T, 2, 2, true, MULTI>(g, y, ta * 256, tb * 256, k_begin, k_end, split, nsteps, ring);
    else wgs_body<T, 2, 2, false, MULTI>(g, y, ta * 256, tb * 256, k_begin, k_end, split, nsteps, ring);
  } else if (shape == SLAB_4x1) {
    if (sums) wgs_body<T, 4, 1, true, MULTI>(g, y, ta * 512, tb * 128, k_begin, k_end, split, nsteps, ring);
    else wgs_body<T, 4, 1, false, MULTI>(g, y, ta * 512, tb * 128, k_begin, k_end, split, nsteps, ring);
  } else {
    if (sums) wgs_body<T, 1, 4, true, MULTI>(g, y, ta * 128, tb * 512, k_begin, k_end, split, nsteps, ring);
    else wgs_body<T, 1, 4, false, MULTI>(g, y, ta * 128, tb * 512, k_begin, k_end, split, nsteps, ring);
  }
}

}  // namespace rampde
