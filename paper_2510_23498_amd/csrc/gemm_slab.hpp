// C[M, N] = epilogue( A[M, K] * W[N, K]^T ) for wide layers (N a multiple of 256): the convolutions of the
// parabolic block of the paper's Sec. 6.3 (256 channels: implicit GEMM over (tap, channel), M = pixels) and
// their transposes, in the low-precision evaluation of the velocity and of its vector-Jacobian products.
//
// Same contract as gemm_nt (gemm.hpp) for the epilogues it covers: bias, tanh / ReLU, negation, rounding,
// overflow detector; no time term and no stored-activation factor.
//
// A workgroup owns a 256 x 256 block of C: four wavefronts with 128 x 128 each (256 accumulator registers).
// Per k-step of 32 the two operand slabs (256 rows x 64 bytes each) reach a ring of LDS slots by direct
// global->LDS loads -- no registers and no LDS store instructions, which at 64 B/clk per CU bound the
// 128 x 64-tile kernel on these shapes.  Both operands are K-contiguous, so a lane's 16 bytes of a row are a
// matrix-instruction fragment as they are; the four 16-byte pieces of a row are permuted (XOR with bits of the
// row number) so that the fragment reads are free of bank conflicts.  Convolution: the row of pixel m for tap
// (dy, dx) is the row of pixel m + dy W + dx, or a row of zeros (a small zero buffer in global memory) where
// that pixel is outside the image.  One barrier per k-step; explicit vmcnt waits (every wavefront issues
// the same number of loads per k-step).
#pragma once
#include "gemm.hpp"

namespace rampde {

constexpr int kNtSlabStages = 4;                     // ring of k-steps
constexpr int kNtSlabSlot = 2 * 256 * 64;            // bytes per k-step: A and W slabs
constexpr int kNtSlabLdsBytes = kNtSlabStages * kNtSlabSlot;  // 128 KB

__device__ __attribute__((aligned(64))) const uint16_t g_nt_slab_zeros[32] = {};

inline bool gemm_nt_slab_applies(const GemmNT& g, bool conv) {
  return g.N % 256 == 0 && g.K % 32 == 0 && g.M >= 4096 && !g.wt && !g.dact && !g.tr_c && (!conv || g.Cpad % 32 == 0);
}

template <class T, bool CONV>
__global__ __launch_bounds__(256, 1) void gemm_nt_slab(GemmNT g) {
  if (g.ctl && g.ctl->poison) return;
  constexpr int NS = kNtSlabStages;
  constexpr int PERW = 8;  // 1 KB wave-loads per wavefront and k-step: 4 of A, 4 of W
  typedef __attribute__((address_space(3))) uint8_t lds_u8;
  extern __shared__ __attribute__((aligned(16))) uint8_t nt_smem[];
  lds_u8* ring = (lds_u8*)nt_smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int frow = lane & 31, oct = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t m0 = (int64_t)blockIdx.x * 256;
  const int n0 = blockIdx.y * 256;
  const int KT = g.K / 32;

  // ---- loader role.  Wave-load i of this wavefront: rows 64 * wave + 16 * i + lane / 4 of the A slab (i < 4) or
  // of the W slab (i >= 4); lane % 4 is the 16-byte slot, which holds piece  slot ^ ((row >> 2) & 3).
  const int lrow = lane >> 2;
  const int lpiece = (lane & 3) ^ ((lrow >> 2) & 3);
  const uint16_t* wp[4];   // W rows of this lane
  const uint16_t* ap[4];   // A rows (pixels) of this lane, unshifted
  unsigned avalid[4];      // bit t: the pixel that tap t reads for this row is inside the image (dense: bit 0 = row < M)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 64 * wave + 16 * i + lrow;
    wp[i] = g.W + (size_t)(n0 + r) * g.ldw + lpiece * 8;
    const int64_t m = m0 + r;
    const bool live = m < g.M;
    ap[i] = g.A + (size_t)(live ? m : 0) * g.lda + lpiece * 8;
    avalid[i] = live ? 1u : 0u;
    if (CONV) {
      const int x = (int)(m % g.Wd), y = (int)((m / g.Wd) % g.H);
      unsigned v = 0;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
        v |= (live && yy >= 0 && yy < g.H && xx >= 0 && xx < g.Wd) ? (1u << t) : 0u;
      }
      avalid[i] = v;
    }
  }
  const uintptr_t zeros = (uintptr_t)g_nt_slab_zeros + (uintptr_t)lpiece * 16;
  int wslot = 0;
  // position of the next k-step to load: tap and channel offset (CONV), or just the k offset
  int ld_kt = 0, ld_tap = 0, ld_c0 = 0;
  auto issue = [&]() {
    lds_u8* slot = ring + wslot * kNtSlabSlot;
    wslot = (wslot + 1 == NS) ? 0 : wslot + 1;
    // (uniform) element offset of this k-step's rows from the unshifted ones
    int64_t delta = (int64_t)ld_kt * 32;
    if (CONV) {
      const int dy = ld_tap / 3 - 1, dx = ld_tap - (ld_tap / 3) * 3 - 1;
      delta = (int64_t)(dy * g.Wd + dx) * g.lda + ld_c0;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // (a select on the address bits: a row outside the image or past M reads the zero buffer)
      const uintptr_t in = ((avalid[i] >> (CONV ? ld_tap : 0)) & 1u) ? ~(uintptr_t)0 : (uintptr_t)0;
      const uintptr_t addr = ((uintptr_t)(ap[i] + delta) & in) | (zeros & ~in);
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint16_t*>(addr),
                                       (__attribute__((address_space(3))) void*)(slot + (64 * wave + 16 * i) * 64), 16, 0, 0);
    }
    // (CONV: the k-steps run through the 9 taps of one block of 32 channels before the next block, so that the rows
    // a tap reads are those its predecessor has just brought into the caches; W's K index is tap * Cpad + channel)
    const int64_t wk = CONV ? (int64_t)ld_tap * g.Cpad + ld_c0 : (int64_t)ld_kt * 32;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(wp[i] + wk,
                                       (__attribute__((address_space(3))) void*)(slot + 256 * 64 + (64 * wave + 16 * i) * 64), 16, 0, 0);
    // advance, staying on the last k-step once it is reached (the extra loads of the pipeline tail stay in bounds)
    const bool more = ld_kt + 1 < KT;
    ld_kt += more ? 1 : 0;
    if (CONV) {
      const int t1 = ld_tap + (more ? 1 : 0);
      const bool wrap = t1 == 9;
      ld_tap = wrap ? 0 : t1;
      ld_c0 += wrap ? 32 : 0;
    }
  };
  // ---- consumer role: fragment (row r of a 32-row block, k-octet o) of k16 sub-step kk is piece 2 kk + o
  int rd[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) rd[kk] = frow * 64 + (((2 * kk + oct) ^ ((frow >> 2) & 3)) * 16);
  int rslot = 0;
  auto read_frags = [&](u16x8 (&fa)[2][4], u16x8 (&fb)[2][4]) {
    const lds_u8* slot = ring + rslot * kNtSlabSlot;
    rslot = (rslot + 1 == NS) ? 0 : rslot + 1;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        fa[kk][a] = *reinterpret_cast<const __attribute__((address_space(3))) u16x8*>(slot + (wm * 128 + a * 32) * 64 + rd[kk]);
        fb[kk][a] = *reinterpret_cast<const __attribute__((address_space(3))) u16x8*>(slot + 256 * 64 + (wn * 128 + a * 32) * 64 + rd[kk]);
      }
  };
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.f;
  auto wait_vm = [&](auto cnt) {
    constexpr int c = decltype(cnt)::value;
    static_assert(c < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (c & 15) | ((c >> 4) << 14));  // vmcnt only
  };
  auto mma = [&](const u16x8 (&fa)[2][4], const u16x8 (&fb)[2][4]) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = Low<T>::mfma32(fa[kk][a], fb[kk][b], acc[a][b]);
  };

  // Pipeline: k-steps st + 1 .. st + NS - 2 are in LDS or on their way while k-step st is multiplied; the
  // fragments of k-step st + 1 are read in the shadow of the matrix instructions of st.
  u16x8 fa[2][2][4], fb[2][2][4];
#pragma unroll
  for (int u = 0; u < NS - 1; ++u) issue();
  wait_vm(std::integral_constant<int, (NS - 2) * PERW>{});
  __builtin_amdgcn_s_barrier();
  read_frags(fa[0], fb[0]);
  auto k_step = [&](u16x8 (&ca)[2][4], u16x8 (&cb)[2][4], u16x8 (&na)[2][4], u16x8 (&nb)[2][4]) {
    wait_vm(std::integral_constant<int, (NS - 3) * PERW>{});
    __builtin_amdgcn_s_barrier();  // everyone's part of k-step st + 1 is in LDS; everyone is done reading k-step st
    __builtin_amdgcn_sched_barrier(0);
    issue();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(na, nb);  // k-step st + 1 (past the end: a copy of the last one, never multiplied)
    __builtin_amdgcn_sched_barrier(0);  // (the reads are issued first: the matrix instructions cover their latency)
    mma(ca, cb);
    __builtin_amdgcn_sched_barrier(0);
  };
  int st = 0;
  for (; st + 2 <= KT; st += 2) {
    k_step(fa[0], fb[0], fa[1], fb[1]);
    k_step(fa[1], fb[1], fa[0], fb[0]);
  }
  if (st < KT) k_step(fa[0], fb[0], fa[1], fb[1]);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tail's extra loads

  // ---- epilogue: accumulator lane layout of a 32x32 block: column = lane % 32, row = 8 (q / 4) + 4 (lane / 32) + q % 4
  bool bad = false;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int n = n0 + wn * 128 + b * 32 + frow;
    const float bv = g.bias ? g.bias[n] : 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int64_t mb = m0 + wm * 128 + a * 32 + 4 * oct;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int64_t m = mb + 8 * (q >> 2) + (q & 3);
        if (m < g.M) {
          float v = acc[a][b][q] + bv;
          if (g.act_tanh == 1) v = act_tanh(v);
          else if (g.act_tanh == 2) v = fmaxf(v, 0.f);
          if (g.negate) v = -v;
          const uint16_t qv = Low<T>::from_f32(v);
          bad = bad || Low<T>::nonfinite(qv);
          g.C[(size_t)m * g.ldc + n] = qv;
        }
      }
    }
  }
  if (g.detect) raise_if_any(bad, g.ctl);
}

}  // namespace rampde
