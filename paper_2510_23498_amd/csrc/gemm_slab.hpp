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
  // (the choice of activation and sign is made once, around straight-line code: with one wavefront per SIMD nothing
  // hides a branch per element)
  auto convert = [&](auto act_c, auto neg_c) {
    constexpr int ACT = decltype(act_c)::value;
    constexpr bool NEG = decltype(neg_c)::value != 0;
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
          float v = acc[a][b][q] + bv;
          if (ACT == 1) v = act_tanh(v);
          else if (ACT == 2) v = fmaxf(v, 0.f);
          if (NEG) v = -v;
          const uint16_t qv = Low<T>::from_f32(v);
          if (m < g.M) {
            bad |= Low<T>::nonfinite(qv);
            g.C[(size_t)m * g.ldc + n] = qv;
          }
        }
      }
    }
  };
  typedef std::integral_constant<int, 0> c0;
  typedef std::integral_constant<int, 1> c1;
  typedef std::integral_constant<int, 2> c2;
  if (g.negate) {
    if (g.act_tanh == 1) convert(c1{}, c1{});
    else if (g.act_tanh == 2) convert(c2{}, c1{});
    else convert(c0{}, c1{});
  } else {
    if (g.act_tanh == 1) convert(c1{}, c0{});
    else if (g.act_tanh == 2) convert(c2{}, c0{});
    else convert(c0{}, c0{});
  }
  if (g.detect) raise_if_any(bad, g.ctl);
}


// ---- The same convolution with the input staged by image lines (W in {16, 32, 64} pixels per line, 512 / W lines per
// tile, image heights that are multiples of that).  gemm_nt_slab fetches a 256 x 64-byte slab of shifted input rows for
// every tap: nine passes over the same pixels.  Here a block of 32 input channels of the tile's lines and of the line
// above and below (zeros where that line is off the image), with a zero pixel before and after every line, is brought
// into LDS ONCE and serves all nine taps as row offsets; only the weight slabs (128 output channels x 32 input
// channels of one tap) stream per k-step, through a ring of four slots.  The input blocks alternate between two
// buffers: block c + 1 is requested when block c's first tap is multiplied.  A workgroup owns 512 pixels x 128 output
// channels (a wavefront: 128 x 128): all compute units of an XCD pull the same weight slabs from its L2 at the same
// time, and half as many weight bytes per pixel is what this shape is for.  Fill traffic per k-step and workgroup:
// 12.7 KB (gemm_nt_slab: 32 KB).  Fragment reads, permutation of the 16-byte pieces (XOR with bits of the LDS row
// number), accumulators and epilogue as in gemm_nt_slab.
template <int W16>
struct NtLines {
  static constexpr int W = 16 * W16, LT = 512 / W;
  static constexpr int ROWS = (LT + 2) * (W + 2);     // LDS rows (pixels) of an input block
  static constexpr int XB = ROWS * 64;                // bytes of an input block (32 channels)
  static constexpr int NJ = (LT + 2) * W16;           // its 1 KB wave-loads (16 pixels each)
  static constexpr int XL = (NJ + 3) / 4;             // ... per wavefront (the last ones may be repeated)
  static constexpr int NS = 4, WB = 128 * 64;         // ring of weight slabs
  static constexpr int EP = 272;                      // epilogue: pitch (bytes) of a staged output row of 128 channels
  static constexpr int LDS = (2 * XB + NS * WB > 4 * 128 * EP) ? 2 * XB + NS * WB : 4 * 128 * EP;
};

inline bool conv_nt_lines_applies(const GemmNT& g) {
  if (!(g.Wd == 16 || g.Wd == 32 || g.Wd == 64)) return false;
  return g.N % 128 == 0 && g.M >= 4096 && !g.wt && !g.dact && !g.tr_c && g.Cpad % 32 == 0 && g.K == 9 * g.Cpad &&
         g.H % (512 / g.Wd) == 0 && g.M % 512 == 0;
}

template <class T, int W16>
__global__ __launch_bounds__(256, 1) void conv_nt_lines(GemmNT g) {
  if (g.ctl && g.ctl->poison) return;
  typedef NtLines<W16> P;
  constexpr int W = P::W, LT = P::LT, NS = P::NS, PERW = 2;
  typedef __attribute__((address_space(3))) uint8_t lds_u8;
  extern __shared__ __attribute__((aligned(16))) uint8_t ntl_smem[];
  lds_u8* xbuf = (lds_u8*)ntl_smem;            // two input blocks
  lds_u8* ring = xbuf + 2 * P::XB;             // NS weight slabs
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int frow = lane & 31, oct = lane >> 5;
  const int64_t m0 = (int64_t)blockIdx.x * 512;
  const int n0 = blockIdx.y * 128;
  const int KC = g.Cpad / 32, KT = 9 * KC;

  // the zero pixels before and after every line of both input blocks (never overwritten)
  for (int i = tid; i < 2 * (LT + 2) * 2 * 4; i += 256) {
    const int piece = i & 3, side = (i >> 2) & 1, line = (i >> 3) % (LT + 2), buf = (i >> 3) / (LT + 2);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    *reinterpret_cast<__attribute__((address_space(3))) u32x4*>(xbuf + buf * P::XB + (line * (W + 2) + (side ? W + 1 : 0)) * 64 + piece * 16) =
        u32x4{0u, 0u, 0u, 0u};
  }
  __syncthreads();

  // ---- loader role.  Weight slab: wave-load i of this wavefront = rows 32 * wave + 16 * i + lane / 4; lane % 4 is the
  // 16-byte slot, which holds piece  slot ^ ((row >> 2) & 3).
  const int lrow = lane >> 2;
  const uint16_t* wp[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = 32 * wave + 16 * i + lrow;
    wp[i] = g.W + (size_t)(n0 + r) * g.ldw + (((lane & 3) ^ ((lrow >> 2) & 3))) * 8;
  }
  // Input block: wave-load j = (LDS line j / W16, pixels 16 (j % W16) ..); LDS line i holds the tile's line i - 1.
  const int64_t line0 = m0 / W;                       // the tile's first line (lines over all samples)
  const int y0 = (int)(line0 % g.H);                  // ... within its image (the tile's lines are in one image)
  const uintptr_t zeros = (uintptr_t)g_nt_slab_zeros;
  uintptr_t xsrc[P::XL];   // this lane's 16 bytes of channel block 0, or the zero buffer
  int xdst[P::XL];         // LDS offset of the wave-load within an input block
  bool xlive[P::XL];
#pragma unroll
  for (int i = 0; i < P::XL; ++i) {
    const int j = (wave * P::XL + i < P::NJ) ? wave * P::XL + i : P::NJ - 1;
    const int li = j / W16, x = 16 * (j % W16) + lrow;
    const int pr = li * (W + 2) + 1 + x;
    const int piece = (lane & 3) ^ ((pr >> 2) & 3);
    const int yy = y0 - 1 + li;
    xlive[i] = yy >= 0 && yy < g.H;
    xsrc[i] = xlive[i] ? (uintptr_t)(g.A + ((size_t)(line0 - 1 + li) * W + x) * g.lda + piece * 8) : zeros + (lane & 3) * 16;
    xdst[i] = (li * (W + 2) + 1 + 16 * (j % W16)) * 64;
  }
  auto issue_x = [&](int c) {
    lds_u8* dst = xbuf + (c & 1) * P::XB;
#pragma unroll
    for (int i = 0; i < P::XL; ++i)
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint16_t*>(xsrc[i] + (xlive[i] ? (uintptr_t)c * 64 : 0)),
                                       (__attribute__((address_space(3))) void*)(dst + xdst[i]), 16, 0, 0);
  };
  int wslot = 0, ld_kt = 0, ld_tap = 0, ld_c0 = 0;
  auto issue_w = [&]() {
    lds_u8* slot = ring + wslot * P::WB;
    wslot = (wslot + 1 == NS) ? 0 : wslot + 1;
    const int64_t wk = (int64_t)ld_tap * g.Cpad + ld_c0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
      __builtin_amdgcn_global_load_lds(wp[i] + wk, (__attribute__((address_space(3))) void*)(slot + (32 * wave + 16 * i) * 64), 16, 0, 0);
    // advance, staying on the last k-step once it is reached (the extra loads of the pipeline tail stay in bounds)
    const bool more = ld_kt + 1 < KT;
    ld_kt += more ? 1 : 0;
    const int t1 = ld_tap + (more ? 1 : 0);
    const bool wrap = t1 == 9;
    ld_tap = wrap ? 0 : t1;
    ld_c0 += wrap ? 32 : 0;
  };

  // ---- consumer role.  Input fragment of 32-pixel block a: pixel p = 128 wave + 32 a + lane % 32 of the tile, LDS row
  // (p / W + 1 + dy) (W + 2) + p % W + 1 + dx; weight fragment: row 32 a + lane % 32 of the slab.
  int pr0[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int p = 128 * wave + 32 * a + frow;
    pr0[a] = (p / W + 1) * (W + 2) + p % W + 1;
  }
  int rdw[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) rdw[kk] = frow * 64 + (((2 * kk + oct) ^ ((frow >> 2) & 3)) * 16);
  int rslot = 0, rd_tap = 0, rd_c = 0;   // position of the next k-step to read
  auto read_frags = [&](u16x8 (&fa)[2][4], u16x8 (&fb)[2][4]) {
    const lds_u8* slot = ring + rslot * P::WB;
    rslot = (rslot + 1 == NS) ? 0 : rslot + 1;
    const lds_u8* xb = xbuf + (rd_c & 1) * P::XB;
    const int shift = (rd_tap / 3 - 1) * (W + 2) + (rd_tap % 3 - 1);
    // (in the order in which the matrix instructions use them)
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int pr = pr0[a] + shift, key = (pr >> 2) & 3;
        fa[kk][a] = *reinterpret_cast<const __attribute__((address_space(3))) u16x8*>(xb + pr * 64 + (((2 * kk + oct) ^ key) * 16));
        fb[kk][a] = *reinterpret_cast<const __attribute__((address_space(3))) u16x8*>(slot + a * 32 * 64 + rdw[kk]);
      }
    // (past the end: stays on the last k-step, whose copy is never multiplied)
    const bool more = rd_c * 9 + rd_tap + 1 < KT;
    const int t1 = rd_tap + (more ? 1 : 0);
    rd_c += (t1 == 9) ? 1 : 0;
    rd_tap = (t1 == 9) ? 0 : t1;
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
  // matrix instructions [I0, I1) of a k-step's 32, in the order (kk, a, b)
  auto mma = [&](auto first, auto last, const u16x8 (&fa)[2][4], const u16x8 (&fb)[2][4]) {
    constexpr int I0 = decltype(first)::value, I1 = decltype(last)::value;
#pragma unroll
    for (int i = I0; i < I1; ++i) {
      const int kk = i >> 4, a = (i >> 2) & 3, b = i & 3;
      acc[a][b] = Low<T>::mfma32(fa[kk][a], fb[kk][b], acc[a][b]);
    }
  };

  // Pipeline: weight slabs st + 1 .. st + NS - 2 are in LDS or on their way while k-step st is multiplied; the fragments
  // of k-step st + 1 are read in the shadow of the matrix instructions of st.  Loads complete in the order of their issue,
  // so a wait that leaves only the weight loads of the later k-steps outstanding also covers an input block requested
  // before them (and waits a little longer than needed where one was requested after them).
  u16x8 fa[2][2][4], fb[2][2][4];
  issue_x(0);
#pragma unroll
  for (int u = 0; u < NS - 1; ++u) issue_w();
  wait_vm(std::integral_constant<int, (NS - 2) * PERW>{});
  __builtin_amdgcn_s_barrier();
  read_frags(fa[0], fb[0]);
  int st_tap = 0, st_c = 0;  // position of the k-step being multiplied
  auto k_step = [&](u16x8 (&ca)[2][4], u16x8 (&cb)[2][4], u16x8 (&na)[2][4], u16x8 (&nb)[2][4]) {
    // One wavefront per SIMD: whatever it issues between two matrix instructions runs beside them, whatever it issues in
    // a block of its own leaves the matrix unit idle.  The first quarter of the k-step's matrix instructions goes out
    // before the wait (the unit works on them while this wavefront waits for the slab and the others); the address
    // arithmetic, the requests and the fragment reads of the next k-step are placed between the rest.
    mma(std::integral_constant<int, 0>{}, std::integral_constant<int, 8>{}, ca, cb);
    __builtin_amdgcn_sched_barrier(0);
    wait_vm(std::integral_constant<int, (NS - 3) * PERW>{});
    __builtin_amdgcn_s_barrier();  // everyone's part of k-step st + 1 is in LDS; everyone is done reading k-step st
    __builtin_amdgcn_sched_barrier(0);
    // (the other input buffer was last read for the last tap of block c - 1, one k-step ago)
    if (st_tap == 0 && st_c + 1 < KC) issue_x(st_c + 1);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(na, nb);
    issue_w();
    mma(std::integral_constant<int, 8>{}, std::integral_constant<int, 32>{}, ca, cb);
#pragma unroll
    for (int i = 0; i < 24; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one matrix instruction
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one fragment read
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // at most one request
      __builtin_amdgcn_sched_group_barrier(0x006, 5, 0);   // vector / scalar arithmetic
    }
    __builtin_amdgcn_sched_barrier(0);
    st_c += (st_tap == 8) ? 1 : 0;
    st_tap = (st_tap == 8) ? 0 : st_tap + 1;
  };
  int st = 0;
  for (; st + 2 <= KT; st += 2) {
    k_step(fa[0], fb[0], fa[1], fb[1]);
    k_step(fa[1], fb[1], fa[0], fb[0]);
  }
  if (st < KT) k_step(fa[0], fb[0], fa[1], fb[1]);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tail's extra loads

  // ---- epilogue: accumulator lane layout of a 32x32 block: column = lane % 32, row = 8 (q / 4) + 4 (lane / 32) + q % 4.
  // Storing from that layout is 256 two-byte store instructions per wavefront (a quarter of the kernel's time when it
  // was done so): the rounded block goes through LDS instead -- every wavefront has a region of its own, rows of
  // 128 channels with a pitch of 272 bytes -- and leaves as 16-byte stores of whole 256-byte row segments.
  __builtin_amdgcn_s_barrier();  // everyone is done reading the operand buffers
  lds_u8* stage = (lds_u8*)ntl_smem + wave * (128 * P::EP);
  bool bad = false;
  // (the choice of activation and sign is made once, around straight-line code: taken per element it was a branch per
  // element, and with one wavefront per SIMD nothing hides a branch)
  auto convert = [&](auto act_c, auto neg_c) {
    constexpr int ACT = decltype(act_c)::value;
    constexpr bool NEG = decltype(neg_c)::value != 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int n = n0 + b * 32 + frow;
      const float bv = g.bias ? g.bias[n] : 0.f;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int ml = a * 32 + 4 * oct + 8 * (q >> 2) + (q & 3);
          float v = acc[a][b][q] + bv;
          if (ACT == 1) v = act_tanh(v);
          else if (ACT == 2) v = fmaxf(v, 0.f);
          if (NEG) v = -v;
          const uint16_t qv = Low<T>::from_f32(v);
          bad |= Low<T>::nonfinite(qv);
          *reinterpret_cast<__attribute__((address_space(3))) uint16_t*>(stage + ml * P::EP + (b * 32 + frow) * 2) = qv;
        }
      }
    }
  };
  typedef std::integral_constant<int, 0> c0;
  typedef std::integral_constant<int, 1> c1;
  typedef std::integral_constant<int, 2> c2;
  if (g.negate) {
    if (g.act_tanh == 1) convert(c1{}, c1{});
    else if (g.act_tanh == 2) convert(c2{}, c1{});
    else convert(c0{}, c1{});
  } else {
    if (g.act_tanh == 1) convert(c1{}, c0{});
    else if (g.act_tanh == 2) convert(c2{}, c0{});
    else convert(c0{}, c0{});
  }
  {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int er = lane >> 4, ep = lane & 15;
    uint16_t* crow = g.C + (size_t)(m0 + wave * 128 + er) * g.ldc + n0 + ep * 8;
#pragma unroll 8
    for (int i = 0; i < 32; ++i) {
      const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(stage + (4 * i + er) * P::EP + ep * 16);
      *reinterpret_cast<u32x4*>(crow + (size_t)4 * i * g.ldc) = v;
    }
  }
  if (g.detect) raise_if_any(bad, g.ctl);
}

}  // namespace rampde
