// Weight gradient of a 3x3 convolution with many channels (multiples of 128: the parabolic block of the paper's
// Sec. 6.3), one term of the update of g in Sec. 3:
//   dW[co][ci][tap] += scale * sum_k delta[k][co] * x[k + dy W + dx][ci] * [pixel (y+dy, x+dx) inside]
// over the rows k (pixels of all samples and stages, channels-last) of one K-chunk.
//
// Both operands are stored with the contraction index (the pixel) as the SLOW one, while a matrix instruction wants
// 8 consecutive k per lane.  Here the rows go to LDS exactly as they are in memory (direct global->LDS loads: no
// registers, no LDS store instructions) and the transposing LDS read of gfx950 (64 bits, 16-bit elements) builds
// the fragments: within 16 lanes, lane s supplies the address of 4 consecutive channels of row s / 4 (channel
// group s % 4), and lane j receives the 4 rows of channel j -- 4 consecutive k of one channel (checked on the
// device with an index pattern).  Two such reads are the 8 k of a 32x32x16 fragment.
//
// Work split: a workgroup owns 128 output channels x 128 input channels x the three taps of one dy; its four
// wavefronts take 32 input channels each (192 accumulator registers: 4 co blocks x 3 dx).  Per k-step of 16 pixels
// a wavefront reads 4 cotangent fragments and 3 input fragments (the dx shifts are row offsets of the same line;
// a zero row before and after the line stands for the pixels off the line) for 12 matrix instructions.  A step of
// the pipeline is one image line: cotangent line l and input line l + dy (skipped when that line is off the image)
// in a ring of 16 / (W / 16) slots; explicit vmcnt waits (every wavefront issues the same number of loads per
// line), one barrier per line.  The 16-byte pieces of a row are permuted (XOR of the 32-channel block number
// with the row number mod 4) so that the four rows a transposing read touches fall into different banks.
//
// Needs W in {16, 32, 64}, channel counts that are multiples of 128, no time channel.  Bias gradient: sums of the
// cotangent over k by one extra matrix instruction against a fragment of ones (wavefront w: channel block w), the
// k-steps dealt out among the dy = 0 workgroups.  Every (K-chunk, workgroup tile) accumulates into a private fp32 copy
// over the backward pass (plain read-modify-write), summed at the end: the result does not depend on the order in
// which workgroups finish.
#pragma once
#include "gemm.hpp"

namespace rampde {

struct ConvWgradTr {
  const uint16_t* A; int lda;   // [rows, >= 128 tiles_a] cotangents of the layer's output
  const uint16_t* B; int ldb;   // [rows, >= 128 tiles_b] the layer's input
  int64_t lines;                // image lines over all stages and samples: rows / W
  int lines_per_split;
  float* part;                  // [splits][tiles_a][3 tiles_b][CT_SLOT] fp32
  int tiles_a, tiles_b;         // 128-channel blocks of the output / input channels
  int splits;                   // K-chunks
  float h;                      // scale = h / ctl->S_step
  const Ctl* ctl;
  int H;
  bool want_sums;               // also db[co] += scale * sum_k delta[k][co]
};

// floats of a workgroup's private copy: 12 (co block, dx) accumulator blocks of 4096 in register order, then the
// 128 cotangent sums
constexpr int CT_SLOT = 12 * 4096 + 128;
constexpr size_t conv_wgrad_tr_lds_bytes(int W) { return (size_t)(16 / (W / 16)) * (2 * W + 2) * 256; }

template <class T, int W16>
__global__ __launch_bounds__(256, 1) void conv_wgrad_tr(ConvWgradTr g) {
  if (g.ctl->poison) return;
  constexpr int W = 16 * W16, NS = 16 / W16, PERL = 2 * W16;
  constexpr int GB = W * 256, SLOT = (2 * W + 2) * 256;  // cotangent line, then the input line with its two zero rows
  typedef __attribute__((address_space(3))) uint8_t lds_u8;
  typedef short v4s __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) v4s lds_v4s;
  extern __shared__ __attribute__((aligned(16))) uint8_t cwt_smem[];
  lds_u8* ring = (lds_u8*)cwt_smem;
  const uint32_t ring_base = (uint32_t)(uintptr_t)ring;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // One-dimensional grid.  The 3 tiles_b workgroups that share an output-channel block and a K-chunk (a group: they read
  // the same cotangent lines, and input lines one apart) run on one XCD -- workgroup L is dispatched to XCD L % 8 --
  // so that its L2 fetches those lines from memory once: group number = 8 * (L / 8 / group size) + L % 8.
  const int gsize = 3 * g.tiles_b;
  const int wg_n = (int)(blockIdx.x >> 3);
  const int grp = 8 * (wg_n / gsize) + (int)(blockIdx.x & 7), tile = wg_n % gsize;
  if (grp >= g.tiles_a * g.splits) return;
  const int at = grp % g.tiles_a, chunk = grp / g.tiles_a;
  const int a0 = at * 128;
  const int bt = tile / 3, dy = tile % 3 - 1, b0 = bt * 128;
  const int64_t l_begin = (int64_t)chunk * g.lines_per_split;
  int64_t l_end = l_begin + g.lines_per_split;
  if (l_end > g.lines) l_end = g.lines;
  if (l_begin >= l_end) return;
  const int nl = (int)(l_end - l_begin);

  // the zero rows before and after the input line of every slot (never overwritten)
  for (int i = tid; i < NS * 32; i += 256) {
    const int s = i >> 5, which = (i >> 4) & 1, piece = i & 15;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    *reinterpret_cast<__attribute__((address_space(3))) u32x4*>(ring + s * SLOT + GB + (which ? (W + 1) * 256 : 0) + piece * 16) =
        u32x4{0u, 0u, 0u, 0u};
  }
  __syncthreads();

  // ---- loader role.  Wave-load i of this wavefront: pixels 4 j .. 4 j + 3 of the line, j = wave * W16 + i; lane / 16
  // is the pixel, lane % 16 the 16-byte slot, which holds piece  slot ^ (4 * key)  with key = (LDS row) % 4.
  const int lr = lane >> 4, sp = lane & 15;
  const int pg = sp ^ (lr << 2);               // cotangent: LDS row = pixel
  const int px = sp ^ (((lr + 1) & 3) << 2);   // input: LDS row = pixel + 1
  const uint16_t* gsrc = g.A + ((size_t)l_begin * W + 4 * wave * W16 + lr) * g.lda + a0 + pg * 8;
  const uint16_t* xsrc = g.B + ((size_t)l_begin * W + 4 * wave * W16 + lr) * g.ldb + b0 + px * 8;
  int ld_n = 0, ld_y = (int)(l_begin % g.H), wslot = 0;
  auto issue = [&]() {
    lds_u8* slot = ring + wslot * SLOT;
    wslot = (wslot + 1 == NS) ? 0 : wslot + 1;
    // input line l + dy; where it is off the image the step is not multiplied: any line inside the tensor will do
    const int yy = ld_y + dy;
    const int64_t xoff = (yy >= 0 && yy < g.H) ? (int64_t)dy * W * g.ldb : 0;
#pragma unroll
    for (int i = 0; i < W16; ++i)
      __builtin_amdgcn_global_load_lds(gsrc + (size_t)4 * i * g.lda,
                                       (__attribute__((address_space(3))) void*)(slot + (wave * W16 + i) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < W16; ++i)
      __builtin_amdgcn_global_load_lds(xsrc + xoff + (size_t)4 * i * g.ldb,
                                       (__attribute__((address_space(3))) void*)(slot + GB + 256 + (wave * W16 + i) * 1024), 16, 0, 0);
    // advance, staying on the last line once it is reached (the extra loads of the pipeline tail stay in bounds)
    if (ld_n + 1 < nl) {
      ++ld_n;
      gsrc += (size_t)W * g.lda;
      xsrc += (size_t)W * g.ldb;
      ld_y = (ld_y + 1 == g.H) ? 0 : ld_y + 1;
    }
  };

  // ---- consumer role.  Lane = 32 kg + 16 g2 + s: k-octet kg, channel half g2 of a 32-channel block, s = 4 sr + sc
  // supplies row sr, channel group sc of a transposing read.
  const int kg = lane >> 5, g2 = (lane >> 4) & 1, s = lane & 15, sr = s >> 2, sc = s & 3;
  const int inrow = (2 * g2 + (sc >> 1)) * 16 + 8 * (sc & 1);
  int goff[4], xoffs[3], xrows[3];
#pragma unroll
  for (int a = 0; a < 4; ++a) goff[a] = (8 * kg + sr) * 256 + ((a ^ sr) * 64) + inrow;
#pragma unroll
  for (int d = 0; d < 3; ++d) {
    xoffs[d] = GB + ((wave ^ ((sr + d) & 3)) * 64) + inrow;   // in the zero row before the line
    xrows[d] = (8 * kg + sr + d) * 256;
  }
  // The transposing reads are written as assembly: the compiler, which cannot tell such a read from the slots that
  // direct loads still in flight are filling, would wait for ALL of them (vmcnt(0)) before each.  It does not
  // count these reads either: read_done() is the wait before their results are used.
  // read_done() is the wait before their results are used; the results pass through it as operands, so that nothing
  // that reads them can be placed before it.
  auto tr2 = [&](uint32_t p, v4s& lo, v4s& hi) {
    // rows r .. r + 3 and r + 4 .. r + 7: the 8 consecutive k of this lane's channel
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(p));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:1024" : "=v"(hi) : "v"(p));
  };
  auto read_done = [&](v4s (&r)[14]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7]), "+v"(r[8]),
                   "+v"(r[9]), "+v"(r[10]), "+v"(r[11]), "+v"(r[12]), "+v"(r[13]));
  };
  auto frag = [&](const v4s (&r)[14], int i) -> u16x8 {
    return __builtin_bit_cast(u16x8, __builtin_shufflevector(r[2 * i], r[2 * i + 1], 0, 1, 2, 3, 4, 5, 6, 7));
  };
  // fragments 0..3: cotangent blocks, 4..6: input at dx = -1, 0, +1
  // (xrow: 1 on a line whose input line l + dy is inside the image, else 0: all reads then go to the zero row)
  auto read_frag = [&](uint32_t slot, int ks, int xrow, v4s (&r)[14], auto which) {
    constexpr int i = decltype(which)::value;
    if constexpr (i < 4) {
      tr2(slot + goff[i] + ks * 16 * 256, r[2 * i], r[2 * i + 1]);
    } else {
      constexpr int d = i - 4;
      const uint32_t p = slot + xoffs[d] + xrow * (xrows[d] + ks * 16 * 256);
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r[8 + 2 * d]) : "v"(p));
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r[9 + 2 * d]) : "v"(p + xrow * 1024));
    }
  };
  auto read_frags = [&](uint32_t slot, int ks, int xrow, v4s (&r)[14]) {
    read_frag(slot, ks, xrow, r, std::integral_constant<int, 0>{});
    read_frag(slot, ks, xrow, r, std::integral_constant<int, 1>{});
    read_frag(slot, ks, xrow, r, std::integral_constant<int, 2>{});
    read_frag(slot, ks, xrow, r, std::integral_constant<int, 3>{});
    read_frag(slot, ks, xrow, r, std::integral_constant<int, 4>{});
    read_frag(slot, ks, xrow, r, std::integral_constant<int, 5>{});
    read_frag(slot, ks, xrow, r, std::integral_constant<int, 6>{});
  };
  f32x16 acc[12], sacc;
#pragma unroll
  for (int j = 0; j < 12; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;
#pragma unroll
  for (int q = 0; q < 16; ++q) sacc[q] = 0.f;
  u16x8 ones;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones[i] = Low<T>::from_f32(1.f);
  // cotangent sums: wavefront w forms those of the 32-channel block w; the k-steps are dealt out among the dy = 0
  // workgroups of this (co block, K-chunk)
  const bool sums = g.want_sums && dy == 0;
  const int sum_period = g.tiles_b;
  const int soff = (8 * kg + sr) * 256 + ((wave ^ sr) * 64) + inrow;
  int sum_phase = 0;
  auto wait_vm = [&](auto cnt) {
    constexpr int c = decltype(cnt)::value;
    static_assert(c < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (c & 15) | ((c >> 4) << 14));  // vmcnt only
  };

  // Pipeline: lines n + 1 .. n + NS - 2 are in LDS or on their way while line n is multiplied.  The wait for line n + 1
  // and the workgroup's barrier sit in the MIDDLE of line n's last k-step, behind half of its matrix instructions (the
  // matrix unit works on those while the wavefront waits), and the first fragments of line n + 1 are read behind the
  // other half: with one wavefront per SIMD a wait at the head of every line left the matrix unit idle for its length.
  auto mma_read = [&](auto which, const u16x8 (&fa)[4], const u16x8 (&fb)[3], bool rd, uint32_t rslot_addr, int rks, int rxrow,
                      v4s (&rto)[14]) {
    constexpr int i = decltype(which)::value;
    constexpr int a = i / 3, d = i % 3;
    acc[a * 3 + d] = Low<T>::mfma32(fa[a], fb[d], acc[a * 3 + d]);
    if constexpr (i < 7) {
      if (rd) read_frag(rslot_addr, rks, rxrow, rto, which);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto valid_line = [&](int y) { const int yy = y + dy; return (yy >= 0 && yy < g.H) ? 1 : 0; };
#pragma unroll
  for (int u = 0; u < NS - 1; ++u) issue();
  wait_vm(std::integral_constant<int, (NS - 2) * PERL>{});
  __builtin_amdgcn_s_barrier();
  int rslot = 0, c_y = (int)(l_begin % g.H);
  // input line off the image: multiply by zeros (this lane's columns of the zero row are read for every k), which keeps
  // the loop free of branches around the accumulators
  int xrow = valid_line(c_y);
  v4s raw[2][14];
  read_frags(ring_base, 0, xrow, raw[0]);
  // (par: which of the two fragment register sets the line's first k-step uses -- with one k-step per line, W = 16,
  // the sets alternate from line to line, and the lines are taken in pairs)
  auto do_line = [&](auto par) {
    constexpr int PAR = decltype(par)::value;
    const uint32_t slot = ring_base + rslot * SLOT;
    rslot = (rslot + 1 == NS) ? 0 : rslot + 1;
    c_y = (c_y + 1 == g.H) ? 0 : c_y + 1;
    const uint32_t slot_next = ring_base + rslot * SLOT;
    const int xrow_next = valid_line(c_y);
#pragma unroll
    for (int ks = 0; ks < W16; ++ks) {
      v4s (&cur)[14] = raw[(PAR + ks) & 1];
      v4s (&nxt)[14] = raw[(PAR + ks + 1) & 1];
      read_done(cur);
      __builtin_amdgcn_sched_barrier(0);
      // A wavefront issues a transposing read about every 10 ns (measured: 200 bytes per ns and compute unit with one
      // wavefront per SIMD), as long as a matrix instruction takes: the two reads of a fragment of the next k-step go
      // out behind each of seven matrix instructions of this one.
      u16x8 fa[4], fb[3];
#pragma unroll
      for (int a = 0; a < 4; ++a) fa[a] = frag(cur, a);
#pragma unroll
      for (int d = 0; d < 3; ++d) fb[d] = frag(cur, 4 + d);
      if (ks + 1 < W16) {
        mma_read(std::integral_constant<int, 0>{}, fa, fb, true, slot, ks + 1, xrow, nxt);
        mma_read(std::integral_constant<int, 1>{}, fa, fb, true, slot, ks + 1, xrow, nxt);
        mma_read(std::integral_constant<int, 2>{}, fa, fb, true, slot, ks + 1, xrow, nxt);
        mma_read(std::integral_constant<int, 3>{}, fa, fb, true, slot, ks + 1, xrow, nxt);
        mma_read(std::integral_constant<int, 4>{}, fa, fb, true, slot, ks + 1, xrow, nxt);
        mma_read(std::integral_constant<int, 5>{}, fa, fb, true, slot, ks + 1, xrow, nxt);
        mma_read(std::integral_constant<int, 6>{}, fa, fb, true, slot, ks + 1, xrow, nxt);
        mma_read(std::integral_constant<int, 7>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 8>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 9>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 10>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 11>{}, fa, fb, false, slot, 0, 0, nxt);
      } else {
        // last k-step of the line: matrix instructions 7..11 first (they take no reads with them) ...
        mma_read(std::integral_constant<int, 7>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 8>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 9>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 10>{}, fa, fb, false, slot, 0, 0, nxt);
        mma_read(std::integral_constant<int, 11>{}, fa, fb, false, slot, 0, 0, nxt);
        // ... then line n + 1 (past the chunk's end: a repeated copy of its last line, read but never multiplied) ...
        wait_vm(std::integral_constant<int, (NS - 3) * PERL>{});
        __builtin_amdgcn_s_barrier();  // everyone's part of line n + 1 is in LDS; everyone is done reading line n - 1
        __builtin_amdgcn_sched_barrier(0);
        issue();                       // line n + NS - 1 into the slot of line n - 1
        __builtin_amdgcn_sched_barrier(0);
        // ... and its first fragments behind matrix instructions 0..6
        mma_read(std::integral_constant<int, 0>{}, fa, fb, true, slot_next, 0, xrow_next, nxt);
        mma_read(std::integral_constant<int, 1>{}, fa, fb, true, slot_next, 0, xrow_next, nxt);
        mma_read(std::integral_constant<int, 2>{}, fa, fb, true, slot_next, 0, xrow_next, nxt);
        mma_read(std::integral_constant<int, 3>{}, fa, fb, true, slot_next, 0, xrow_next, nxt);
        mma_read(std::integral_constant<int, 4>{}, fa, fb, true, slot_next, 0, xrow_next, nxt);
        mma_read(std::integral_constant<int, 5>{}, fa, fb, true, slot_next, 0, xrow_next, nxt);
        mma_read(std::integral_constant<int, 6>{}, fa, fb, true, slot_next, 0, xrow_next, nxt);
      }
      if (sums) {
        if (sum_phase == bt) {
          v4s lo, hi;
          tr2(slot + soff + ks * 16 * 256, lo, hi);
          asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(lo), "+v"(hi));
          const u16x8 fs = __builtin_bit_cast(u16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          sacc = Low<T>::mfma32(fs, ones, sacc);
        }
        sum_phase = (sum_phase + 1 == sum_period) ? 0 : sum_phase + 1;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    xrow = xrow_next;
  };
  for (int n = 0; n < nl; n += (W16 == 1 ? 2 : 1)) {
    do_line(std::integral_constant<int, 0>{});
    if constexpr (W16 == 1) {
      if (n + 1 < nl) do_line(std::integral_constant<int, 1>{});
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tail's extra loads

  // ---- epilogue: plain read-modify-write, the slot belongs to this workgroup for the whole backward pass.  Its layout
  // follows the accumulator registers: float4 number ((j * 4 + q / 4) * 256 + thread), j = 3 a + dx + 1, holds rows (co)
  // 32 a + 8 (q / 4) + 4 (lane / 32) + 0..3 of column (ci) 32 wave + lane % 32.
  const float scale = g.h / g.ctl->S_step;
  float* slotf = g.part + ((size_t)(chunk * g.tiles_a + at) * gsize + tile) * CT_SLOT;
  float4* slot4 = reinterpret_cast<float4*>(slotf);
#pragma unroll
  for (int j0 = 0; j0 < 12; j0 += 3) {
    float4 old[3][4];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) old[t][q4] = slot4[((j0 + t) * 4 + q4) * 256 + tid];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 v = old[t][q4];
        v.x = fmaf(scale, acc[j0 + t][q4 * 4 + 0], v.x);
        v.y = fmaf(scale, acc[j0 + t][q4 * 4 + 1], v.y);
        v.z = fmaf(scale, acc[j0 + t][q4 * 4 + 2], v.z);
        v.w = fmaf(scale, acc[j0 + t][q4 * 4 + 3], v.w);
        slot4[((j0 + t) * 4 + q4) * 256 + tid] = v;
      }
  }
  if (sums && (lane & 31) == 0) {
    // column 0 of the sums block: rows 8 (q / 4) + 4 (lane / 32) + q % 4
    float* tail = slotf + 12 * 4096 + wave * 32;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      float* d = tail + 8 * (q >> 2) + 4 * kg + (q & 3);
      *d = fmaf(scale, sacc[q], *d);
    }
  }
}

// dW[co][ci][tap] and db[co] += sum over K-chunks of the private copies (end of the backward pass, or of a piece of
// piecewise-constant weights).  tiles_a, tiles_b: 128-channel blocks of the output / input channels.
__global__ void conv_wgrad_tr_reduce(float* __restrict__ G, int ldg, const float* __restrict__ part, int splits,
                                     int tiles_a, int tiles_b, int Na, int Nb, float* __restrict__ gb, const Ctl* ctl) {
  if (ctl->poison) return;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nW = (int64_t)Na * Nb * 9;
  if (i >= nW + Na) return;
  const size_t per_split = (size_t)tiles_a * tiles_b * 3 * CT_SLOT;
  if (i >= nW) {
    if (!gb) return;
    const int na = (int)(i - nW);
    float acc = 0.f;
    for (int c = 0; c < splits; ++c)
      for (int b = 0; b < tiles_b; ++b)
        acc += part[c * per_split + ((size_t)(na >> 7) * tiles_b * 3 + b * 3 + 1) * CT_SLOT + 12 * 4096 + (na & 127)];
    gb[na] += acc;
    return;
  }
  const int nb = (int)(i % Nb), t = (int)((i / Nb) % 9), na = (int)(i / ((int64_t)Nb * 9));
  // (position of element (co, ci, tap) in a workgroup's copy: see the epilogue of conv_wgrad_tr)
  const int a = (na & 127) >> 5, r = na & 31, wave = (nb & 127) >> 5, c = nb & 31;
  const int thread = wave * 64 + ((r >> 2) & 1) * 32 + c;
  const int j = a * 3 + t % 3;
  const size_t in_tile = ((size_t)(j * 4 + (r >> 3)) * 256 + thread) * 4 + (r & 3);
  const size_t tile = ((size_t)(na >> 7) * tiles_b + (nb >> 7)) * 3 + t / 3;
  float acc = 0.f;
  for (int c2 = 0; c2 < splits; ++c2) acc += part[c2 * per_split + tile * CT_SLOT + in_tile];
  G[(size_t)na * ldg + (size_t)nb * 9 + t] += acc;
}


// ---- The same design for 64 x 64 channels (the two-convolution velocity with a time channel): a drop-in for conv_wgrad
// (same argument structure, same layout of the private copies and of their tail of bias / time-channel sums, so
// conv_wgrad_reduce serves both).  One workgroup per K-chunk; its four wavefronts own the quadrants 32 co x 32 ci with all
// nine taps (144 accumulator registers): per k-step of 16 pixels one cotangent fragment and nine input fragments (three
// lines x three dx) for nine matrix instructions.  LDS holds a ring of 512 / W image lines (cotangent line + input line
// with a zero pixel at both ends; row = 64 channels = 128 bytes, the two 64-byte halves of a row swapped on every other
// pair of rows against bank conflicts); a pipeline step is 64 pixels (64 / W lines); lines arrive in groups of a step,
// six groups ahead.  The loaded range is the chunk's lines plus one line before and after (input halo).
// Bias and time-channel sums (and the time cotangent sums of the time-grid gradient): the wavefronts of the first input
// block multiply the cotangent fragment with a 0/1 fragment built in registers -- column t < 9: [pixel + tap t inside],
// column 9: ones -- into one more accumulator block, which is folded into fp32 sums with the stage's time factors
// whenever the stage changes (a K-chunk can span stages).
template <class T, bool TS, int W16>
__global__ __launch_bounds__(256, 1) void conv_wgrad_tr64(ConvWgrad g) {
  if (g.ctl->poison) return;
  constexpr int W = 16 * W16, LPS = 4 / W16, NL = 32 / W16;   // lines per step, lines in the ring
  constexpr int GB = W * 128, LSLOT = (2 * W + 2) * 128;      // cotangent line, then the input line with its zero rows
  constexpr int NG = NL / LPS;                                 // groups in the ring (8)
  constexpr int AHEAD = NG - 1;                                // groups requested ahead of the step being multiplied
  constexpr int D = (LPS == 1) ? 2 : 1;                        // step j needs the groups up to j + D
  typedef __attribute__((address_space(3))) uint8_t lds_u8;
  typedef short v4s __attribute__((ext_vector_type(4)));
  extern __shared__ __attribute__((aligned(16))) uint8_t cwt64_smem[];
  lds_u8* ring = (lds_u8*)cwt64_smem;
  const uint32_t ring_base = (uint32_t)(uintptr_t)ring;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t total_lines = g.rows / W;
  const int64_t c0 = (int64_t)blockIdx.z * (g.rows_per_split / W);
  int64_t c1 = c0 + g.rows_per_split / W;
  if (c1 > total_lines) c1 = total_lines;
  if (c0 >= c1) return;
  const int nl = (int)(c1 - c0);
  const int nsteps = (nl + LPS - 1) / LPS;
  const int lines_per_stage = (int)(g.R / W);

  // the zero rows before and after the input line of every ring slot (never overwritten)
  for (int i = tid; i < NL * 16; i += 256) {
    const int sl = i >> 4, which = (i >> 3) & 1, piece = i & 7;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    *reinterpret_cast<__attribute__((address_space(3))) u32x4*>(ring + sl * LSLOT + GB + (which ? (W + 1) * 128 : 0) + piece * 16) =
        u32x4{0u, 0u, 0u, 0u};
  }
  __syncthreads();

  // ---- loader role.  A group = LPS loaded lines = 64 pixels of cotangent + 64 of input = 16 wave-loads of 8 rows; this
  // wavefront's four: u = 4 wave + i -> (operand u / 8, pixels 8 (u % 8) .. of the group).  Loaded line lam is line
  // c0 - 1 + lam (clamped into the tensor: the two halo lines are only used where they are inside the image).
  const int lr = lane >> 3, sp = lane & 7;
  int ld_line[4], ld_px[4], ld_dst[4];
  const uint16_t* ld_src[4];
  int ld_ldx[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int u = 4 * wave + i, op = u >> 3, px = 8 * (u & 7) + lr;   // pixel within the group
    ld_line[i] = px / W;
    ld_px[i] = px % W;
    const int prow = op ? ld_px[i] + 1 : ld_px[i];                    // LDS row of the lane's pixel
    const int piece = sp ^ (((prow >> 1) & 1) << 2);
    ld_src[i] = (op ? g.B : g.A) + piece * 8;
    ld_ldx[i] = op ? g.ldb : g.lda;
    ld_dst[i] = (op ? GB + 128 : 0) + (8 * (u & 7) % W) * 128;        // (+ the line's slot)
  }
  int ld_group = 0;
  auto issue = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int lam = ld_group * LPS + ld_line[i];
      int64_t line = c0 - 1 + lam;
      line = line < 0 ? 0 : (line >= total_lines ? total_lines - 1 : line);
      const int slot = lam % NL;
      __builtin_amdgcn_global_load_lds(ld_src[i] + ((size_t)line * W + ld_px[i]) * ld_ldx[i],
                                       (__attribute__((address_space(3))) void*)(ring + slot * LSLOT + ld_dst[i]), 16, 0, 0);
    }
    ++ld_group;
  };

  // ---- consumer role.  Lane = 32 kg + 16 g2 + s, s = 4 sr + sc: see conv_wgrad_tr.
  const int kg = lane >> 5, g2 = (lane >> 4) & 1, sfrag = lane & 15, sr = sfrag >> 2, sc = sfrag & 3;
  const int incol = 32 * g2 + 8 * sc;
  const int goff = (8 * kg + sr) * 128 + ((wm ^ ((sr >> 1) & 1)) * 64) + incol;
  int xcol[3], xrow[3];
#pragma unroll
  for (int d = 0; d < 3; ++d) {
    xcol[d] = GB + ((wn ^ (((sr + d) >> 1) & 1)) * 64) + incol;   // in the zero row before the line
    xrow[d] = (8 * kg + sr + d) * 128;
  }
  auto tr1 = [&](uint32_t p, v4s& v) { asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(p)); };
  // fragments of a k-step: 0 = cotangent, 1 + 3 dyv + dxv = input of tap (dyv, dxv); two reads each
  // what a k-step needs to know of its image line: LDS positions of the cotangent line and of the three input lines,
  // which of those are inside the image, the on / off word of this lane's column of the sums block
  struct LineCtx {
    uint32_t gline, xline[3];
    int vy[3];
    uint32_t mbase;
  };
  auto read_frag = [&](auto which, const LineCtx& c, int ks, v4s (&r)[20]) {
    constexpr int i = decltype(which)::value;
    if constexpr (i == 0) {
      const uint32_t p = c.gline + goff + ks * 16 * 128;
      tr1(p, r[0]);
      tr1(p + 512, r[1]);
    } else {
      constexpr int dyv = (i - 1) / 3, dxv = (i - 1) % 3;
      // (input line off the image: this lane's columns of the zero row, for every k)
      const uint32_t p = c.xline[dyv] + xcol[dxv] + c.vy[dyv] * (xrow[dxv] + ks * 16 * 128);
      tr1(p, r[2 * i]);
      tr1(p + c.vy[dyv] * 512, r[2 * i + 1]);
    }
  };
  auto read_done = [&](v4s (&r)[20]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7]), "+v"(r[8]),
                   "+v"(r[9]));
    asm volatile("" : "+v"(r[10]), "+v"(r[11]), "+v"(r[12]), "+v"(r[13]), "+v"(r[14]), "+v"(r[15]), "+v"(r[16]), "+v"(r[17]),
                      "+v"(r[18]), "+v"(r[19]));
  };
  auto frag = [&](const v4s (&r)[20], int i) -> u16x8 {
    return __builtin_bit_cast(u16x8, __builtin_shufflevector(r[2 * i], r[2 * i + 1], 0, 1, 2, 3, 4, 5, 6, 7));
  };
  f32x16 acc[9], am;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[t][q] = 0.f;
#pragma unroll
  for (int q = 0; q < 16; ++q) am[q] = 0.f;
  // sums: column n = lane % 32 of the extra block is tap n (n < 9) or the plain sum (n = 9)
  const bool sums = g.want_sums && wn == 0;
  const int ncol = lane & 31;
  const uint32_t one2 = (uint32_t)Low<T>::from_f32(1.f) * 0x10001u;
  const int vsel = ncol < 9 ? ncol / 3 : (ncol == 9 ? 3 : 4);           // bit of the validity word that switches the column on
  const bool edge_l = ncol < 9 && ncol % 3 == 0 && kg == 0;             // dx = -1: pixel 0 of the line is off
  const bool edge_r = ncol < 9 && ncol % 3 == 2 && kg == 1;             // dx = +1: pixel W - 1 of the line is off
  float s_tau[16], s_one[16], s_c[16];   // tau-, un- and c_j-weighted sums of this lane's column
#pragma unroll
  for (int q = 0; q < 16; ++q) s_tau[q] = s_one[q] = s_c[q] = 0.f;
  // (image row and stage of the line being multiplied are stepped from line to line: no division in the loop)
  int cur_stage = (int)(c0 / lines_per_stage);
  int stage_end_m = (int)((int64_t)(cur_stage + 1) * lines_per_stage - c0);   // first line (chunk-relative) of the next stage

  auto flush_sums = [&]() {
    float tau = 0.f, cj = 0.f;
#pragma unroll
    for (int q = 0; q < kMaxStages; ++q) {
      tau = (q == cur_stage) ? g.taus[q] : tau;
      cj = (q == cur_stage) ? g.cs[q] : cj;
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      s_tau[q] = fmaf(tau, am[q], s_tau[q]);
      s_one[q] += am[q];
      if (TS) s_c[q] = fmaf(cj, am[q], s_c[q]);
      am[q] = 0.f;
    }
  };
  auto wait_vm = [&](auto cnt) {
    constexpr int c = decltype(cnt)::value;
    static_assert(c < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (c & 15) | ((c >> 4) << 14));  // vmcnt only
  };

  // (image row and stage are stepped from line to line: no division in the loop)
  int y_ctx = (int)(c0 % g.H);   // image row of the next line that gets a context (lines are taken in order)
  auto make_ctx = [&](int m) -> LineCtx {
    LineCtx c;
    const int lam = m + 1;      // cotangent line c0 + m = loaded line m + 1
    c.gline = ring_base + (lam % NL) * LSLOT;
    c.xline[0] = ring_base + ((lam - 1) % NL) * LSLOT;
    c.xline[1] = c.gline;
    c.xline[2] = ring_base + ((lam + 1) % NL) * LSLOT;
    c.vy[0] = y_ctx > 0 ? 1 : 0;
    c.vy[1] = 1;
    c.vy[2] = y_ctx < g.H - 1 ? 1 : 0;
    const uint32_t vword = (uint32_t)(c.vy[0] | 2 | (c.vy[2] << 2) | 8);
    c.mbase = ((vword >> vsel) & 1u) ? one2 : 0u;
    y_ctx = (y_ctx + 1 == g.H) ? 0 : y_ctx + 1;
    return c;
  };
  auto read_all = [&](const LineCtx& c, int ks, v4s (&r)[20]) {
    read_frag(std::integral_constant<int, 0>{}, c, ks, r);
    read_frag(std::integral_constant<int, 1>{}, c, ks, r);
    read_frag(std::integral_constant<int, 2>{}, c, ks, r);
    read_frag(std::integral_constant<int, 3>{}, c, ks, r);
    read_frag(std::integral_constant<int, 4>{}, c, ks, r);
    read_frag(std::integral_constant<int, 5>{}, c, ks, r);
    read_frag(std::integral_constant<int, 6>{}, c, ks, r);
    read_frag(std::integral_constant<int, 7>{}, c, ks, r);
    read_frag(std::integral_constant<int, 8>{}, c, ks, r);
    read_frag(std::integral_constant<int, 9>{}, c, ks, r);
  };

  // Pipeline: step j multiplies cotangent lines [LPS j, LPS (j + 1)) of the chunk = loaded lines + 1, four k-steps, and
  // needs the loaded groups up to j + D.  With one wavefront per SIMD nothing runs beside a wait or a block of reads, so:
  // the fragments of k-step i + 1 are read between the matrix instructions of k-step i (also from line to line and from
  // step to step), and the wait for step j + 1's groups, the barrier and the request of group j + AHEAD sit behind the
  // first five matrix instructions of step j's last k-step.  Group j + AHEAD takes the ring position of group j - 1,
  // whose lines step j - 1 was the last to read.
#pragma unroll
  for (int u = 0; u < AHEAD; ++u) issue();
  wait_vm(std::integral_constant<int, (AHEAD - 2 - D) * 4>{});
  __builtin_amdgcn_s_barrier();
  v4s raw[2][20];
  LineCtx cur = make_ctx(0);
  read_all(cur, 0, raw[0]);
  for (int j = 0; j < nsteps; ++j) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int li = i / W16, ks = i % W16;
      const int m = j * LPS + li;
      const bool live = m < nl;            // (uniform: a chunk's last step may be cut short)
      // the k-step after this one
      const int nks = (i + 1) % W16;
      LineCtx nxt = cur;
      if (nks == 0) nxt = make_ctx(i == 3 ? (j + 1) * LPS : m + 1);
      v4s (&rc)[20] = raw[i & 1];
      v4s (&rn)[20] = raw[(i + 1) & 1];
      read_done(rc);
      if (ks == 0 && sums && m >= stage_end_m && live) {
        flush_sums();
        ++cur_stage;
        stage_end_m += lines_per_stage;
      }
      __builtin_amdgcn_sched_barrier(0);
      // (a k-step past the chunk's end multiplies zeros: no branch around the accumulators)
      u16x8 fa = frag(rc, 0);
      if (!live) fa = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
      u16x8 fb[9];
#pragma unroll
      for (int t = 0; t < 9; ++t) fb[t] = frag(rc, 1 + t);
      auto mm = [&](auto which) {
        constexpr int t = decltype(which)::value;
        acc[t] = Low<T>::mfma32(fa, fb[t], acc[t]);
      };
      auto rd = [&](auto which) { read_frag(which, nxt, nks, rn); };
      typedef std::integral_constant<int, 0> I0; typedef std::integral_constant<int, 1> I1;
      typedef std::integral_constant<int, 2> I2; typedef std::integral_constant<int, 3> I3;
      typedef std::integral_constant<int, 4> I4; typedef std::integral_constant<int, 5> I5;
      typedef std::integral_constant<int, 6> I6; typedef std::integral_constant<int, 7> I7;
      typedef std::integral_constant<int, 8> I8; typedef std::integral_constant<int, 9> I9;
#define CWT64_FENCE __builtin_amdgcn_sched_barrier(0)
      if (i < 3) {
        // every matrix instruction takes the reads of a fragment of the next k-step with it
        mm(I0{}); rd(I0{}); rd(I1{}); CWT64_FENCE;
        mm(I1{}); rd(I2{}); CWT64_FENCE;
        mm(I2{}); rd(I3{}); CWT64_FENCE;
        mm(I3{}); rd(I4{}); CWT64_FENCE;
        mm(I4{}); rd(I5{}); CWT64_FENCE;
        mm(I5{}); rd(I6{}); CWT64_FENCE;
        mm(I6{}); rd(I7{}); CWT64_FENCE;
        mm(I7{}); rd(I8{}); CWT64_FENCE;
        mm(I8{}); rd(I9{}); CWT64_FENCE;
      } else {
        mm(I0{}); mm(I1{}); mm(I2{}); mm(I3{}); mm(I4{});
        CWT64_FENCE;
        wait_vm(std::integral_constant<int, (AHEAD - 2 - D) * 4>{});
        __builtin_amdgcn_s_barrier();   // everyone's part of step j + 1's groups is in LDS; everyone is done with step j - 1
        CWT64_FENCE;
        issue();
        CWT64_FENCE;
        mm(I5{}); rd(I0{}); rd(I1{}); rd(I2{}); CWT64_FENCE;
        mm(I6{}); rd(I3{}); rd(I4{}); rd(I5{}); CWT64_FENCE;
        mm(I7{}); rd(I6{}); rd(I7{}); CWT64_FENCE;
        mm(I8{}); rd(I8{}); rd(I9{}); CWT64_FENCE;
      }
#undef CWT64_FENCE
      if (sums) {
        // this lane's 8 pixels of the k-step against its column's tap: all on, except the line's first / last pixel
        uint32_t mk[4] = {cur.mbase, cur.mbase, cur.mbase, cur.mbase};
        if (edge_l && ks == 0) mk[0] &= 0xffff0000u;
        if (edge_r && ks == W16 - 1) mk[3] &= 0x0000ffffu;
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        am = Low<T>::mfma32(fa, __builtin_bit_cast(u16x8, u32x4{mk[0], mk[1], mk[2], mk[3]}), am);
      }
      __builtin_amdgcn_sched_barrier(0);
      cur = nxt;
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the requests past the chunk's end

  const float scale = g.h / g.ctl->S_step;
  float* slotf = g.part + (size_t)blockIdx.z * CW_SLOT;
  if (g.want_sums) {
    float p0 = 0.f, p1 = 0.f;
    if (sums) {
      flush_sums();
      // column n of block wm: rows (co) 32 wm + 8 (q / 4) + 4 (lane / 32) + q % 4; tail entry 0 = bias, 1 + t = tap t
      if (ncol <= 9) {
        const int e = ncol == 9 ? 0 : 1 + ncol;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int co = 32 * wm + 8 * (q >> 2) + 4 * kg + (q & 3);
          float* d = slotf + 9 * 4096 + co * 16 + e;
          *d = fmaf(scale, ncol == 9 ? s_one[q] : s_tau[q], *d);
          if (TS && ncol < 9 && co < g.Na) {
            const float wv = g.wt[ncol * g.ldwt + co];
            p0 = fmaf(wv, s_one[q] - s_c[q], p0);
            p1 = fmaf(wv, s_c[q], p1);
          }
        }
      }
    }
    if (TS) block_sum2(scale * p0, scale * p1, g.tpart + 2 * (size_t)blockIdx.z);
  }
  // plain read-modify-write in conv_wgrad's layout: float4 number ((tap * 4 + q / 4) * 256 + thread) holds rows (co)
  // 32 wm + 8 (q / 4) + 4 (lane / 32) + 0..3 of column (ci) 32 wn + lane % 32
  float4* slot = reinterpret_cast<float4*>(slotf);
#pragma unroll
  for (int t0 = 0; t0 < 9; t0 += 3) {
    float4 old[3][4];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) old[t][q4] = slot[((t0 + t) * 4 + q4) * 256 + tid];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 v = old[t][q4];
        v.x = fmaf(scale, acc[t0 + t][q4 * 4 + 0], v.x);
        v.y = fmaf(scale, acc[t0 + t][q4 * 4 + 1], v.y);
        v.z = fmaf(scale, acc[t0 + t][q4 * 4 + 2], v.z);
        v.w = fmaf(scale, acc[t0 + t][q4 * 4 + 3], v.w);
        slot[((t0 + t) * 4 + q4) * 256 + tid] = v;
      }
  }
}
constexpr size_t conv_wgrad_tr64_lds_bytes(int W) { return (size_t)(512 / W) * (2 * W + 2) * 128; }

}  // namespace rampde
