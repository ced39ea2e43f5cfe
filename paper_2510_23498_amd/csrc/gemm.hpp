// MFMA contractions of the velocity network and of its vector-Jacobian products.
//
//   gemm_nt : C[M, N] = epilogue( A[M, K] * W[N, K]^T )        (both operands K-contiguous)
//             forward layers  (paper Alg. 1, the low-precision evaluation of Phi)  and the
//             input-cotangent products  delta_{l-1} = (delta_l W_l) * tanh'  of eq. (vjp).
//             With CONV the rows of A are pixels of a channels-last image and the K axis
//             runs over (3x3 tap, channel): an implicit-GEMM convolution with zero padding.
//   gemm_tn : G[Na, Nb] += scale * sum_k A[k, Na] * B[k, Nb]   (contraction over rows)
//             the parameter-gradient products  dW_l = delta_l^T act_{l-1}, accumulated in
//             fp32 straight into the gradient vector (paper Sec. 3, update of g).
//
// Tiles are built from v_mfma_f32_32x32x16_{f16,bf16}; a workgroup is 4 wavefronts (2x2).
// Low-precision values travel as raw 16-bit patterns (uint16_t).
#pragma once
#include <type_traits>

#include "common.hpp"

namespace rampde {

constexpr int BK = 64;        // K extent of one LDS tile
constexpr int LDS_PITCH = BK + 8;  // elements; 144 B rows keep 16-byte reads conflict-light

struct GemmNT {
  const uint16_t* A; int lda;
  const uint16_t* W; int ldw;
  uint16_t* C; int ldc;
  int M, N, K;                 // N, K multiples of 64 (padded)
  const float* bias;           // [N] fp32 (already rounded to low) or null
  const float* wt;             // time weights: MLP [N]; conv [9][N]; or null
  float tau;                   // stage time, already rounded to low
  int act_tanh;                // activation applied before rounding: 0 none, 1 tanh, 2 ReLU
  int negate;                  // store the negated result (the -W^T of the parabolic block, Sec. 6.3)
  // exact-trace row of a normalising-flow state (Sec. 6.1): with dact, the activation's cotangent gets the
  // term 2 kbar_l[m] c[n] act[m][n] before the tanh' factor (tr_kl: the l column of the slope cotangent)
  const float* tr_c; const uint16_t* tr_kl; int tr_ld;
  const uint16_t* dact; int ldd;  // stored activation for the factor (1 - act^2), or null
  Ctl* ctl;                    // may be null (forward pass)
  int detect;                  // raise ctl->nonfinite if any output is inf/nan
  // conv geometry (CONV only)
  int H, Wd, Cpad;
};

template <class T, int MI, int NI, bool CONV>
__global__ __launch_bounds__(256) void gemm_nt(GemmNT g) {
  if (g.ctl && g.ctl->poison) return;
  constexpr int BM = 64 * MI, BN = 64 * NI;
  __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDS_PITCH];
  __shared__ __attribute__((aligned(16))) uint16_t sW[BN * LDS_PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;

  constexpr int A_CHUNKS = BM * (BK / 8) / 256;  // 16-byte chunks per thread
  constexpr int W_CHUNKS = BN * (BK / 8) / 256;
  u16x8 ra[A_CHUNKS], rw[W_CHUNKS];

  // per-chunk row bookkeeping (row index and, for conv, pixel coordinates)
  int a_row[A_CHUNKS], a_kc[A_CHUNKS], a_x[A_CHUNKS], a_y[A_CHUNKS];
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    int id = tid + i * 256;
    a_row[i] = m0 + (id >> 3);
    a_kc[i] = (id & 7) * 8;
    if (CONV) {
      a_x[i] = a_row[i] % g.Wd;
      a_y[i] = (a_row[i] / g.Wd) % g.H;
    }
  }

  auto load_tiles = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (a_row[i] < g.M) {
        if (CONV) {
          int per_tap = g.Cpad / BK;
          int tap = kt / per_tap, c0 = (kt - tap * per_tap) * BK;
          int dy = tap / 3 - 1, dx = tap % 3 - 1;
          int yy = a_y[i] + dy, xx = a_x[i] + dx;
          if (yy >= 0 && yy < g.H && xx >= 0 && xx < g.Wd) {
            const uint16_t* p = g.A + (size_t)(a_row[i] + dy * g.Wd + dx) * g.lda + c0 + a_kc[i];
            v = *reinterpret_cast<const u16x8*>(p);
          }
        } else {
          const uint16_t* p = g.A + (size_t)a_row[i] * g.lda + kt * BK + a_kc[i];
          v = *reinterpret_cast<const u16x8*>(p);
        }
      }
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
      int id = tid + i * 256;
      const uint16_t* p = g.W + (size_t)(n0 + (id >> 3)) * g.ldw + kt * BK + (id & 7) * 8;
      rw[i] = *reinterpret_cast<const u16x8*>(p);
    }
  };
  auto store_tiles = [&]() {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      int id = tid + i * 256;
      *reinterpret_cast<u16x8*>(&sA[(id >> 3) * LDS_PITCH + (id & 7) * 8]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
      int id = tid + i * 256;
      *reinterpret_cast<u16x8*>(&sW[(id >> 3) * LDS_PITCH + (id & 7) * 8]) = rw[i];
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int a = 0; a < MI; ++a)
#pragma unroll
    for (int b = 0; b < NI; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // conv: the constant time channel contributes tau * (sum of its tap weights whose neighbour pixel
  // exists).  That sum depends only on which of the four borders the pixel touches: 16 cases per
  // output channel, tabulated once (same summation order as tap-by-tap accumulation).
  __shared__ float s_tt[CONV ? 16 * BN : 1];
  if (CONV && g.wt) {
    for (int i = tid; i < 16 * BN; i += 256) {
      const int combo = i / BN, n = n0 + i % BN;
      float sum = 0.f;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int dy = t / 3 - 1, dx = t % 3 - 1;
        const bool ok = (dy >= 0 || (combo & 8)) && (dy <= 0 || (combo & 4)) && (dx >= 0 || (combo & 2)) &&
                        (dx <= 0 || (combo & 1));
        if (ok) sum += g.wt[t * g.N + n] * g.tau;
      }
      s_tt[i] = sum;
    }
  }

  const int KT = g.K / BK;
  load_tiles(0);
  store_tiles();
  __syncthreads();
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  for (int kt = 0; kt < KT; ++kt) {
    if (kt + 1 < KT) load_tiles(kt + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      u16x8 fa[MI], fb[NI];
#pragma unroll
      for (int a = 0; a < MI; ++a)
        fa[a] = *reinterpret_cast<const u16x8*>(&sA[(wm * 32 * MI + a * 32 + frow) * LDS_PITCH + kk * 16 + fk]);
#pragma unroll
      for (int b = 0; b < NI; ++b)
        fb[b] = *reinterpret_cast<const u16x8*>(&sW[(wn * 32 * NI + b * 32 + frow) * LDS_PITCH + kk * 16 + fk]);
#pragma unroll
      for (int a = 0; a < MI; ++a)
#pragma unroll
        for (int b = 0; b < NI; ++b) acc[a][b] = Low<T>::mfma32(fa[a], fb[b], acc[a][b]);
    }
    __syncthreads();
    if (kt + 1 < KT) {
      store_tiles();
      __syncthreads();
    }
  }

  // ---- epilogue: accumulator lane layout of the 32x32 tile:
  //      column = lane % 32, row = 8 * (r / 4) + 4 * (lane / 32) + r % 4
  bool bad = false;
#pragma unroll
  for (int b = 0; b < NI; ++b) {
    const int nn = wn * 32 * NI + b * 32 + (lane & 31);
    const int n = n0 + nn;
    const float bv = g.bias ? g.bias[n] : 0.f;
    const float tv = (!CONV && g.wt) ? g.wt[n] * g.tau : 0.f;
#pragma unroll
    for (int a = 0; a < MI; ++a) {
      // pixel coordinates of the lane's first row; the other 15 rows follow by stepping
      const int mb = m0 + wm * 32 * MI + a * 32 + 4 * (lane >> 5);
      int x = 0, y = 0;
      if (CONV && g.wt) {
        x = mb % g.Wd;
        y = (mb / g.Wd) % g.H;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mb + 8 * (r >> 2) + (r & 3);
        if (CONV && g.wt && r > 0) {
          x += (r & 3) ? 1 : 5;
          while (x >= g.Wd) {
            x -= g.Wd;
            y = (y + 1 == g.H) ? 0 : y + 1;
          }
        }
        if (m < g.M) {
          float v = acc[a][b][r] + bv;
          if (g.wt) {
            if (CONV) {
              const int combo = ((y > 0) << 3) | ((y < g.H - 1) << 2) | ((x > 0) << 1) | (x < g.Wd - 1 ? 1 : 0);
              v += s_tt[combo * BN + nn];
            } else {
              v += tv;
            }
          }
          if (g.act_tanh == 1) v = act_tanh(v);
          else if (g.act_tanh == 2) v = fmaxf(v, 0.f);
          if (g.negate) v = -v;
          if (g.dact) {
            float av = Low<T>::to_f32(g.dact[(size_t)m * g.ldd + n]);
            if (g.tr_c) v = fmaf(2.f * g.tr_c[n] * av, Low<T>::to_f32(g.tr_kl[(size_t)m * g.tr_ld]), v);
            v = v * (1.f - av * av);
          }
          uint16_t q = Low<T>::from_f32(v);
          bad = bad || Low<T>::nonfinite(q);
          g.C[(size_t)m * g.ldc + n] = q;
        }
      }
    }
  }
  if (g.detect) raise_if_any(bad, g.ctl);
}

// ------------------------------------------------------------------------------------
struct GemmTN {
  const uint16_t* A; int lda;   // [rows, >= Na] cotangents delta_l
  const uint16_t* B; int ldb;   // [rows, >= Nb] layer inputs act_{l-1}
  int64_t rows;                 // contraction length (stages * batch rows)
  int rows_per_split;           // multiple of BK
  float* G; int ldg;            // fp32 gradient block, row pitch ldg
  int Na, Nb;                   // valid extents (unpadded)
  int NaPad, NbPad;             // padded extents (multiples of 64): columns that exist in A / B
  float h;                      // step size; scale = h / ctl->S_step
  const Ctl* ctl;
  // conv: B rows are gathered with a tap shift, G index = na*ldg + nb*9 + tap
  int H, Wd, taps;              // taps = 1 (dense) or 9 (conv)
};

template <class T, bool CONV>
__global__ __launch_bounds__(256) void gemm_tn(GemmTN g) {
  if (g.ctl->poison) return;
  constexpr int BM = 128, BN = 128;
  __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDS_PITCH];  // [feature][k]
  __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LDS_PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int a0 = blockIdx.x * BM, b0 = blockIdx.y * BN;
  int split = blockIdx.z, tap = 0;
  if (CONV) { tap = split % 9; split /= 9; }
  const int dy = tap / 3 - 1, dx = tap % 3 - 1;
  const int64_t k_begin = (int64_t)split * g.rows_per_split;
  int64_t k_end = k_begin + g.rows_per_split;
  if (k_end > g.rows) k_end = g.rows;

  // each thread owns one 8(k) x 8(feature) block of A (threads 0..127) or B (128..255)
  const bool isB = tid >= 128;
  const int t7 = tid & 127;
  const int fg = t7 & 15, kg = t7 >> 4;
  u16x8 r[8];

  auto load_block = [&](int64_t k0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int64_t k = k0 + kg * 8 + i;
      u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (k < k_end) {
        if (!isB) {
          if (a0 + fg * 8 < g.NaPad) v = *reinterpret_cast<const u16x8*>(g.A + (size_t)k * g.lda + a0 + fg * 8);
        } else if (b0 + fg * 8 >= g.NbPad) {
          // column block beyond the padded width: stays zero
        } else if (CONV) {
          int x = (int)(k % g.Wd), y = (int)((k / g.Wd) % g.H);
          int yy = y + dy, xx = x + dx;
          if (yy >= 0 && yy < g.H && xx >= 0 && xx < g.Wd)
            v = *reinterpret_cast<const u16x8*>(g.B + (size_t)(k + dy * g.Wd + dx) * g.ldb + b0 + fg * 8);
        } else {
          v = *reinterpret_cast<const u16x8*>(g.B + (size_t)k * g.ldb + b0 + fg * 8);
        }
      }
      r[i] = v;
    }
  };
  auto store_block = [&]() {
    uint16_t* s = isB ? sB : sA;
#pragma unroll
    for (int f = 0; f < 8; ++f) {
      u16x8 o;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = r[i][f];
      *reinterpret_cast<u16x8*>(&s[(fg * 8 + f) * LDS_PITCH + kg * 8]) = o;
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.f;

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  if (k_begin < k_end) {
    load_block(k_begin);
    store_block();
    __syncthreads();
    for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
      const bool more = k0 + BK < k_end;
      if (more) load_block(k0 + BK);
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        u16x8 fa[2], fb[2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
          fa[a] = *reinterpret_cast<const u16x8*>(&sA[(wm * 64 + a * 32 + frow) * LDS_PITCH + kk * 16 + fk]);
#pragma unroll
        for (int b = 0; b < 2; ++b)
          fb[b] = *reinterpret_cast<const u16x8*>(&sB[(wn * 64 + b * 32 + frow) * LDS_PITCH + kk * 16 + fk]);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < 2; ++b) acc[a][b] = Low<T>::mfma32(fa[a], fb[b], acc[a][b]);
      }
      __syncthreads();
      if (more) {
        store_block();
        __syncthreads();
      }
    }
  }

  const float scale = g.h / g.ctl->S_step;
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int nb = b0 + wn * 64 + b * 32 + (lane & 31);
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int na = a0 + wm * 64 + a * 32 + 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3);
        if (na < g.Na && nb < g.Nb) {
          size_t idx = CONV ? ((size_t)na * g.ldg + (size_t)nb * 9 + tap) : ((size_t)na * g.ldg + nb);
          unsafeAtomicAdd(&g.G[idx], scale * acc[a][b][q]);
        }
      }
    }
  }
}


// ------------------------------------------------------------------------------------
// Weight gradient of a 3x3 zero-padded convolution on channels-last rows (paper Sec. 3, update
// of g, for the convolutional velocity):
//   dW[co][ci][tap] += scale * sum_k delta[k][co] * x[k + dy W + dx][ci] * [pixel (y+dy, x+dx) inside]
// over the rows k (pixels of all samples and stages) of one K-chunk, all 9 taps in one workgroup.
// A workgroup owns a 64 (co) x 64 (ci) block.  Per k-step of CW_KS = 128 rows it transposes into LDS
//   - the cotangent tile, in 3 copies: as is, and with the rows of the first / last image line
//     zeroed (taps with dy = -1 / +1: the line above / below does not exist),
//   - the input tile with a halo of one image line on both sides (CW_KS + 2 W rows), in 3 copies
//     shifted by dx = -1, 0, +1 rows with the pixels that fall off the line zeroed,
// so that the operand fragment of tap (dy, dx) is an aligned read at row offset (1 + dy) W of copy
// dx, and every tap is one MFMA per 16 k.  Needs W % 8 == 0 (the 8-row blocks a thread transposes
// then lie within one image line), W <= 64 and rows per stage % CW_KS == 0 (a k-step lies within one stage).
struct ConvWgrad {
  const uint16_t* A; int lda;   // [rows, >= 64 gridDim.x] cotangents of the layer's output
  const uint16_t* B; int ldb;   // [rows, >= 64 gridDim.y] the layer's input
  int64_t rows;                 // stages * batch * H * W
  int rows_per_split;           // multiple of CW_KS
  float* part;                  // [gridDim.z][gridDim.x][gridDim.y][CW_SLOT] fp32 (tap blocks in register order): the private
                                // accumulators of every (K-chunk, channel block), summed at the end of the pass
  float h;                      // scale = h / ctl->S_step
  const Ctl* ctl;
  int H, Wd;
  // bias and time-channel gradients (folded into the workgroups of the first input-channel block):
  //   db[co] += scale * sum_k delta[k][co];   dwt[co][tap] += scale * sum_k tau(k) delta[k][co] * [tap inside]
  // (accumulated in the tail of the private copy: atomics on these few addresses from every workgroup
  // would serialise in the L2)
  bool want_sums;
  int Na;                       // valid output channels
  int64_t R;                    // rows per stage (a multiple of CW_KS)
  float taus[kMaxStages];       // stage times
  // time-grid gradient (paper Sec. 3, update lines of t'): the time cotangent of stage j is
  // taubar_j = sum_{k, co, tap} delta[k][co] * wt[tap][co] * [tap inside]; the step's sums get
  //   tpart[0] += scale * sum_j (1 - c_j) taubar_j,   tpart[1] += scale * sum_j c_j taubar_j
  const float* wt; int ldwt;    // rounded time-channel weights [9][ldwt], or null
  float* tpart;                 // or null: the launch's table of per-workgroup slots (fold_time_slots)
  float cs[kMaxStages];         // c_j
};

constexpr int CW_KS = 128;          // pixels (rows) per k-step
constexpr int CW_SLOT = 9 * 4096 + 64 * 16;  // floats of a workgroup's private copy: 9 tap blocks, then per output
                                             // channel [db, dwt[9 taps], 6 unused]
constexpr int CW_PA = CW_KS + 8;    // LDS pitch of the cotangent copies (elements)
// loader items (8 rows x 8 channels) per thread for image lines of up to 32 / up to 64 pixels
constexpr int CW_MAXI_LO = (3 * (CW_KS + 64) + CW_KS + 255) / 256;
constexpr int CW_MAXI_HI = (3 * (CW_KS + 128) + CW_KS + 255) / 256;
inline size_t conv_wgrad_lds_bytes(int Wd) { return (size_t)(3 * 64 * CW_PA + 3 * 64 * (CW_KS + 2 * Wd + 8)) * 2; }

// TS: also form the time cotangent sums for the time-grid gradient (g.tpart, g.wt non-null).
// MAXI: loader items (8 rows x 8 channels) per thread: CW_MAXI_LO = 3 cover image lines of up to 32
// pixels, CW_MAXI_HI = 4 are needed for lines of 64 (that instance spills a few registers).
template <class T, bool TS, int MAXI>
__global__ __launch_bounds__(256) void conv_wgrad(ConvWgrad g) {
  if (g.ctl->poison) return;
  extern __shared__ __attribute__((aligned(16))) uint16_t cw_smem[];
  const int W = g.Wd, XR = CW_KS + 2 * W, PX = XR + 8;
  uint16_t* sA = cw_smem;                 // [3 (dy)][64 co][CW_PA]
  uint16_t* sX = cw_smem + 3 * 64 * CW_PA;  // [3 (dx)][64 ci][PX]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int a0 = blockIdx.x * 64, b0 = blockIdx.y * 64;
  const int64_t k_begin = (int64_t)blockIdx.z * g.rows_per_split;
  int64_t k_end = k_begin + g.rows_per_split;
  if (k_end > g.rows) k_end = g.rows;
  if (k_begin >= k_end) return;

  // work items of the transposing loaders: 8 rows x 8 channels each.  Items [0, CW_KS): the
  // cotangent tile (8-row block, channel group) - only a thread's first item can be one, and it is
  // one for whole wavefronts; then 3 XR items of the input copies (copy, 8-row block, channel group).
  // The pixel coordinates of an item (x of its first row; image line y for cotangent items) are
  // stepped from k-step to k-step: no division inside the loop.
  const int nXb = XR;  // (XR / 8) row blocks x 8 channel groups
  const int nI = 3 * nXb + CW_KS;
  const int ksx = CW_KS % W, dlm = (CW_KS / W) % g.H;
  bool it_on[MAXI];
  int it_rel[MAXI], it_dx[MAXI], it_fg[MAXI], it_dst[MAXI], it_x[MAXI];
  const bool isA0 = tid < CW_KS;
  int yA = 0;
#pragma unroll
  for (int j = 0; j < MAXI; ++j) {
    const int id = tid + 256 * j;
    it_on[j] = id < nI;
    // (consecutive lanes take consecutive 8-row blocks of one channel group: their 16-byte LDS
    // writes then fall into different banks; with the channel group in the low lane bits they
    // would all hit the same ones)
    if (j == 0 && isA0) {
      const int rb = id & (CW_KS / 8 - 1);
      it_fg[j] = id / (CW_KS / 8);
      it_rel[j] = rb * 8;
      it_dx[j] = 0;
      it_dst[j] = it_fg[j] * 8 * CW_PA + rb * 8;
      yA = (int)(((k_begin + it_rel[j]) / W) % g.H);
    } else {
      const int nrb = XR / 8;
      const int idx = it_on[j] ? id - CW_KS : 0;
      const int v = idx / nXb, r = idx - v * nXb;
      const int rb = r % nrb;
      it_fg[j] = r / nrb;
      it_rel[j] = -W + rb * 8;
      it_dx[j] = v - 1;
      it_dst[j] = (v * 64 + it_fg[j] * 8) * PX + rb * 8;
    }
    it_x[j] = (int)((k_begin + W + it_rel[j]) % W);
  }
  auto advance_items = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < MAXI; ++j) {
      int x = it_x[j] + ksx;
      const int carry = x >= W ? 1 : 0;
      it_x[j] = x - (carry ? W : 0);
      if (j == 0) {
        const int y = yA + dlm + carry;
        yA = y >= g.H ? y - g.H : y;
      }
    }
  };
  u16x8 reg[MAXI][8];
  auto load_items = [&](int64_t k0) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < MAXI; ++j) {
      if (!it_on[j]) continue;
      const int64_t qb = k0 + it_rel[j];
      if (j == 0 && isA0) {
        const uint16_t* src = g.A + (size_t)qb * g.lda + a0 + it_fg[j] * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) reg[j][i] = *reinterpret_cast<const u16x8*>(src + (size_t)i * g.lda);
      } else {
        const bool inside = qb >= 0 && qb < g.rows;
        const uint16_t* src = g.B + ((int64_t)qb + it_dx[j]) * g.ldb + b0 + it_fg[j] * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int xi = it_x[j] + i + it_dx[j];
          // (branch-free: a row that falls off the image line is read from a valid address here and
          // zeroed when it is written to LDS)
          const bool ok = inside && xi >= 0 && xi < W;
          reg[j][i] = *reinterpret_cast<const u16x8*>(ok ? src + (int64_t)i * g.ldb : g.B);
        }
      }
    }
  };
  auto store_items = [&](int64_t k0) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < MAXI; ++j) {
      if (!it_on[j]) continue;
      if (j == 0 && isA0) {
        // copies for dy = -1 / +1: rows of the first / last image line zeroed
        const uint16_t m_top = yA == 0 ? 0 : 0xffff, m_bot = yA == g.H - 1 ? 0 : 0xffff;
#pragma unroll
        for (int f = 0; f < 8; ++f) {
          u16x8 o, ot, ob;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            o[i] = reg[j][i][f];
            ot[i] = o[i] & m_top;
            ob[i] = o[i] & m_bot;
          }
          uint16_t* d = sA + it_dst[j] + f * CW_PA;
          *reinterpret_cast<u16x8*>(d) = ot;
          *reinterpret_cast<u16x8*>(d + 64 * CW_PA) = o;
          *reinterpret_cast<u16x8*>(d + 2 * 64 * CW_PA) = ob;
        }
      } else {
        const int64_t qb = k0 + it_rel[j];
        const bool inside = qb >= 0 && qb < g.rows;
        uint16_t m[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int xi = it_x[j] + i + it_dx[j];
          m[i] = (inside && xi >= 0 && xi < W) ? 0xffff : 0;
        }
#pragma unroll
        for (int f = 0; f < 8; ++f) {
          u16x8 o;
#pragma unroll
          for (int i = 0; i < 8; ++i) o[i] = reg[j][i][f] & m[i];
          *reinterpret_cast<u16x8*>(sX + it_dst[j] + f * PX) = o;
        }
      }
    }
  };

  f32x16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[t][q] = 0.f;

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  const bool sums = blockIdx.y == 0 && g.want_sums;
  constexpr bool tsums = TS;
  float sum_b = 0.f, sum_t[9], sum_1[9], sum_c[9];  // tau-, un- and c_j-weighted tap sums
#pragma unroll
  for (int t = 0; t < 9; ++t) sum_t[t] = sum_1[t] = sum_c[t] = 0.f;
  // sums: thread -> (channel tid / 4, quarter tid % 4 of the k-step's rows, in 8-row blocks); a block
  // lies in one image line: only its first row can have x = 0, only its last x = W - 1
  int sx[CW_KS / 32];
#pragma unroll
  for (int b = 0; b < CW_KS / 32; ++b) sx[b] = (int)((k_begin + (tid & 3) * (CW_KS / 4) + b * 8) % W);
  int jst = (int)(k_begin / g.R);
  int64_t stage_end = (int64_t)(jst + 1) * g.R;
  load_items(k_begin);
  for (int64_t k0 = k_begin; k0 < k_end; k0 += CW_KS) {
    store_items(k0);
    __syncthreads();
    if (sums) {
      const int co = tid >> 2, qt = tid & 3;
      if (k0 >= stage_end) {
        ++jst;
        stage_end += g.R;
      }
      const int j = jst;
      float tau = 0.f, cj = 0.f;
#pragma unroll
      for (int q = 0; q < kMaxStages; ++q) {
        tau = (q == j) ? g.taus[q] : tau;
        cj = (q == j) ? g.cs[q] : cj;
      }
      // (all reads first: the loader registers are free at this point)
      u16x8 sv[CW_KS / 32][3];
#pragma unroll
      for (int b = 0; b < CW_KS / 32; ++b)
#pragma unroll
        for (int dyv = 0; dyv < 3; ++dyv)
          sv[b][dyv] = *reinterpret_cast<const u16x8*>(&sA[(dyv * 64 + co) * CW_PA + qt * (CW_KS / 4) + b * 8]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int b = 0; b < CW_KS / 32; ++b) {
        const int xq0 = sx[b];
        sx[b] = xq0 + ksx >= W ? xq0 + ksx - W : xq0 + ksx;
#pragma unroll
        for (int dyv = 0; dyv < 3; ++dyv) {
          const u16x8 v = sv[b][dyv];
          float inner = 0.f;
#pragma unroll
          for (int e = 1; e < 7; ++e) inner += Low<T>::to_f32(v[e]);
          const float f0 = Low<T>::to_f32(v[0]), f7 = Low<T>::to_f32(v[7]);
          const float full = inner + f0 + f7;
          const float left = inner + f7 + (xq0 == 0 ? 0.f : f0);       // dx = -1
          const float right = inner + f0 + (xq0 == W - 8 ? 0.f : f7);  // dx = +1
          sum_t[dyv * 3 + 0] = fmaf(tau, left, sum_t[dyv * 3 + 0]);
          sum_t[dyv * 3 + 1] = fmaf(tau, full, sum_t[dyv * 3 + 1]);
          sum_t[dyv * 3 + 2] = fmaf(tau, right, sum_t[dyv * 3 + 2]);
          if (tsums) {
            sum_1[dyv * 3 + 0] += left;
            sum_1[dyv * 3 + 1] += full;
            sum_1[dyv * 3 + 2] += right;
            sum_c[dyv * 3 + 0] = fmaf(cj, left, sum_c[dyv * 3 + 0]);
            sum_c[dyv * 3 + 1] = fmaf(cj, full, sum_c[dyv * 3 + 1]);
            sum_c[dyv * 3 + 2] = fmaf(cj, right, sum_c[dyv * 3 + 2]);
          }
          if (dyv == 1) sum_b += full;
        }
      }
    }
    // the next k-step's rows are fetched into registers while this one is multiplied
    advance_items();
    if (k0 + CW_KS < k_end) load_items(k0 + CW_KS);
    // (kk, dy) steps of 3 MFMAs; the 4 operand fragments of step i + 2 are read from LDS before the
    // MFMAs of step i are issued (one wavefront per SIMD: nothing else hides the LDS latency)
    {
      constexpr int NST = (CW_KS / 16) * 3;
      auto load_frags = [&](int st, u16x8& fa, u16x8(&fb)[3]) __attribute__((always_inline)) {
        const int kk = st / 3, dyv = st % 3;
        fa = *reinterpret_cast<const u16x8*>(&sA[(dyv * 64 + wm * 32 + frow) * CW_PA + kk * 16 + fk]);
#pragma unroll
        for (int dxv = 0; dxv < 3; ++dxv)
          fb[dxv] = *reinterpret_cast<const u16x8*>(&sX[(dxv * 64 + wn * 32 + frow) * PX + dyv * W + kk * 16 + fk]);
      };
      u16x8 fa[3], fb[3][3];
      load_frags(0, fa[0], fb[0]);
      load_frags(1, fa[1], fb[1]);
#pragma unroll
      for (int st = 0; st < NST; ++st) {
        if (st + 2 < NST) load_frags(st + 2, fa[(st + 2) % 3], fb[(st + 2) % 3]);
        __builtin_amdgcn_sched_barrier(0);
        const int dyv = st % 3;
#pragma unroll
        for (int dxv = 0; dxv < 3; ++dxv)
          acc[dyv * 3 + dxv] = Low<T>::mfma32(fa[st % 3], fb[st % 3][dxv], acc[dyv * 3 + dxv]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
  }

  const float scale = g.h / g.ctl->S_step;
  float* slotf = g.part + ((size_t)(blockIdx.z * gridDim.x + blockIdx.x) * gridDim.y + blockIdx.y) * CW_SLOT;
  if (sums) {
    sum_b += __shfl_xor(sum_b, 1);
    sum_b += __shfl_xor(sum_b, 2);
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      sum_t[t] += __shfl_xor(sum_t[t], 1);
      sum_t[t] += __shfl_xor(sum_t[t], 2);
    }
    const int na = a0 + (tid >> 2);
    if ((tid & 3) == 0) {
      float4* tail = reinterpret_cast<float4*>(slotf + 9 * 4096 + (tid >> 2) * 16);
      float4 v0 = tail[0], v1 = tail[1], v2 = tail[2];
      v0.x = fmaf(scale, sum_b, v0.x);
      v0.y = fmaf(scale, sum_t[0], v0.y); v0.z = fmaf(scale, sum_t[1], v0.z); v0.w = fmaf(scale, sum_t[2], v0.w);
      v1.x = fmaf(scale, sum_t[3], v1.x); v1.y = fmaf(scale, sum_t[4], v1.y);
      v1.z = fmaf(scale, sum_t[5], v1.z); v1.w = fmaf(scale, sum_t[6], v1.w);
      v2.x = fmaf(scale, sum_t[7], v2.x); v2.y = fmaf(scale, sum_t[8], v2.y);
      tail[0] = v0; tail[1] = v1; tail[2] = v2;
    }
    if (tsums) {
      // this thread's quarter of its channel's rows: contract the tap sums with the time weights
      float p0 = 0.f, p1 = 0.f;
      if (na < g.Na) {
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          const float wv = g.wt[t * g.ldwt + na];
          p0 = fmaf(wv, sum_1[t] - sum_c[t], p0);
          p1 = fmaf(wv, sum_c[t], p1);
        }
      }
      block_sum2(scale * p0, scale * p1, g.tpart + 2 * (((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x));
    }
  }
  // plain read-modify-write: the slot belongs to this workgroup for the whole backward pass.  Its
  // layout follows the accumulator registers: float4 number ((tap * 4 + q / 4) * 256 + thread) holds
  // rows (co) wm * 32 + 8 (q / 4) + 4 (lane / 32) + 0..3 of column (ci) wn * 32 + lane % 32.  The old
  // values of three taps are fetched together (one memory latency per group, not one per value).
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

// dW[co][ci][tap], db[co] and dwt[co][tap] += sum over K-chunks of the private accumulators (end of the
// backward pass).  gb / gwt null: no bias / no time channel; element (co, tap) of dwt at co * wt_stride + tap.
__global__ void conv_wgrad_reduce(float* __restrict__ G, int ldg, const float* __restrict__ part, int splits,
                                  int tiles_a, int tiles_b, int Na, int Nb, float* __restrict__ gb,
                                  float* __restrict__ gwt, int wt_stride, const Ctl* ctl) {
  if (ctl->poison) return;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nW = (int64_t)Na * Nb * 9;
  if (i >= nW + (int64_t)Na * 10) return;
  if (i >= nW) {
    const int na = (int)((i - nW) / 10), e = (int)((i - nW) % 10);
    float* dst = e == 0 ? (gb ? gb + na : nullptr) : (gwt ? gwt + (size_t)na * wt_stride + (e - 1) : nullptr);
    if (!dst) return;
    const size_t off = (size_t)(na >> 6) * tiles_b * CW_SLOT + 9 * 4096 + (na & 63) * 16 + e;
    float acc = 0.f;
    for (int c = 0; c < splits; ++c) acc += part[(size_t)c * tiles_a * tiles_b * CW_SLOT + off];
    *dst += acc;
    return;
  }
  const int nb = (int)(i % Nb), t = (int)((i / Nb) % 9), na = (int)(i / ((int64_t)Nb * 9));
  // (position of element (tap, co, ci) in a workgroup's copy: see the epilogue of conv_wgrad)
  const int r = na & 31, c = nb & 31;
  const int thread = (((na >> 5) & 1) * 2 + ((nb >> 5) & 1)) * 64 + ((r >> 2) & 1) * 32 + c;
  const size_t in_tile = ((size_t)(t * 4 + (r >> 3)) * 256 + thread) * 4 + (r & 3);
  const size_t tile = (size_t)(na >> 6) * tiles_b + (nb >> 6);
  float acc = 0.f;
  for (int c2 = 0; c2 < splits; ++c2) acc += part[((size_t)c2 * tiles_a * tiles_b + tile) * CW_SLOT + in_tile];
  G[(size_t)na * ldg + (size_t)nb * 9 + t] += acc;
}

// The MFMAs of one k-step of 64 on a wavefront's 64 x 64 output block: operand fragments of k-block
// kk + 1 are read from LDS before the MFMAs of k-block kk are issued (left to itself the compiler
// puts a full wait between every fragment read and its MFMA).  pa / pb: this lane's first fragment
// of the two operand tiles (row (lane % 32), k offset 8 (lane / 32)).
template <class T, int PITCH>
__device__ __forceinline__ void mma_k64(const uint16_t* pa, const uint16_t* pb, f32x16 (&acc)[2][2]) {
  u16x8 fa[2][2], fb[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a) fa[0][a] = *reinterpret_cast<const u16x8*>(pa + a * 32 * PITCH);
#pragma unroll
  for (int b = 0; b < 2; ++b) fb[0][b] = *reinterpret_cast<const u16x8*>(pb + b * 32 * PITCH);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    if (kk + 1 < 4) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
        fa[(kk + 1) & 1][a] = *reinterpret_cast<const u16x8*>(pa + a * 32 * PITCH + (kk + 1) * 16);
#pragma unroll
      for (int b = 0; b < 2; ++b)
        fb[(kk + 1) & 1][b] = *reinterpret_cast<const u16x8*>(pb + b * 32 * PITCH + (kk + 1) * 16);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) acc[a][b] = Low<T>::mfma32(fa[kk & 1][a], fb[kk & 1][b], acc[a][b]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ------------------------------------------------------------------------------------
// Parameter gradients of one adjoint step for dense networks whose cotangents and layer
// inputs were stored FEATURE-GROUP-MAJOR by the row-tile-persistent adjoint kernel: element
// (feature f, k) at ((f / 4) * ldk + k) * 4 + f % 4, k = stage * Rp + row, Rp = rows padded to
// 64, padding zero.  For a feature group k runs contiguously, so the tiles of both operands of
// dW_l = delta_l^T act_{l-1}  are read with coalesced 16-byte loads (2 k x 4 features) and
// regrouped into k-contiguous LDS rows on the way in.  One launch covers every layer:
//   one workgroup per (K-chunk, 128 x 128 output tile); chunk c accumulates into its own copy c of
//   the gradient vector (no atomics, fixed summation order); the copies are summed once at the end
//   of the backward pass;
//   the workgroups of the first tile column also sum their cotangent tile over k (from LDS) for
//   db_l and the time-column gradient.
// All contributions are scaled by h / S_step (paper Sec. 3, update of g).
struct WgradLayer {
  const uint16_t* DT;   // [NaPad / 4][ldk][4] cotangent of the layer's output
  const uint16_t* AT;   // [NbPad / 4][ldk][4] the layer's input
  float* G;             // dW_l block of partial-gradient copy 0, row pitch ldg
  float* gb;            // db_l
  float* gwt;           // time-column gradient (element stride ldg) or null
  int ldg;
  int Na, Nb;           // valid extents
  int NaPad, NbPad;     // rows that exist in DT / AT
  int tiles_a, tiles_b; // 128-tiles
  int tile0;            // index of this layer's first tile among all layers' tiles
};

struct WgradArgs {
  WgradLayer layer[8];
  int L;
  int ntiles;           // output tiles of all layers
  int64_t P;            // parameters: distance between the per-K-chunk copies of the gradient
  int ksplits;          // K-chunks per output tile
  int kchunk;           // k extent of a chunk (multiple of 64)
  int64_t ldk;          // s * Rp
  int64_t Rp;
  int s;
  float taus[kMaxStages];
  float h;
  const float* scale_hist;  // [N + 1]: scale_hist[step] = accepted scale of the step, 0 = not accepted
  int step;
  // several steps per launch (wgrad_feature_major_steps): steps step, step - 1, ..., step - nsteps + 1;
  // the buffers of step i are set i % nsets, set_stride elements apart; row i of steptab = (h_i, tau_i1..tau_is)
  int nsteps, nsets;
  int64_t set_stride;
  const float* steptab;
};
constexpr int kMaxWgradSteps = 64;  // steps per launch of wgrad_feature_major_steps

// (register cap: for narrow networks this kernel shares the SIMDs with the 4-wave adjoint kernel,
// which leaves it a little over 200 of the 512 registers of a lane)
template <class T>
__global__ __launch_bounds__(256, 2) __attribute__((amdgpu_num_vgpr(104))) void wgrad_feature_major(WgradArgs g) {
  const float S = g.scale_hist[g.step];
  if (S == 0.f) return;  // the step's cotangent chain was rejected (or never ran)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float scale = g.h / S;
  // Workgroups go to the 8 XCDs round-robin by block index.  Re-linearise so that an XCD owns a
  // contiguous range of (K-chunk, tile) pairs, K-chunk-major: the tiles that run together on an
  // XCD then read the same k range of the operands and share it through that XCD's L2.
  const int per_xcd = (int)gridDim.x >> 3;
  const int gp = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (gp >= g.ntiles * g.ksplits) return;
  const int split = gp / g.ntiles;
  const int t = gp - split * g.ntiles;

  // ---- 128 x 128 tile of dW_l over one K-chunk
  WgradLayer y = g.layer[0];
#pragma unroll
  for (int q = 1; q < 8; ++q)
    if (q < g.L && t >= g.layer[q].tile0) y = g.layer[q];
  const int r = t - y.tile0;
  const int ta = r % y.tiles_a, tb = r / y.tiles_a;
  const int a0 = ta * 128, b0 = tb * 128;
  const int64_t k_begin = (int64_t)split * g.kchunk;
  int64_t k_end = k_begin + g.kchunk;
  if (k_end > g.ldk) k_end = g.ldk;
  if (k_begin >= k_end) return;

  __shared__ __attribute__((aligned(16))) uint16_t sA[128 * LDS_PITCH];
  __shared__ __attribute__((aligned(16))) uint16_t sB[128 * LDS_PITCH];
  const int wm = wave >> 1, wn = wave & 1;
  // tile of an operand: 32 feature groups x 64 k.  A thread owns one feature group and 8
  // consecutive k: 64 contiguous bytes in memory (8 k x 4 features), which it regroups in
  // registers into 4 rows of 8 k (one per feature) for k-contiguous LDS rows.
  // The loads run WG_STAGES k-steps ahead of the MFMAs (a workgroup streams its operands once,
  // from the other XCDs' writes via memory: the latency is long and there is no reuse to hide it).
  constexpr int WG_STAGES = 2;
  const int fg = tid >> 3, oct = tid & 7;
  u16x8 ra[WG_STAGES][4], rb[WG_STAGES][4];
  // feature groups beyond the padded extent read group 0 instead and are masked in the epilogue
  const uint16_t* pa0 = y.DT + ((size_t)((a0 + fg * 4 < y.NaPad) ? a0 / 4 + fg : 0) * g.ldk + oct * 2) * 4;
  const uint16_t* pb0 = y.AT + ((size_t)((b0 + fg * 4 < y.NbPad) ? b0 / 4 + fg : 0) * g.ldk + oct * 2) * 4;
  const int nsteps = (int)((k_end - k_begin) / BK);
  auto load_tiles = [&](u16x8 (&qa)[4], u16x8 (&qb)[4], int step) {
    const int64_t k0 = k_begin + (int64_t)(step < nsteps ? step : nsteps - 1) * BK;  // clamped: branch-free
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qa[i] = *reinterpret_cast<const u16x8*>(pa0 + k0 * 4 + i * 64);  // k = 16 i + 2 oct, + 1
      qb[i] = *reinterpret_cast<const u16x8*>(pb0 + k0 * 4 + i * 64);
    }
  };
  // r[i] = (k = 2i: f0 f1 f2 f3, k = 2i + 1: f0 f1 f2 f3); row of feature f = 8 consecutive k.
  // One byte permute per output word: halves of word d (k even) and word d + 2 (k odd).
  auto regroup_store = [&](uint16_t* sX, const u16x8 (&r)[4]) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = __builtin_bit_cast(u32x4, r[i]);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      const int d = f >> 1;
      const uint32_t sel = (f & 1) ? 0x07060302u : 0x05040100u;
      u32x4 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = __builtin_amdgcn_perm(w[i][d + 2], w[i][d], sel);
      *reinterpret_cast<u32x4*>(&sX[(fg * 4 + f) * LDS_PITCH + oct * 8]) = o;
    }
  };
  auto store_tiles = [&](const u16x8 (&qa)[4], const u16x8 (&qb)[4]) {
    regroup_store(sA, qa);
    regroup_store(sB, qb);
  };
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.f;

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  float sum_b = 0.f, sum_t = 0.f;
#pragma unroll
  for (int u = 0; u < WG_STAGES; ++u) load_tiles(ra[u], rb[u], u);
  // One k-step, free of branches (a branch inside the software pipeline makes every wait for a
  // load a wait for all of them).  SUMS: also accumulate the sums of the cotangent tile over k for
  // db_l and the time-column gradient: thread -> (feature tid / 2, half tid % 2 of the 64 k);
  // a k-step lies within one stage.
  auto k_step = [&](auto sums, u16x8 (&qa)[4], u16x8 (&qb)[4], int step) {
    // (scheduling fences: the loads of step + WG_STAGES must issue here, a full WG_STAGES k-steps
    // ahead of their use, and the next step's regrouping must not drift up into this one)
    __builtin_amdgcn_sched_barrier(0);
    store_tiles(qa, qb);
    __syncthreads();
    load_tiles(qa, qb, step + WG_STAGES);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(sums)::value) {
      const int64_t k0 = k_begin + (int64_t)step * BK;
      const int j = (int)(k0 / g.Rp);
      float tau = 0.f;
#pragma unroll
      for (int q = 0; q < kMaxStages; ++q) tau = (q == j) ? g.taus[q] : tau;
      float part = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const u16x8 v = *reinterpret_cast<const u16x8*>(&sA[(tid >> 1) * LDS_PITCH + (tid & 1) * 32 + c * 8]);
#pragma unroll
        for (int e = 0; e < 8; ++e) part += Low<T>::to_f32(v[e]);
      }
      sum_b += part;
      sum_t = fmaf(tau, part, sum_t);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      u16x8 fa[2], fb[2];
#pragma unroll
      for (int a = 0; a < 2; ++a)
        fa[a] = *reinterpret_cast<const u16x8*>(&sA[(wm * 64 + a * 32 + frow) * LDS_PITCH + kk * 16 + fk]);
#pragma unroll
      for (int b = 0; b < 2; ++b)
        fb[b] = *reinterpret_cast<const u16x8*>(&sB[(wn * 64 + b * 32 + frow) * LDS_PITCH + kk * 16 + fk]);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = Low<T>::mfma32(fa[a], fb[b], acc[a][b]);
    }
    __syncthreads();
  };
  auto k_loop = [&](auto sums) {
    static_assert(WG_STAGES == 2, "the loop below rotates two register stages");
    int step = 0;
    for (; step + 2 <= nsteps; step += 2) {
      k_step(sums, ra[0], rb[0], step);
      k_step(sums, ra[1], rb[1], step + 1);
    }
    if (step < nsteps) k_step(sums, ra[0], rb[0], step);
  };
  if (tb == 0)
    k_loop(std::true_type{});
  else
    k_loop(std::false_type{});
  if (tb == 0) {
    sum_b += __shfl_xor(sum_b, 1);
    sum_t += __shfl_xor(sum_t, 1);
    const int na = a0 + (tid >> 1);
    if ((tid & 1) == 0 && na < y.Na) {
      float* db = y.gb + (size_t)split * g.P + na;
      *db = fmaf(scale, sum_b, *db);
      if (y.gwt) {
        float* dt = y.gwt + (size_t)split * g.P + (size_t)na * y.ldg;
        *dt = fmaf(scale, sum_t, *dt);
      }
    }
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int nb = b0 + wn * 64 + b * 32 + (lane & 31);
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int na = a0 + wm * 64 + a * 32 + 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3);
        // every (K-chunk, tile) owns its slot of the partial-gradient copies: plain read-modify-write
        if (na < y.Na && nb < y.Nb) {
          float* dst = y.G + (size_t)split * g.P + (size_t)na * y.ldg + nb;
          *dst = fmaf(scale, acc[a][b][q], *dst);
        }
      }
    }
  }
}


// The same contraction over SEVERAL steps in one launch (steps step, step - 1, ... of which the
// accepted ones at the head of the range are taken: see s_accepted).  A workgroup keeps its (K-chunk, tile)
// and walks through the steps' buffer sets as one continuous sequence of k-steps, so the load
// pipeline never drains at a step boundary; the per-step factor h_i / S_i is applied when a
// step's partial sum is folded into the running total.  One launch then costs one epilogue and
// one pipeline fill per workgroup instead of one per step.
template <class T>
__global__ __launch_bounds__(256, 2) void wgrad_feature_major_steps(WgradArgs g) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per_xcd = (int)gridDim.x >> 3;
  const int gp = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (gp >= g.ntiles * g.ksplits) return;
  const int split = gp / g.ntiles;
  const int t = gp - split * g.ntiles;
  WgradLayer y = g.layer[0];
#pragma unroll
  for (int q = 1; q < 8; ++q)
    if (q < g.L && t >= g.layer[q].tile0) y = g.layer[q];
  const int r = t - y.tile0;
  const int ta = r % y.tiles_a, tb = r / y.tiles_a;
  const int a0 = ta * 128, b0 = tb * 128;
  const int64_t k_begin = (int64_t)split * g.kchunk;
  int64_t k_end = k_begin + g.kchunk;
  if (k_end > g.ldk) k_end = g.ldk;
  if (k_begin >= k_end) return;

  __shared__ __attribute__((aligned(16))) uint16_t sA[128 * LDS_PITCH];
  __shared__ __attribute__((aligned(16))) uint16_t sB[128 * LDS_PITCH];
  __shared__ float s_scale[kMaxWgradSteps];
  __shared__ float s_tau[kMaxWgradSteps][kMaxStages];
  // Steps whose cotangent chain was rejected (or that never ran because an earlier one was) have no
  // recorded scale: the launch covers the accepted steps at the head of its range only.  The host
  // redoes the rest, from the rejected step on, with launches of their own.
  __shared__ int s_accepted;
  if (tid == 0) {
    int n = 0;
    while (n < g.nsteps && g.scale_hist[g.step - n] != 0.f) ++n;
    s_accepted = n;
  }
  __syncthreads();
  g.nsteps = s_accepted;
  if (g.nsteps == 0) return;
  // s_scale[i] = c_i / c_{i+1} with c_i = h / S of the launch's i-th step (the last: c_i itself):
  // multiplying the running sums by it when step i is complete leaves, at the end,
  // sum_i c_i * (partial sum of step i) without a second set of accumulators
  for (int i = tid; i < g.nsteps; i += 256) {
    const int step = g.step - i;
    const float* row = g.steptab + (size_t)step * (1 + g.s);
    const float c = row[0] / g.scale_hist[step];
    float cn = 1.f;
    if (i + 1 < g.nsteps) cn = g.steptab[(size_t)(step - 1) * (1 + g.s)] / g.scale_hist[step - 1];
    s_scale[i] = c / cn;
    for (int j = 0; j < kMaxStages; ++j) s_tau[i][j] = j < g.s ? row[1 + j] : 0.f;
  }
  __syncthreads();

  const int wm = wave >> 1, wn = wave & 1;
  constexpr int WG_STAGES = 2;
  const int fg = tid >> 3, oct = tid & 7;
  u16x8 ra[WG_STAGES][4], rb[WG_STAGES][4];
  const uint16_t* pa0 = y.DT + ((size_t)((a0 + fg * 4 < y.NaPad) ? a0 / 4 + fg : 0) * g.ldk + oct * 2) * 4;
  const uint16_t* pb0 = y.AT + ((size_t)((b0 + fg * 4 < y.NbPad) ? b0 / 4 + fg : 0) * g.ldk + oct * 2) * 4;
  const int nk = (int)((k_end - k_begin) / BK);  // k-steps per step
  const int total = nk * g.nsteps;
  // position of the next tile to load: (step number it within the launch, k-step kk, buffer set)
  int ld_it = 0, ld_kk = 0, ld_set = g.step % g.nsets;
  auto load_tiles = [&](u16x8 (&qa)[4], u16x8 (&qb)[4]) __attribute__((always_inline)) {
    const int64_t off = (int64_t)ld_set * g.set_stride + (k_begin + (int64_t)ld_kk * BK) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qa[i] = *reinterpret_cast<const u16x8*>(pa0 + off + i * 64);
      qb[i] = *reinterpret_cast<const u16x8*>(pb0 + off + i * 64);
    }
    // advance, staying on the last tile once it is reached (the extra loads of the pipeline tail)
    const bool last = (ld_it == g.nsteps - 1) && (ld_kk == nk - 1);
    const bool wrap = (ld_kk == nk - 1);
    ld_kk = last ? ld_kk : (wrap ? 0 : ld_kk + 1);
    ld_it = (last || !wrap) ? ld_it : ld_it + 1;
    ld_set = (last || !wrap) ? ld_set : (ld_set == 0 ? g.nsets - 1 : ld_set - 1);
  };
  auto regroup_store = [&](uint16_t* sX, const u16x8 (&rr)[4]) __attribute__((always_inline)) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = __builtin_bit_cast(u32x4, rr[i]);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      const int d = f >> 1;
      const uint32_t sel = (f & 1) ? 0x07060302u : 0x05040100u;
      u32x4 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = __builtin_amdgcn_perm(w[i][d + 2], w[i][d], sel);
      *reinterpret_cast<u32x4*>(&sX[(fg * 4 + f) * LDS_PITCH + oct * 8]) = o;
    }
  };
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.f;

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  float sum_b = 0.f, sum_t = 0.f;
#pragma unroll
  for (int u = 0; u < WG_STAGES; ++u) load_tiles(ra[u], rb[u]);
  int it = 0, kk = 0;  // position of the tile being consumed
  const int j_first = (int)(k_begin / g.Rp);
  int jst = j_first;
  int64_t stage_end = (int64_t)(j_first + 1) * g.Rp;
  auto k_step = [&](auto sums, u16x8 (&qa)[4], u16x8 (&qb)[4]) __attribute__((always_inline)) {
    __builtin_amdgcn_sched_barrier(0);
    regroup_store(sA, qa);
    regroup_store(sB, qb);
    __syncthreads();
    load_tiles(qa, qb);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(sums)::value) {
      if (kk == 0) {  // (a new step starts over at the chunk's first stage; no division per k-step)
        jst = j_first;
        stage_end = (int64_t)(j_first + 1) * g.Rp;
      }
      if (k_begin + (int64_t)kk * BK >= stage_end) {
        ++jst;
        stage_end += g.Rp;
      }
      const float tau = s_tau[it][jst];
      float part = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const u16x8 v = *reinterpret_cast<const u16x8*>(&sA[(tid >> 1) * LDS_PITCH + (tid & 1) * 32 + c * 8]);
#pragma unroll
        for (int e = 0; e < 8; ++e) part += Low<T>::to_f32(v[e]);
      }
      sum_b += part;
      sum_t = fmaf(tau, part, sum_t);
    }
    static_assert(BK == 64, "mma_k64 covers a k-step of 64");
    mma_k64<T, LDS_PITCH>(&sA[(wm * 64 + frow) * LDS_PITCH + fk], &sB[(wn * 64 + frow) * LDS_PITCH + fk], acc);
    if (kk == nk - 1) {
      // the step's partial sums are complete: rescale the running sums for the next step
      const float sc = s_scale[it];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int q = 0; q < 16; ++q) acc[a][b][q] *= sc;
      sum_b *= sc;
      sum_t *= sc;
      kk = 0;
      ++it;
    } else {
      ++kk;
    }
    __syncthreads();
  };
  auto k_loop = [&](auto sums) __attribute__((always_inline)) {
    int n = 0;
    for (; n + 2 <= total; n += 2) {
      k_step(sums, ra[0], rb[0]);
      k_step(sums, ra[1], rb[1]);
    }
    if (n < total) k_step(sums, ra[0], rb[0]);
  };
  if (tb == 0)
    k_loop(std::true_type{});
  else
    k_loop(std::false_type{});

  if (tb == 0) {
    sum_b += __shfl_xor(sum_b, 1);
    sum_t += __shfl_xor(sum_t, 1);
    const int na = a0 + (tid >> 1);
    if ((tid & 1) == 0 && na < y.Na) {
      y.gb[(size_t)split * g.P + na] += sum_b;
      if (y.gwt) y.gwt[(size_t)split * g.P + (size_t)na * y.ldg] += sum_t;
    }
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int nb = b0 + wn * 64 + b * 32 + (lane & 31);
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int na = a0 + wm * 64 + a * 32 + 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3);
        if (na < y.Na && nb < y.Nb) y.G[(size_t)split * g.P + (size_t)na * y.ldg + nb] += acc[a][b][q];
      }
    }
  }
}

// g[i] += sum_c part[c][i]   (end of the backward pass: fold the per-K-chunk copies)
__global__ void reduce_partial_gradients(float* __restrict__ g, const float* __restrict__ part, int64_t P, int copies,
                                         const Ctl* ctl) {
  if (ctl->poison) return;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= P) return;
  float acc = 0.f;
  for (int c = 0; c < copies; ++c) acc += part[(size_t)c * P + i];
  g[i] += acc;
}

}  // namespace rampde
