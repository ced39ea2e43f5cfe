// 3x3 zero-padded convolution (and its transpose: the same kernel with the flipped, transposed
// weights) on channels-last rows, for at most 64 channels: the velocity evaluations, their
// recomputation and the input-cotangent products of the convolutional velocity (paper Alg. 1, the
// low-precision evaluation of Phi; eq. (vjp)) as one persistent kernel per call.
//
// A workgroup keeps the whole weight tensor of the layer (9 taps x 64 x 64, low precision) in LDS
// for as long as it lives and walks over tiles of 256 pixels (whole image lines).  Per tile the
// input lines with a halo of one line above and below and one zero column left and right are
// staged in LDS once; every tap is then the same tile read at a shifted pixel address, and a
// wavefront computes 64 pixels x 64 output channels with v_mfma_f32_32x32x16 (weights as the first
// operand, so a lane ends with 4 consecutive output channels of a pixel: 8-byte stores and loads
// in the epilogue).  The next tile's input is fetched into registers while the current one is
// being multiplied.  Epilogue as in gemm_nt: bias, time-channel term (tabulated by border class),
// tanh or the tanh' factor from the stored activation, rounding, overflow detector.
//
// Shapes: padded channels = 64, W a power of two in [8, 64], H * W a multiple of 256 (a tile never
// spans two images); anything else goes to gemm_nt<CONV>.
#pragma once
#include "fused.hpp"
#include "gemm.hpp"

namespace rampde {

constexpr int CT_PITCH = 72;      // elements per LDS row of 64 channels (144 B)
constexpr int CT_TILE = 256;      // pixels per tile
constexpr int CT_MAXCHUNK = 12;   // 16-byte input chunks per thread and tile (W = 64)

inline bool conv_tile_applies(int Cpad, int N, int H, int Wd, int64_t M) {
  const bool pow2 = Wd >= 8 && Wd <= 64 && (Wd & (Wd - 1)) == 0;
  return Cpad == 64 && N == 64 && pow2 && ((int64_t)H * Wd) % CT_TILE == 0 && M % CT_TILE == 0;
}
inline size_t conv_tile_lds_bytes(int Wd) {
  const int lines = CT_TILE / Wd + 2;
  return (size_t)(9 * 64 * CT_PITCH + lines * (Wd + 2) * CT_PITCH) * 2 + (16 * 64 + 10 * 64) * 4;
}

// NWV wavefronts per workgroup (4 or 8): a wavefront owns 256 / NWV pixels of the tile x all 64 output channels.
template <class T, int NWV>
__global__ __launch_bounds__(64 * NWV) void conv3x3_tile(GemmNT g) {
  constexpr int NT = 64 * NWV;        // threads
  constexpr int NB = 8 / NWV;         // 32-pixel blocks per wavefront (2 or 1)
  if (g.ctl && g.ctl->poison) return;
  extern __shared__ __attribute__((aligned(16))) uint16_t ct_smem[];
  const int W = g.Wd, H = g.H;
  const int PR = CT_TILE / W;          // image lines per tile
  const int LW = W + 2;                // staged pixels per line
  const int wshift = 31 - __builtin_clz(W);
  uint16_t* sW = ct_smem;                              // [9][64 co][CT_PITCH]
  uint16_t* sIn = ct_smem + 9 * 64 * CT_PITCH;         // [PR + 2][W + 2][CT_PITCH]
  float* s_tt = reinterpret_cast<float*>(sIn + (PR + 2) * LW * CT_PITCH);  // [16][64]: bias + time term by border class
  float* s_wt = s_tt + 16 * 64;                                            // [9][64] time-channel weights, [64] bias
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ntiles = (int)(g.M / CT_TILE);

  // ---- input chunks of a tile: chunk id -> (staged line ly, pixel x, 8 channels c8)
  const int nchunk = (PR + 2) * W * 8;
  constexpr int MAXC = CT_MAXCHUNK * 256 / NT;
  u16x8 reg[MAXC];
  auto load_tile = [&](int t) __attribute__((always_inline)) {
    const int64_t row0 = (int64_t)t * CT_TILE;          // first pixel row of the tile
    const int y0 = (int)((row0 >> wshift) % H);         // its image line
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int id = tid + NT * i;
      u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (id < nchunk) {
        const int c8 = id & 7, px = id >> 3;
        const int x = px & (W - 1), ly = px >> wshift;  // ly = 0 is the line above the tile
        const int y = y0 + ly - 1;
        if (y >= 0 && y < H)
          v = *reinterpret_cast<const u16x8*>(g.A + (size_t)(row0 + (int64_t)(ly - 1) * W + x) * g.lda + c8 * 8);
      }
      reg[i] = v;
    }
  };
  auto store_tile = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int id = tid + NT * i;
      if (id < nchunk) {
        const int c8 = id & 7, px = id >> 3;
        const int x = px & (W - 1), ly = px >> wshift;
        *reinterpret_cast<u16x8*>(&sIn[(ly * LW + x + 1) * CT_PITCH + c8 * 8]) = reg[i];
      }
    }
  };

  // (the first tile's input is requested before the weights: both are in flight together)
  if ((int)blockIdx.x < ntiles) load_tile(blockIdx.x);

  // ---- once per workgroup: weights, zero halo columns, time-term table
  {
    // (all 18 loads of a thread are issued before the first is stored: one memory latency, not 18)
    constexpr int NWC = 9 * 64 * 8 / NT;
    u16x8 wr[NWC];
#pragma unroll
    for (int i = 0; i < NWC; ++i) {
      const int id = tid + NT * i;
      const int c8 = id & 7, co = (id >> 3) & 63, tap = id >> 9;
      wr[i] = *reinterpret_cast<const u16x8*>(g.W + (size_t)co * g.ldw + tap * 64 + c8 * 8);
    }
#pragma unroll
    for (int i = 0; i < NWC; ++i) {
      const int id = tid + NT * i;
      const int c8 = id & 7, co = (id >> 3) & 63, tap = id >> 9;
      *reinterpret_cast<u16x8*>(&sW[(tap * 64 + co) * CT_PITCH + c8 * 8]) = wr[i];
    }
  }
  for (int id = tid; id < (PR + 2) * 2 * 8; id += NT) {
    const int c8 = id & 7, side = (id >> 3) & 1, ly = id >> 4;
    const u16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    *reinterpret_cast<u16x8*>(&sIn[(ly * LW + (side ? W + 1 : 0)) * CT_PITCH + c8 * 8]) = z;
  }
  // (one global load per thread, then the table from LDS: a chain of dependent global loads per
  // table entry would cost more than the tile's multiplication)
  for (int i = tid; i < 10 * 64; i += NT) {
    float v = 0.f;
    if (i < 9 * 64) {
      if (g.wt) v = g.wt[(i >> 6) * g.N + (i & 63)];
    } else if (g.bias) {
      v = g.bias[i & 63];
    }
    s_wt[i] = v;
  }
  __syncthreads();
  for (int i = tid; i < 16 * 64; i += NT) {
    const int combo = i >> 6, n = i & 63;
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      const int dy = t / 3 - 1, dx = t % 3 - 1;
      const bool ok = (dy >= 0 || (combo & 8)) && (dy <= 0 || (combo & 4)) && (dx >= 0 || (combo & 2)) &&
                      (dx <= 0 || (combo & 1));
      sum += ok ? s_wt[t * 64 + n] * g.tau : 0.f;
    }
    s_tt[i] = s_wt[9 * 64 + n] + sum;
  }


  // this lane's two pixel columns (operand B) and weight rows (operand A)
  const int fk = (lane >> 5) * 8;
  int in_base[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int p = wave * (32 * NB) + nb * 32 + (lane & 31);
    const int x = p & (W - 1), ly = p >> wshift;        // line within the tile, 0-based
    in_base[nb] = ((ly + 1) * LW + x + 1) * CT_PITCH + fk;
  }
  const int w_base = (lane & 31) * CT_PITCH + fk;

  int t = blockIdx.x;
  bool bad = false;
  for (; t < ntiles; t += gridDim.x) {
    __syncthreads();  // the previous tile's fragments have been read (and the tables are written)
    store_tile();
    __syncthreads();
    if (t + (int)gridDim.x < ntiles) load_tile(t + gridDim.x);

    f32x16 acc[2][NB];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.f;
    // the stored activations for the tanh' factor of this lane's outputs: in flight during the
    // multiplication
    uint2 dv[NB][2][4];
    if (g.dact) {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int64_t m = (int64_t)t * CT_TILE + wave * (32 * NB) + b * 32 + (lane & 31);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
            dv[b][a][q4] =
                *reinterpret_cast<const uint2*>(g.dact + (size_t)m * g.ldd + a * 32 + 8 * q4 + 4 * (lane >> 5));
      }
    }
    // 36 k-blocks of 16 (9 taps x 64 channels); the fragments of block i + 1 are read from LDS
    // before the MFMAs of block i are issued (a workgroup is alone on its CU: nothing else hides
    // the LDS latency)
    auto load_frags = [&](int it, u16x8 (&fa)[2], u16x8 (&fb)[NB]) __attribute__((always_inline)) {
      const int tap = it >> 2, kk = it & 3;
      const int shift = ((tap / 3 - 1) * LW + (tap % 3 - 1)) * CT_PITCH;
#pragma unroll
      for (int a = 0; a < 2; ++a)
        fa[a] = *reinterpret_cast<const u16x8*>(&sW[(tap * 64 + a * 32) * CT_PITCH + w_base + kk * 16]);
#pragma unroll
      for (int b = 0; b < NB; ++b) fb[b] = *reinterpret_cast<const u16x8*>(&sIn[in_base[b] + shift + kk * 16]);
    };
    u16x8 fa[2][2], fb[2][NB];
    load_frags(0, fa[0], fb[0]);
#pragma unroll
    for (int it = 0; it < 36; ++it) {
      if (it + 1 < 36) load_frags(it + 1, fa[(it + 1) & 1], fb[(it + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);  // (keep the reads of block i + 1 ahead of the MFMAs of block i)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[a][b] = Low<T>::mfma32(fa[it & 1][a], fb[it & 1][b], acc[a][b]);
      __builtin_amdgcn_sched_barrier(0);
    }

    // ---- epilogue: accumulator row = output channel 8 (q / 4) + 4 (lane / 32) + q % 4 of block a,
    //      column = pixel lane % 32 of block b
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int p = wave * (32 * NB) + b * 32 + (lane & 31);
      const int64_t m = (int64_t)t * CT_TILE + p;
      int combo = 0;
      if (g.wt) {
        const int x = p & (W - 1);
        const int y = (int)((m >> wshift) % H);
        combo = ((y > 0) << 3) | ((y < H - 1) << 2) | ((x > 0) << 1) | (x < W - 1 ? 1 : 0);
      }
      float4 tv[2][4];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          tv[a][q4] = *reinterpret_cast<const float4*>(&s_tt[combo * 64 + a * 32 + 8 * q4 + 4 * (lane >> 5)]);
#pragma unroll
      for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int n = a * 32 + 8 * q4 + 4 * (lane >> 5);
          float v[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[a][b][q4 * 4 + r];
          v[0] += tv[a][q4].x; v[1] += tv[a][q4].y; v[2] += tv[a][q4].z; v[3] += tv[a][q4].w;
          if (g.act_tanh) {
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = tanh_fast(v[r]);
          }
          if (g.dact) {
            float av[4];
            unpack4<T>(dv[b][a][q4], av);
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = v[r] * (1.f - av[r] * av[r]);
          }
          const uint2 q = pack4<T>(v);
          bad = bad || any_nonfinite4<T>(q);
          *reinterpret_cast<uint2*>(g.C + (size_t)m * g.ldc + n) = q;
        }
      }
    }
  }
  if (g.detect) raise_if_any(bad, g.ctl);
}

}  // namespace rampde
