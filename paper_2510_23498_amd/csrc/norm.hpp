// Instance normalisation of the parabolic convolution block  f = -W^T N(relu(W y + b))
// (paper Sec. 6.3, eq. (NODE_STL10)) and its vector-Jacobian product.
//
// Activations are channels-last rows [B * HW][ld] of 16-bit values.  N acts per sample and channel
// over the HW pixels: n = (r - mean) * rstd, rstd = 1 / sqrt(var + eps), biased variance, no affine
// parameters.  Statistics and arithmetic are fp32, the result is rounded to low precision.  The
// cotangent of r given the cotangent dn of n:
//   dr = rstd * (dn - mean(dn) - n * mean(dn * n)),     du = dr * [r > 0]   (ReLU mask),
// with the stored (rounded) n and the forward pass's fp32 rstd.
//
// Both directions are three launches:
//   instnorm_partial   sums over pixel chunks: (sum x, sum x^2) forward, (sum dn, sum dn * n) backward,
//                      one slot per (chunk, sample, channel): no atomics, fixed summation order;
//   instnorm_finalize  folds the chunks: (mean, rstd) forward, (mean(dn), mean(dn * n)) backward;
//   instnorm_apply / instnorm_apply_vjp   the elementwise part, 8 channels (16 bytes) per thread.
#pragma once
#include <algorithm>
#include "common.hpp"

namespace rampde {

constexpr float kNormEps = 1e-5f;  // added to the variance (the paper does not state it: the usual default)

struct NormPartial {
  const uint16_t* X;     // forward: r; backward: dn
  const uint16_t* Nrm;   // backward: n; forward: unused
  int ld;                // row pitch of X and Nrm (elements)
  int Cpad;              // channels that exist in a row (multiple of 64)
  int B;
  int64_t HW;
  int rows_per_chunk;
  float* part;           // [gridDim.z][B][Cpad][2]
  const Ctl* ctl;        // may be null (forward pass)
};

// grid (Cpad / 64, B, chunks), 256 threads = 32 row phases x 8 channel octets
template <class T, bool VJP>
__global__ __launch_bounds__(256) void instnorm_partial(NormPartial g) {
  if (g.ctl && g.ctl->poison) return;
  const int oct = threadIdx.x & 7, phase = threadIdx.x >> 3;
  const int c0 = blockIdx.x * 64 + oct * 8, b = blockIdx.y;
  const int64_t r0 = (int64_t)blockIdx.z * g.rows_per_chunk;
  int64_t r1 = r0 + g.rows_per_chunk;
  if (r1 > g.HW) r1 = g.HW;
  float s1[8], s2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) s1[e] = s2[e] = 0.f;
  for (int64_t r = r0 + phase; r < r1; r += 32) {
    const size_t at = ((size_t)b * g.HW + r) * g.ld + c0;
    const u16x8 x = *reinterpret_cast<const u16x8*>(g.X + at);
    if (VJP) {
      const u16x8 n = *reinterpret_cast<const u16x8*>(g.Nrm + at);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xv = Low<T>::to_f32(x[e]);
        s1[e] += xv;
        s2[e] = fmaf(xv, Low<T>::to_f32(n[e]), s2[e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xv = Low<T>::to_f32(x[e]);
        s1[e] += xv;
        s2[e] = fmaf(xv, xv, s2[e]);
      }
    }
  }
  __shared__ float sh[32][64][2];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sh[phase][oct * 8 + e][0] = s1[e];
    sh[phase][oct * 8 + e][1] = s2[e];
  }
  __syncthreads();
  if (threadIdx.x < 128) {
    const int c = threadIdx.x >> 1, w = threadIdx.x & 1;
    float acc = 0.f;
#pragma unroll
    for (int ph = 0; ph < 32; ++ph) acc += sh[ph][c][w];
    g.part[(((size_t)blockIdx.z * g.B + b) * g.Cpad + blockIdx.x * 64 + c) * 2 + w] = acc;
  }
}

// stat[b][c] = (mean, rstd) (forward) or (mean(dn), mean(dn * n)) (backward); n = B * Cpad entries
template <bool VJP>
__global__ void instnorm_finalize(const float* __restrict__ part, int chunks, int64_t n, float inv_hw, float eps,
                                  float* __restrict__ stat, const Ctl* ctl) {
  if (ctl && ctl->poison) return;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s1 = 0.f, s2 = 0.f;
  for (int c = 0; c < chunks; ++c) {
    s1 += part[((size_t)c * n + i) * 2];
    s2 += part[((size_t)c * n + i) * 2 + 1];
  }
  if (VJP) {
    stat[2 * i] = s1 * inv_hw;
    stat[2 * i + 1] = s2 * inv_hw;
  } else {
    const float mean = s1 * inv_hw;
    const float var = fmaxf(fmaf(-mean, mean, s2 * inv_hw), 0.f);
    stat[2 * i] = mean;
    stat[2 * i + 1] = 1.f / sqrtf(var + eps);
  }
}

struct NormApply {
  const uint16_t* X;      // forward: r; backward: dn
  const uint16_t* Nrm;    // backward: n
  const uint16_t* Rl;     // backward: r (ReLU mask r > 0)
  uint16_t* Out;          // forward: n; backward: du
  int ld, Cpad;
  int64_t HW, rows;       // rows = B * HW
  const float* stat;      // forward statistics [B][Cpad][2] = (mean, rstd)
  const float* stat_vjp;  // backward means [B][Cpad][2]
  Ctl* ctl;               // may be null (forward pass)
  int detect;
};

// grid (row blocks, B); a workgroup of gcols * rpi <= 256 threads (gcols = min(Cpad / 8, 256) channel groups x rpi rows per
// iteration): a thread keeps its channel group, so the sample's statistics of its 8 channels are loaded once, and the
// loop over rows is three 16-byte loads, the arithmetic and one 16-byte store, without index divisions.
inline int instnorm_apply_threads(int Cpad) {
  const int gcols = std::min(Cpad / 8, 256);
  return gcols * (256 / gcols);
}
template <class T, bool VJP>
__global__ __launch_bounds__(256) void instnorm_apply(NormApply g) {
  if (g.ctl && g.ctl->poison) return;
  const int gpr = g.Cpad >> 3;  // groups of 8 channels per row
  const int gcols = gpr < 256 ? gpr : 256;
  const int rpi = (int)blockDim.x / gcols;
  const int rr = (int)threadIdx.x / gcols;
  const int Bn = (int)(g.rows / g.HW);
  bool bad = false;
  for (int b = blockIdx.y; b < Bn; b += gridDim.y)   // (one sample per workgroup row, unless the grid's y extent is short of B)
  for (int cg = (int)threadIdx.x % gcols; cg < gpr; cg += gcols) {
    const int c0 = cg * 8;
    float st[16], sv[16];
    const float4* sp = reinterpret_cast<const float4*>(g.stat + ((size_t)b * g.Cpad + c0) * 2);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 v = sp[q];
      st[4 * q] = v.x; st[4 * q + 1] = v.y; st[4 * q + 2] = v.z; st[4 * q + 3] = v.w;
    }
    if (VJP) {
      const float4* vp = reinterpret_cast<const float4*>(g.stat_vjp + ((size_t)b * g.Cpad + c0) * 2);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = vp[q];
        sv[4 * q] = v.x; sv[4 * q + 1] = v.y; sv[4 * q + 2] = v.z; sv[4 * q + 3] = v.w;
      }
    }
    const size_t base = (size_t)b * g.HW * g.ld + c0;
    for (int64_t r = (int64_t)blockIdx.x * rpi + rr; r < g.HW; r += (int64_t)gridDim.x * rpi) {
      const size_t at = base + (size_t)r * g.ld;
      const u16x8 x = *reinterpret_cast<const u16x8*>(g.X + at);
      u16x8 o;
      if (VJP) {
        const u16x8 n = *reinterpret_cast<const u16x8*>(g.Nrm + at);
        const u16x8 rl = *reinterpret_cast<const u16x8*>(g.Rl + at);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float dn = Low<T>::to_f32(x[e]), nv = Low<T>::to_f32(n[e]);
          float v = st[2 * e + 1] * (dn - sv[2 * e] - nv * sv[2 * e + 1]);
          if (!(Low<T>::to_f32(rl[e]) > 0.f)) v = 0.f;  // ReLU mask of the stored activation
          o[e] = Low<T>::from_f32(v);
          bad |= Low<T>::nonfinite(o[e]);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = Low<T>::from_f32((Low<T>::to_f32(x[e]) - st[2 * e]) * st[2 * e + 1]);
      }
      *reinterpret_cast<u16x8*>(g.Out + at) = o;
    }
  }
  if (VJP && g.detect) raise_if_any(bad, g.ctl);
}

// zero fill that leaves the buffer alone once a cotangent chain has been rejected (the private
// parameter-gradient copies of a block of piecewise-constant weights must survive until the retry)
__global__ void fill_zero_unless_poisoned(uint32_t* p, size_t n, const Ctl* ctl) {
  if (ctl->poison) return;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

}  // namespace rampde
