// Exact-trace row of a continuous-normalising-flow state  y = [z; l],  dl/dt = -tr(dv/dz)  (paper Sec. 6.1)
// for a one-hidden-layer velocity  v = W2 tanh(W1 [z; t] + b1) + b2:
//     tr(dv/dz) = sum_h c_h (1 - a_h^2),   c_h = sum_i W2[i,h] W1[h,i],   a = tanh(.).
// The velocity part runs on the dense per-layer kernels (the l column of the state meets zero weights);
// the kernels here add what the trace row needs:
//   cnf_trace_coef   c_h from the rounded weights (once per pass), fp32;
//   cnf_trace_row    dl/dt of every row into column d of the slope buffer, rounded to low precision;
//   (gemm_nt epilogue) the extra term 2 kbar_l c_h a_h of the activation's cotangent, eq. (vjp);
//   cnf_trace_sums   s_h = sum over rows of kbar_l (1 - a_h^2), the cotangent of -c_h;
//   cnf_trace_grad   dW2[i,h] -= (h/S) W1[h,i] s_h,   dW1[h,i] -= (h/S) W2[i,h] s_h   (fp32, paper Sec. 3 update of g).
#pragma once
#include "common.hpp"

namespace rampde {

// W1p [Hpad][ld1] and W2p [dpad][ld2]: the padded rounded copies of the two layers (row = output feature)
template <class T>
__global__ void cnf_trace_coef(const uint16_t* __restrict__ W1p, int ld1, const uint16_t* __restrict__ W2p, int ld2, int d,
                               int H, int Hpad, float* __restrict__ c) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= Hpad) return;
  float acc = 0.f;
  if (h < H)
    for (int i = 0; i < d; ++i) acc = fmaf(Low<T>::to_f32(W2p[(size_t)i * ld2 + h]), Low<T>::to_f32(W1p[(size_t)h * ld1 + i]), acc);
  c[h] = acc;
}

// one wavefront per row; act [R][Hpad]; writes K[row * ldk + col] = Q(-sum_h c_h (1 - a_h^2))
template <class T>
__global__ __launch_bounds__(256) void cnf_trace_row(const uint16_t* __restrict__ act, int Hpad, const float* __restrict__ c,
                                                     int64_t R, uint16_t* __restrict__ K, int ldk, int col, const Ctl* ctl) {
  if (ctl && ctl->poison) return;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= R) return;
  float acc = 0.f;
  for (int h0 = lane * 8; h0 < Hpad; h0 += 512) {
    const u16x8 a = *reinterpret_cast<const u16x8*>(act + (size_t)row * Hpad + h0);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float av = Low<T>::to_f32(a[e]);
      acc = fmaf(c[h0 + e], fmaf(-av, av, 1.f), acc);
    }
  }
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if (lane == 0) K[(size_t)row * ldk + col] = Low<T>::from_f32(-acc);
}

// s[h] += sum_{rows} kl[row] (1 - a[row][h]^2); grid (Hpad / 64, row chunks), 256 threads = 4 row phases x 64 columns
template <class T>
__global__ __launch_bounds__(256) void cnf_trace_sums(const uint16_t* __restrict__ act, int Hpad,
                                                      const uint16_t* __restrict__ kbar, int ldk, int col, int64_t rows,
                                                      int rows_per_block, float* __restrict__ s, const Ctl* ctl) {
  if (ctl->poison) return;
  const int cidx = threadIdx.x & 63, ph = threadIdx.x >> 6;
  const int h = blockIdx.x * 64 + cidx;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  int64_t r1 = r0 + rows_per_block;
  if (r1 > rows) r1 = rows;
  float acc = 0.f;
  for (int64_t r = r0 + ph; r < r1; r += 4) {
    const float av = Low<T>::to_f32(act[(size_t)r * Hpad + h]);
    acc = fmaf(Low<T>::to_f32(kbar[(size_t)r * ldk + col]), fmaf(-av, av, 1.f), acc);
  }
  __shared__ float sh[4][64];
  sh[ph][cidx] = acc;
  __syncthreads();
  if (ph == 0) unsafeAtomicAdd(&s[h], sh[0][cidx] + sh[1][cidx] + sh[2][cidx] + sh[3][cidx]);
}

// gW1: dW1 block of the gradient vector, row pitch ldg1 (= d + time column); gW2: row pitch ldg2 (= H)
template <class T>
__global__ void cnf_trace_grad(const float* __restrict__ s, const uint16_t* __restrict__ W1p, int ld1,
                               const uint16_t* __restrict__ W2p, int ld2, int d, int H, float h_step, const Ctl* ctl,
                               float* __restrict__ gW1, int ldg1, float* __restrict__ gW2, int ldg2) {
  if (ctl->poison) return;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= H * d) return;
  const int h = idx / d, i = idx - h * d;
  const float f = (h_step / ctl->S_step) * s[h];
  gW2[(size_t)i * ldg2 + h] -= f * Low<T>::to_f32(W1p[(size_t)h * ld1 + i]);
  gW1[(size_t)h * ldg1 + i] -= f * Low<T>::to_f32(W2p[(size_t)i * ld2 + h]);
}

}  // namespace rampde
