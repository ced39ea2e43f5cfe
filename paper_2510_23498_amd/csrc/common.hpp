// Shared device-side definitions for the gfx950 neural-ODE time stepper.
// Low-precision formats, rounding (the paper's Q16 operator, Sec. 2: round to
// nearest even into fp16 or bfloat16), the MFMA wrappers and the device control
// block of the dynamic adjoint scaling (paper Algorithm 2).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rampde {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxStages = 8;
constexpr int kPad = 64;  // every internal feature dimension is padded to a multiple of this

// Device control block: one per backward pass, lives in the workspace.
struct Ctl {
  float S;             // current adjoint scale (power of two)
  int attempt;         // attempt number at the current step (1 = first)
  int poison;          // non-zero: a VJP chain produced a non-finite value; all later kernels exit
  int failed_step;     // step at which poison was raised (N for a non-finite dL/dy_N)
  unsigned nonfinite;  // raised by the overflow detector of the cotangent chain
  unsigned amax_bits;  // bit pattern of max |a| (non-negative floats order like unsigned ints)
  int retries;         // number of halvings so far
  float s_min, s_max;
  int done;            // workgroups of the current adjoint-step kernel that have finished
  float S_step;        // scale of the most recently accepted step (used by its parameter-gradient kernels)
  int pad[5];
};
static_assert(sizeof(Ctl) == 64, "control block layout");

struct F16 {};
struct BF16 {};

template <class T>
struct Low;

template <>
struct Low<F16> {
  static constexpr int p_bits = 11;  // unit roundoff 2^-11
  __device__ static inline uint16_t from_f32(float x) {
    _Float16 h = (_Float16)x;  // v_cvt_f16_f32: round to nearest even, gradual underflow, overflow -> inf
    return __builtin_bit_cast(uint16_t, h);
  }
  __device__ static inline float to_f32(uint16_t u) { return (float)__builtin_bit_cast(_Float16, u); }
  // two values rounded and packed (first in the low half): one v_cvt_pkrtz-free RNE conversion pair
  __device__ static inline uint32_t pack2(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v;
    v[0] = (_Float16)a;
    v[1] = (_Float16)b;
    return __builtin_bit_cast(uint32_t, v);
  }
  __device__ static inline bool nonfinite(uint16_t u) { return (u & 0x7C00u) == 0x7C00u; }
  __device__ static inline f32x16 mfma32(u16x8 a, u16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
  __device__ static inline f32x4 mfma16(u16x8 a, u16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};

template <>
struct Low<BF16> {
  static constexpr int p_bits = 8;  // unit roundoff 2^-8
  __device__ static inline uint16_t from_f32(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;  // NaN
    u += 0x7FFFu + ((u >> 16) & 1u);                       // ties to even; carries into inf on overflow
    return (uint16_t)(u >> 16);
  }
  __device__ static inline float to_f32(uint16_t u) { return __builtin_bit_cast(float, (uint32_t)u << 16); }
  // two values rounded (nearest even, hardware conversion of gfx950) and packed, first in the low half
  __device__ static inline uint32_t pack2(float a, float b) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
  }
  __device__ static inline bool nonfinite(uint16_t u) { return (u & 0x7F80u) == 0x7F80u; }
  __device__ static inline f32x16 mfma32(u16x8 a, u16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  __device__ static inline f32x4 mfma16(u16x8 a, u16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

// tanh of an fp32 pre-activation; the result is rounded to low precision by the caller.
__device__ inline float act_tanh(float x) { return tanhf(x); }

// Wavefront-level OR of a per-lane overflow flag, one atomic per wavefront that saw one.
__device__ inline void raise_if_any(bool bad, Ctl* ctl) {
  if (__any(bad ? 1 : 0)) {
    if ((threadIdx.x & 63) == 0) atomicOr(&ctl->nonfinite, 1u);
  }
}

// Block-wide max of |x| bit patterns, then one atomicMax per workgroup.
__device__ inline void block_amax(unsigned bits, unsigned* dst) {
  for (int o = 32; o > 0; o >>= 1) {
    unsigned other = __shfl_xor(bits, o);
    bits = bits > other ? bits : other;
  }
  __shared__ unsigned wmax[16];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) wmax[w] = bits;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned m = 0;
    int nw = (blockDim.x + 63) >> 6;
    for (int i = 0; i < nw; ++i) m = wmax[i] > m ? wmax[i] : m;
    if (m) atomicMax(dst, m);
  }
}

// Block-wide sums of two per-thread values, stored to dst[0], dst[1]: the workgroup's slot of a launch-wide table that
// a one-workgroup kernel folds in a fixed order afterwards (fold_time_slots), so that the result does not depend on
// the order in which workgroups finish.  (Must be reached by every thread of the workgroup.)
__device__ inline void block_sum2(float a, float b, float* dst) {
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_xor(a, o);
    b += __shfl_xor(b, o);
  }
  __shared__ float wsum[16][2];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();  // (a previous call's readers are done)
  if (lane == 0) {
    wsum[w][0] = a;
    wsum[w][1] = b;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float s0 = 0.f, s1 = 0.f;
    const int nw = (blockDim.x + 63) >> 6;
    for (int i = 0; i < nw; ++i) {
      s0 += wsum[i][0];
      s1 += wsum[i][1];
    }
    dst[0] = s0;
    dst[1] = s1;
  }
}

}  // namespace rampde
