// Launchers of the row-tile-persistent kernels.  The kernels are instantiated per hidden width
// (0 = run-time widths, 256 / 512 / 1024 = all hidden layers padded to that width, known at
// compile time), one translation unit each so that they compile in parallel.
#pragma once
#include <hip/hip_runtime.h>

#include "fused.hpp"

namespace rampde {

// Wavefronts per workgroup.  Forward: 8, two per SIMD (hides the latencies of a single row tile).
// Adjoint step: 8, or 4 (one per SIMD) for narrow networks, which leaves registers and LDS for the
// parameter-gradient kernel of the previous step to run on the same compute units at the same time.
constexpr int kForwardWaves = 8;

struct FusedLaunch {
  int adjoint;   // 0: mlp_forward_fused, 1: mlp_adjoint_step
  int waves;     // adjoint only: 4 or 8 wavefronts per workgroup
  int bf16;      // 0: fp16, 1: bfloat16
  int MT;        // row tile = 16 * MT rows, MT in {1, 2, 4}
  int NTL;       // dpad / 64, in {1, 2, 4}
  unsigned grid;
  size_t lds_bytes;
  hipStream_t stream;
};

// Each returns hipSuccess or the error of the attribute call / launch.  One function per hidden
// width and precision, each in a translation unit of its own (they compile in parallel).
#define RAMPDE_DECLARE_FUSED(hp)                                                   \
  hipError_t fused_launch_hp##hp##_f16(const FusedLaunch& l, const FusedArgs& a);  \
  hipError_t fused_launch_hp##hp##_bf16(const FusedLaunch& l, const FusedArgs& a); \
  inline hipError_t fused_launch_hp##hp(const FusedLaunch& l, const FusedArgs& a) { \
    return l.bf16 ? fused_launch_hp##hp##_bf16(l, a) : fused_launch_hp##hp##_f16(l, a); \
  }
RAMPDE_DECLARE_FUSED(0)
RAMPDE_DECLARE_FUSED(256)
RAMPDE_DECLARE_FUSED(512)
RAMPDE_DECLARE_FUSED(1024)
#undef RAMPDE_DECLARE_FUSED

// the 64-row-tile kernels for 512-wide networks (wide.hpp): state width 128; l.MT, l.NTL and l.waves are not used
hipError_t wide_launch(const FusedLaunch& l, const FusedArgs& a);

}  // namespace rampde
