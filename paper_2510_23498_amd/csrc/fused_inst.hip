// One translation unit per hidden width and precision: compile with
// -DRAMPDE_INST_HP={0,256,512,1024} -DRAMPDE_INST_BF16={0,1}.
#include "fused_launch.hpp"

#if !defined(RAMPDE_INST_HP) || !defined(RAMPDE_INST_BF16)
#error "define RAMPDE_INST_HP and RAMPDE_INST_BF16"
#endif
#define RAMPDE_CAT2(a, b) a##b
#define RAMPDE_CAT(a, b) RAMPDE_CAT2(a, b)

namespace rampde {

namespace {

template <class Kern>
hipError_t launch_kernel(Kern kern, int waves, const FusedLaunch& l, const FusedArgs& a) {
  if (l.lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)l.lds_bytes);
    if (e != hipSuccess) return e;
  }
  kern<<<l.grid, 64 * waves, l.lds_bytes, l.stream>>>(a);
  return hipGetLastError();
}

template <class T, int MT, int NTL>
hipError_t pick_kernel(const FusedLaunch& l, const FusedArgs& a) {
  // forward pass of 16-row tiles: 16 wavefronts (four per SIMD, under 128 registers each) hide more of
  // the per-pass latencies than 8; the adjoint kernel does not fit that register budget
  if constexpr (MT == 1) {
    if (!l.adjoint && l.waves == 16)
      return launch_kernel(mlp_forward_fused<T, MT, NTL, 16, RAMPDE_INST_HP>, 16, l, a);
  }
  if (l.adjoint) {
    // (the host caps the adjoint's row tile at 32 rows: 64-row tiles spill; several steps per launch
    // only with 8 wavefronts)
    if constexpr (MT <= 2) {
      if (a.tpart) {  // with the sums of the time-grid gradient
        if (a.nsteps > 1) return launch_kernel(mlp_adjoint_step<T, MT, NTL, 8, RAMPDE_INST_HP, true, true>, 8, l, a);
        if (l.waves == 4) return launch_kernel(mlp_adjoint_step<T, MT, NTL, 4, RAMPDE_INST_HP, false, true>, 4, l, a);
        return launch_kernel(mlp_adjoint_step<T, MT, NTL, 8, RAMPDE_INST_HP, false, true>, 8, l, a);
      }
      if (a.nsteps > 1) return launch_kernel(mlp_adjoint_step<T, MT, NTL, 8, RAMPDE_INST_HP, true, false>, 8, l, a);
      if (l.waves == 4) return launch_kernel(mlp_adjoint_step<T, MT, NTL, 4, RAMPDE_INST_HP, false, false>, 4, l, a);
      return launch_kernel(mlp_adjoint_step<T, MT, NTL, 8, RAMPDE_INST_HP, false, false>, 8, l, a);
    } else {
      return hipErrorInvalidValue;
    }
  }
  return launch_kernel(mlp_forward_fused<T, MT, NTL, kForwardWaves, RAMPDE_INST_HP>, kForwardWaves, l, a);
}

template <class T, int MT>
hipError_t pick_ntl(const FusedLaunch& l, const FusedArgs& a) {
  switch (l.NTL) {
    case 1: return pick_kernel<T, MT, 1>(l, a);
    case 2: return pick_kernel<T, MT, 2>(l, a);
    case 4: return pick_kernel<T, MT, 4>(l, a);
    default: return hipErrorInvalidValue;
  }
}

template <class T>
hipError_t pick_mt(const FusedLaunch& l, const FusedArgs& a) {
  switch (l.MT) {
    case 1: return pick_ntl<T, 1>(l, a);
    case 2: return pick_ntl<T, 2>(l, a);
    case 4: return pick_ntl<T, 4>(l, a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

#if RAMPDE_INST_BF16
hipError_t RAMPDE_CAT(RAMPDE_CAT(fused_launch_hp, RAMPDE_INST_HP), _bf16)(const FusedLaunch& l, const FusedArgs& a) {
  return pick_mt<BF16>(l, a);
}
#else
hipError_t RAMPDE_CAT(RAMPDE_CAT(fused_launch_hp, RAMPDE_INST_HP), _f16)(const FusedLaunch& l, const FusedArgs& a) {
  return pick_mt<F16>(l, a);
}
#endif

}  // namespace rampde
