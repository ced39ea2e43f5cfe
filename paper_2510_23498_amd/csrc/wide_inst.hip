// Instantiations and launcher of the 64-row-tile kernels for 512-wide dense networks.
#include "fused_launch.hpp"
#include "wide.hpp"

namespace rampde {

namespace {
template <class Kern>
hipError_t launch_wide_kernel(Kern kern, const FusedLaunch& l, const FusedArgs& a) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)l.lds_bytes);
  if (e != hipSuccess) return e;
  kern<<<l.grid, 64 * kWideWaves, l.lds_bytes, l.stream>>>(a);
  return hipGetLastError();
}
}  // namespace

hipError_t wide_launch(const FusedLaunch& l, const FusedArgs& a) {
  if (a.dpad != 128 || a.d != 128 || a.L < 2 || a.L > kMaxLayers || a.ldk >= ((int64_t)1 << 27)) return hipErrorInvalidValue;
  for (int q = 0; q + 1 < a.L; ++q)
    if (a.layer[q].Npad != 512) return hipErrorInvalidValue;
  if (l.lds_bytes != wide_lds_bytes<512, 128>(a.nparam)) return hipErrorInvalidValue;
  if (l.adjoint) {
    if (a.nsteps != 1 || a.tpart) return hipErrorInvalidValue;
    return l.bf16 ? launch_wide_kernel(mlp_adjoint_wide<BF16, 512, 128>, l, a)
                  : launch_wide_kernel(mlp_adjoint_wide<F16, 512, 128>, l, a);
  }
  if (!a.bsum) return hipErrorInvalidValue;
  return l.bf16 ? launch_wide_kernel(mlp_forward_wide<BF16, 512, 128>, l, a)
                : launch_wide_kernel(mlp_forward_wide<F16, 512, 128>, l, a);
}

}  // namespace rampde
