// backward_kernel<TTC_D> (ttc_lqr_backward, ttc_lqr_backward_tv): one translation unit per state size.
#include "ttc_backward.hpp"
#include "ttc_launch.hpp"

namespace ttc {
template <>
hipError_t launch_backward<TTC_D>(const BackwardArgs& a, bool bf16, dim3 grid, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((backward_kernel<TTC_D, uint16_t>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  else hipLaunchKernelGGL((backward_kernel<TTC_D, float>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
int occupancy_backward<TTC_D>(bool bf16) {
  return bf16 ? occupancy_query(backward_kernel<TTC_D, uint16_t>, Cfg<TTC_D>::NTHR)
              : occupancy_query(backward_kernel<TTC_D, float>, Cfg<TTC_D>::NTHR);
}
}  // namespace ttc
