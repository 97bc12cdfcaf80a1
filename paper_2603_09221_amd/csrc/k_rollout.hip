// rollout_kernel<TTC_D> (ttc_lqr_rollout): one translation unit per state size.
#include "ttc_rollout.hpp"
#include "ttc_launch.hpp"

namespace ttc {
template <>
hipError_t launch_rollout<TTC_D>(const RolloutArgs& a, bool bf16, dim3 grid, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((rollout_kernel<TTC_D, uint16_t>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  else hipLaunchKernelGGL((rollout_kernel<TTC_D, float>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
int occupancy_rollout<TTC_D>(bool bf16) {
  return bf16 ? occupancy_query(rollout_kernel<TTC_D, uint16_t>, Cfg<TTC_D>::NTHR)
              : occupancy_query(rollout_kernel<TTC_D, float>, Cfg<TTC_D>::NTHR);
}
}  // namespace ttc
