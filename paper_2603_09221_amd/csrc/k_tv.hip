// solve_tv_kernel<TTC_D> and rollout_tv_kernel<TTC_D> (ttc_lqr_solve_tv, ttc_lqr_rollout_tv): one
// translation unit per state size.
#include "ttc_tv.hpp"
#include "ttc_launch.hpp"

namespace ttc {
template <>
hipError_t launch_tv<TTC_D>(const TvArgs& a, bool bf16, dim3 grid, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((solve_tv_kernel<TTC_D, uint16_t>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  else hipLaunchKernelGGL((solve_tv_kernel<TTC_D, float>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
int occupancy_tv<TTC_D>(bool bf16) {
  return bf16 ? occupancy_query(solve_tv_kernel<TTC_D, uint16_t>, Cfg<TTC_D>::NTHR)
              : occupancy_query(solve_tv_kernel<TTC_D, float>, Cfg<TTC_D>::NTHR);
}
template <>
hipError_t launch_rollout_tv<TTC_D>(const TvRolloutArgs& a, bool bf16, dim3 grid, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((rollout_tv_kernel<TTC_D, uint16_t>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  else hipLaunchKernelGGL((rollout_tv_kernel<TTC_D, float>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
int occupancy_rollout_tv<TTC_D>(bool bf16) {
  return bf16 ? occupancy_query(rollout_tv_kernel<TTC_D, uint16_t>, Cfg<TTC_D>::NTHR)
              : occupancy_query(rollout_tv_kernel<TTC_D, float>, Cfg<TTC_D>::NTHR);
}
}  // namespace ttc
