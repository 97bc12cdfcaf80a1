// scan_leaf_kernel<TTC_D>, scan_combine_kernel<TTC_D> (ttc_lqr_solve_tv_scan) and the down-sweep of
// ttc_lqr_tv_scan_values: one translation unit per state size.
#include "ttc_scan.hpp"
#include "ttc_launch.hpp"

namespace ttc {
template <>
hipError_t launch_scan_leaf<TTC_D>(const ScanArgs& a, bool bf16, dim3 grid, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((scan_leaf_kernel<TTC_D, uint16_t>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  else hipLaunchKernelGGL((scan_leaf_kernel<TTC_D, float>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
hipError_t launch_scan_combine<TTC_D>(const ScanArgs& a, dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((scan_combine_kernel<TTC_D>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
hipError_t launch_scan_apply<TTC_D>(const ScanArgs& a, dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((scan_apply_kernel<TTC_D>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
hipError_t launch_scan_gather<TTC_D>(const ScanArgs& a, float* P, dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((scan_gather_kernel<TTC_D>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a, P);
  return hipGetLastError();
}
template <>
int occupancy_scan<TTC_D>() {  // the pairwise compositions (the leaf kernel uses fewer registers)
  return occupancy_query(scan_combine_kernel<TTC_D>, Cfg<TTC_D>::NTHR);
}
}  // namespace ttc
