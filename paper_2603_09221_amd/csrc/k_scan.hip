// scan_leaf_kernel<TTC_D>, scan_combine_kernel<TTC_D> (ttc_lqr_solve_tv_scan) and the down-sweep of
// ttc_lqr_tv_scan_values: one translation unit per state size.  At d = 16 the kernels of ttc_scan16.hpp, which take
// four items per wavefront, serve the rounds with many items (ipw = 4: the grid counts groups of four items).
#if TTC_D == 16
#include "ttc_scan16.hpp"
#else
#include "ttc_scan.hpp"
#endif
#include "ttc_launch.hpp"

namespace ttc {
template <>
hipError_t launch_scan_leaf<TTC_D>(const ScanArgs& a, bool bf16, int ipw, dim3 grid, hipStream_t st) {
#if TTC_D == 16
  if (ipw == 4) {
    if (bf16) hipLaunchKernelGGL((scan_leaf16_kernel<uint16_t>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((scan_leaf16_kernel<float>), grid, dim3(64), 0, st, a);
    return hipGetLastError();
  }
#endif
  if (bf16) hipLaunchKernelGGL((scan_leaf_kernel<TTC_D, uint16_t>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  else hipLaunchKernelGGL((scan_leaf_kernel<TTC_D, float>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
hipError_t launch_scan_combine<TTC_D>(const ScanArgs& a, int ipw, dim3 grid, hipStream_t st) {
#if TTC_D == 16
  if (ipw == 4) {
    hipLaunchKernelGGL(scan_combine16_kernel, grid, dim3(64), 0, st, a);
    return hipGetLastError();
  }
#endif
  hipLaunchKernelGGL((scan_combine_kernel<TTC_D>), grid, dim3(Cfg<TTC_D>::NTHR), 0, st, a);
  return hipGetLastError();
}
template <>
hipError_t launch_scan_apply<TTC_D>(const ScanArgs& a, int ipw, dim3 grid, hipStream_t st) {
#if TTC_D == 16
  if (ipw == 4) {
    hipLaunchKernelGGL(scan_apply16_kernel, grid, dim3(64), 0, st, a);
    return hipGetLastError();
  }
#endif
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
