// solve_tv_small_kernel (ttc_lqr_solve_tv at d = 16): one or four problems per wavefront.
#include "ttc_tv.hpp"
#include "ttc_launch.hpp"

namespace ttc {
hipError_t launch_tv_small(const TvArgs& a, bool bf16, int ppw, dim3 grid, hipStream_t st) {
  if (ppw == 4) {
    if (bf16) hipLaunchKernelGGL((solve_tv_small_kernel<uint16_t, 4>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((solve_tv_small_kernel<float, 4>), grid, dim3(64), 0, st, a);
  } else {
    if (bf16) hipLaunchKernelGGL((solve_tv_small_kernel<uint16_t, 1>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((solve_tv_small_kernel<float, 1>), grid, dim3(64), 0, st, a);
  }
  return hipGetLastError();
}
int occupancy_tv_small(bool bf16) {
  return bf16 ? occupancy_query(solve_tv_small_kernel<uint16_t, 4>, 64)
              : occupancy_query(solve_tv_small_kernel<float, 4>, 64);
}
}  // namespace ttc
