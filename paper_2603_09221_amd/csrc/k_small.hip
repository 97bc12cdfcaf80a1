// solve_small_kernel (ttc_lqr_solve at d = 16, default path): one or four problems per wavefront.
#include "ttc_small_kernel.hpp"
#include "ttc_launch.hpp"

namespace ttc {
hipError_t launch_small(const SolveArgs& a, bool bf16, int ppw, dim3 grid, hipStream_t st) {
  if (ppw == 4) {
    if (bf16) hipLaunchKernelGGL((solve_small_kernel<uint16_t, 4>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((solve_small_kernel<float, 4>), grid, dim3(64), 0, st, a);
  } else {
    if (bf16) hipLaunchKernelGGL((solve_small_kernel<uint16_t, 1>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((solve_small_kernel<float, 1>), grid, dim3(64), 0, st, a);
  }
  return hipGetLastError();
}
int occupancy_small(bool bf16) {
  return bf16 ? occupancy_query(solve_small_kernel<uint16_t, 4>, 64) : occupancy_query(solve_small_kernel<float, 4>, 64);
}
}  // namespace ttc
