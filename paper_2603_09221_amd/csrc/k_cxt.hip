// solve_cxt_kernel and rollout_cxt_forward_kernel (ttc_lqr_solve_cxt, ttc_lqr_rollout_cxt; d = 16).
#include "ttc_cxt.hpp"
#include "ttc_launch.hpp"

namespace ttc {
hipError_t launch_cxt(const CxtArgs& a, bool bf16, int ppw, dim3 grid, hipStream_t st) {
  if (ppw == 4) {
    if (bf16) hipLaunchKernelGGL((solve_cxt_kernel<uint16_t, 4>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((solve_cxt_kernel<float, 4>), grid, dim3(64), 0, st, a);
  } else {
    if (bf16) hipLaunchKernelGGL((solve_cxt_kernel<uint16_t, 1>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((solve_cxt_kernel<float, 1>), grid, dim3(64), 0, st, a);
  }
  return hipGetLastError();
}
int occupancy_cxt(bool bf16) {
  return bf16 ? occupancy_query(solve_cxt_kernel<uint16_t, 4>, 64) : occupancy_query(solve_cxt_kernel<float, 4>, 64);
}
hipError_t launch_rollout_cxt_forward(const CxtRolloutArgs& a, bool bf16, dim3 grid, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((rollout_cxt_forward_kernel<uint16_t>), grid, dim3(64), 0, st, a);
  else hipLaunchKernelGGL((rollout_cxt_forward_kernel<float>), grid, dim3(64), 0, st, a);
  return hipGetLastError();
}
}  // namespace ttc
