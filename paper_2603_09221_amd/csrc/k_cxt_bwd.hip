// backward_cxt_vec_kernel, cxt_basis_kernel (ttc_lqr_backward_cxt).
#include "ttc_cxt_backward.hpp"
#include "ttc_launch.hpp"

namespace ttc {
hipError_t launch_cxt_backward_vec(const CxtBackwardArgs& a, bool bf16, dim3 grid, hipStream_t st) {
  if (bf16) hipLaunchKernelGGL((backward_cxt_vec_kernel<uint16_t>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((backward_cxt_vec_kernel<float>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_cxt_basis(const CxtBackwardArgs& a, bool bf16, hipStream_t st) {
  const dim3 grid((unsigned)((a.count + a.basis_slab - 1) / a.basis_slab));
  if (bf16) hipLaunchKernelGGL((cxt_basis_kernel<uint16_t>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((cxt_basis_kernel<float>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_zero_floats(float* dst, long long n, hipStream_t st) {
  long long blocks = (n + 255) / 256;
  blocks = blocks < 1 ? 1 : blocks > 4096 ? 4096 : blocks;
  hipLaunchKernelGGL(zero_floats_kernel, dim3((unsigned)blocks), dim3(256), 0, st, dst, n);
  return hipGetLastError();
}
}  // namespace ttc
