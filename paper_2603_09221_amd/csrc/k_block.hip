// ln_stats_kernel, gemm_ln_kernel, cxt_maps_kernel, qbasis_kernel (ttc_block_forward).
#include "ttc_block.hpp"
#include "ttc_launch.hpp"

namespace ttc {
hipError_t launch_ln_stats(const LnStatsArgs& a, bool bf16, hipStream_t st) {
  const dim3 grid((unsigned)((a.M + 3) / 4));
  if (bf16) hipLaunchKernelGGL((ln_stats_kernel<unsigned short>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((ln_stats_kernel<float>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}
// x_bf16: X is bfloat16 (else float32); out_bf16: Y is bfloat16 (else float32)
hipError_t launch_gemm_ln_bf16(const GemmLnBf16Args& a, bool x_bf16, bool out_bf16, hipStream_t st) {
  const long long total = ((a.M + GEMM_BM - 1) / GEMM_BM) * ((a.N + GEMM_BN - 1) / GEMM_BN);
  const dim3 grid((unsigned)(8 * ((total + 7) / 8)));
  if (x_bf16 && !out_bf16) hipLaunchKernelGGL((gemm_ln_bf16_kernel<unsigned short, false>), grid, dim3(256), 0, st, a);
  else if (!x_bf16 && out_bf16) hipLaunchKernelGGL((gemm_ln_bf16_kernel<float, true>), grid, dim3(256), 0, st, a);
  else if (x_bf16 && out_bf16) hipLaunchKernelGGL((gemm_ln_bf16_kernel<unsigned short, true>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((gemm_ln_bf16_kernel<float, false>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_gemm_ln(const GemmLnArgs& a, hipStream_t st) {
  const long long total = ((a.M + GEMM_BM - 1) / GEMM_BM) * ((a.N + GEMM_BN - 1) / GEMM_BN);
  const long long per = (total + 7) / 8;
  hipLaunchKernelGGL(gemm_ln_kernel, dim3((unsigned)(8 * per)), dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_cxt_maps(const CxtMapsArgs& a, int blocks, hipStream_t st) {
  if (a.r == 16 && a.H % 4 == 0) {  // `blocks` counts (token chunk, group of four heads) pairs here
    hipLaunchKernelGGL(cxt_maps16_kernel, dim3((unsigned)blocks), dim3(512), 0, st, a);
    return hipGetLastError();
  }
  const int nout = 80 + 3 * a.r;
  hipLaunchKernelGGL(cxt_maps_kernel, dim3((unsigned)blocks), dim3((unsigned)(64 * ((nout + 63) / 64))), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_qbasis(const float* Qc, float* Qb, int r, hipStream_t st) {
  hipLaunchKernelGGL(qbasis_kernel, dim3((unsigned)r), dim3(256), 0, st, Qc, Qb);
  return hipGetLastError();
}
}  // namespace ttc
