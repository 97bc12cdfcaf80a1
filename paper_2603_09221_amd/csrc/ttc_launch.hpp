// Host-side interface between the C-ABI entry points (ttc_api.hip) and the kernel families, each of which
// is compiled in its own translation unit, once per state size D (the kernels are templates over D and
// the input element type; a translation unit defines the specialisations for its -DTTC_D).
#pragma once
#include <hip/hip_runtime.h>

#include "ttc_args.hpp"

namespace ttc {

// launch_*: enqueue the kernel on `st` with `grid` workgroups; bf16 selects the bfloat16-input instance.
// occupancy_*: resident workgroups per compute unit the runtime reports for that instance (0 on error).
template <int D> hipError_t launch_solve(const SolveArgs& a, bool bf16, dim3 grid, hipStream_t st);
template <int D> int occupancy_solve(bool bf16);
template <int D> hipError_t launch_doubling(const DoublingArgs& a, bool bf16, dim3 grid, hipStream_t st);
template <int D> int occupancy_doubling(bool bf16);
template <int D> hipError_t launch_rollout(const RolloutArgs& a, bool bf16, dim3 grid, hipStream_t st);
template <int D> int occupancy_rollout(bool bf16);
template <int D> hipError_t launch_tv(const TvArgs& a, bool bf16, dim3 grid, hipStream_t st);
template <int D> int occupancy_tv(bool bf16);
template <int D> hipError_t launch_rollout_tv(const TvRolloutArgs& a, bool bf16, dim3 grid, hipStream_t st);
template <int D> int occupancy_rollout_tv(bool bf16);
// ipw = items per workgroup: 1, or 4 (d = 16 only: the kernels that take four items per wavefront)
template <int D> hipError_t launch_scan_leaf(const ScanArgs& a, bool bf16, int ipw, dim3 grid, hipStream_t st);
template <int D> hipError_t launch_scan_combine(const ScanArgs& a, int ipw, dim3 grid, hipStream_t st);
template <int D> hipError_t launch_scan_apply(const ScanArgs& a, int ipw, dim3 grid, hipStream_t st);
template <int D> hipError_t launch_scan_gather(const ScanArgs& a, float* P, dim3 grid, hipStream_t st);
template <int D> int occupancy_scan();

template <int D> hipError_t launch_backward(const BackwardArgs& a, bool bf16, dim3 grid, hipStream_t st);
template <int D> int occupancy_backward(bool bf16);

// d = 16 only; ppw = problems per wavefront (1 or 4)
hipError_t launch_small(const SolveArgs& a, bool bf16, int ppw, dim3 grid, hipStream_t st);
int occupancy_small(bool bf16);
hipError_t launch_tv_small(const TvArgs& a, bool bf16, int ppw, dim3 grid, hipStream_t st);
int occupancy_tv_small(bool bf16);
hipError_t launch_cxt(const CxtArgs& a, bool bf16, int ppw, dim3 grid, hipStream_t st);
int occupancy_cxt(bool bf16);
hipError_t launch_rollout_cxt_forward(const CxtRolloutArgs& a, bool bf16, dim3 grid, hipStream_t st);

// backward pass of the structured problems (ttc_cxt_backward.hpp): one wavefront per four problems of the chunk (vec),
// one workgroup per slab of problems (basis), a plain fill
hipError_t launch_cxt_backward_vec(const CxtBackwardArgs& a, bool bf16, dim3 grid, hipStream_t st);
hipError_t launch_cxt_basis(const CxtBackwardArgs& a, bool bf16, hipStream_t st);
hipError_t launch_zero_floats(float* dst, long long n, hipStream_t st);
// the block around the structured solver (ttc_block.hpp)
hipError_t launch_ln_stats(const LnStatsArgs& a, bool bf16, hipStream_t st);
hipError_t launch_gemm_ln_bf16(const GemmLnBf16Args& a, bool x_bf16, bool out_bf16, hipStream_t st);
hipError_t launch_gemm_ln(const GemmLnArgs& a, hipStream_t st);
hipError_t launch_cxt_maps(const CxtMapsArgs& a, int blocks, hipStream_t st);
hipError_t launch_qbasis(const float* Qc, float* Qb, int r, hipStream_t st);

template <typename K>
inline int occupancy_query(K kernel, int nthr) {
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, nthr, 0) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return nb;
}

}  // namespace ttc
