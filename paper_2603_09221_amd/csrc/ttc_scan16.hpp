// The tree over the horizon (ttc_scan.hpp) at d = 16: four elements, compositions or applications per wavefront.
//
// At d = 16 an element fills a quarter of a wavefront and the dense solve inside a composition is most of its
// instructions; as in the d = 16 solve kernels (ttc_small.hpp) a workgroup of one wavefront takes four items at a
// time, forms the products item by item on the matrix cores and runs the four dense solves side by side, lane
// 16q + r owning row r of item q.  The arithmetic, the workspace layout and the order of the rounds are those of the
// kernels of ttc_scan.hpp; a ragged last group of four repeats its last item and writes it once.
#pragma once
#include "ttc_scan.hpp"
#include "ttc_small.hpp"

namespace ttc {

constexpr int SCAN16_PPW = 4;

template <typename TIn>
__global__ void __launch_bounds__(64, 2) scan_leaf16_kernel(const ScanArgs a) {
  constexpr int D = 16, PPW = SCAN16_PPW;
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  const SolveArgs& p = a.tv.s;
  const long long items = p.n * p.T;
  const long long nquads = (items + PPW - 1) / PPW;
  for (long long quad = blockIdx.x; quad < nquads; quad += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, i = lane & 15, g = lane >> 4;
    constexpr int w = 0;
    float* const Wmine = Wm[g & (PPW - 1)];
    bool valid[PPW], terminal[PPW];
    const TIn *Ap[PPW], *Rp[PPW];
    float* gA[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      valid[q] = quad * PPW + q < items;
      const long long item = valid[q] ? quad * PPW + q : items - 1;
      const long long prob = item / p.T;
      const int k = (int)(item % p.T);
      terminal[q] = k == p.T - 1;
      // the terminal element has no step of its own: it reads the last step's matrices (in bounds) and writes zeros
      const int s = terminal[q] ? k : k + 1;
      Ap[q] = reinterpret_cast<const TIn*>(p.A) + prob * p.sA + (long long)s * a.tv.tA;
      Rp[q] = reinterpret_cast<const TIn*>(p.R) + prob * p.sR + (long long)s * a.tv.tR;
      const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB + (long long)s * a.tv.tB;
      const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ + (long long)k * a.tv.tQ;  // Q[k] = Q_{s-1}
      gA[q] = a.ws + item * 3 * D * D;
      load_half<D, TIn, false>(Wm[q], Qp, tid);
      load_half<D, TIn, true>(Wm[q] + D, Bp, tid);  // right-hand sides: B^T
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
    __syncthreads();
    floatx4 acc[PPW][C::RB][C::NT];
    float cB[PPW][C::RB][C::KS];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      if (valid[q]) store_half_global<D>(gA[q] + 2 * D * D, Wm[q], tid);  // H = sym(Q[k])
      load_aopT_lds<D>(Wm[q] + D, cB[q], w, i, g);                        // rows of B = columns of B^T
      load_rows_input<D, TIn>(Ap[q], acc[q], w, i, g);
      if (terminal[q]) zero_acc<D>(acc[q]);
      if (valid[q]) write_rows_global<D>(gA[q], acc[q], w, i, g);         // A
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) load_half<D, TIn, false>(Wm[q], Rp[q], tid);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
    __syncthreads();
    const unsigned long long badm = __ballot(solve_rows16<false>(Wmine, lane) != 0);  // right halves: X = R^{-1} B^T
#pragma unroll
    for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
    gemm_acc_quad<PPW>(acc, cB, Wm, D, i, g);  // G = B X
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      if (!valid[q]) continue;
      const bool bad = !terminal[q] && ((badm >> (16 * q)) & 0xFFFFull) != 0;
      if (terminal[q]) zero_acc<D>(acc[q]);
      if (bad) poison<D>(acc[q]);
      write_rows_global<D>(gA[q] + D * D, acc[q], w, i, g);
      if (bad) write_rows_global<D>(gA[q] + 2 * D * D, acc[q], w, i, g);  // the breakdown reaches P_1 whatever follows
    }
    __syncthreads();
  }
}

// one round of pairwise compositions, four pairs per wavefront
__global__ void __launch_bounds__(64, 2) scan_combine16_kernel(const ScanArgs a) {
  constexpr int D = 16, PPW = SCAN16_PPW;
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  const SolveArgs& p = a.tv.s;
  const int st = a.stride;
  const long long per = (p.T - st + 2LL * st - 1) / (2LL * st);  // pairs per problem in this round
  const long long items = p.n * per;
  const long long nquads = (items + PPW - 1) / PPW;
  for (long long quad = blockIdx.x; quad < nquads; quad += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, i = lane & 15, g = lane >> 4;
    constexpr int w = 0;
    float* const Wmine = Wm[g & (PPW - 1)];
    bool valid[PPW];
    float* out[PPW];   // A1, G1, H1 in the workspace: rewritten
    const float* e1[PPW];
    const float* e2[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      valid[q] = quad * PPW + q < items;
      const long long item = valid[q] ? quad * PPW + q : items - 1;
      const long long prob = item / per;
      const long long j = (item % per) * 2 * st;
      out[q] = a.ws + (prob * p.T + j) * 3 * D * D;
      e1[q] = out[q];
      e2[q] = a.ws + (prob * p.T + j + st) * 3 * D * D;  // A2, G2, H2
    }
    floatx4 acc[PPW][C::RB][C::NT], accY[PPW][C::RB][C::NT];
    float rM[PPW][C::RB][C::KS], rA1T[PPW][C::RB][C::KS], rA2[PPW][C::RB][C::KS];
    {
      float rG1[PPW][C::RB][C::KS];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_half<D, float, false>(Wm[q] + D, e2[q] + 2 * D * D, tid);  // H2
        load_aop_global<D, float>(e1[q] + D * D, rG1[q], w, i, g);
        eye_acc<D>(acc[q], w, i, g);
      }
      __syncthreads();
      gemm_acc_quad<PPW>(acc, rG1, Wm, D, i, g);  // I + G1 H2
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
      __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < PPW; ++q) set_half_identity<D>(Wm[q] + D, tid);
    __syncthreads();
    const unsigned long long badm = __ballot(solve_rows16<true>(Wmine, lane) != 0);  // right halves: M = (I + G1 H2)^{-1}
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      load_aop_lds<D>(Wm[q] + D, rM[q], w, i, g);
      load_half<D, float, false>(Wm[q], e1[q], tid);  // A1
      zero_acc<D>(acc[q]);
      zero_acc<D>(accY[q]);
    }
    __syncthreads();
    gemm_acc_quad<PPW>(acc, rM, Wm, 0, i, g);  // X1 = M A1
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      load_aopT_lds<D>(Wm[q], rA1T[q], w, i, g);
      load_half<D, float, false>(Wm[q] + D, e1[q] + D * D, tid);  // G1 (M is in registers)
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);  // left halves: X1
    gemm_acc_quad<PPW>(accY, rM, Wm, D, i, g);                             // Y = M G1
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      load_aop_global<D, float>(e2[q], rA2[q], w, i, g);
      zero_acc<D>(acc[q]);
    }
    gemm_acc_quad<PPW>(acc, rA2, Wm, 0, i, g);  // A = A2 X1
    {
      float rH2[PPW][C::RB][C::KS];
      floatx4 accV[PPW][C::RB][C::NT];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_aop_global<D, float>(e2[q] + 2 * D * D, rH2[q], w, i, g);
        zero_acc<D>(accV[q]);
      }
      gemm_acc_quad<PPW>(accV, rH2, Wm, 0, i, g);  // V = H2 X1
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q] + D, accV[q], w, i, g);  // right halves: V (G1 has been used)
    }
    __syncthreads();
    {
      floatx4 accH[PPW][C::RB][C::NT];
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_rows_global<D>(e1[q] + 2 * D * D, accH[q], w, i, g);
      gemm_acc_quad<PPW>(accH, rA1T, Wm, D, i, g);  // H = H1 + A1^T V
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if ((badm >> (16 * q)) & 0xFFFFull) poison<D>(accH[q]);
        if (valid[q]) {
          write_rows_global<D>(out[q], acc[q], w, i, g);               // A
          write_rows_global<D>(out[q] + 2 * D * D, accH[q], w, i, g);  // H
        }
        store_rows<D>(Wm[q], accY[q], w, i, g);  // left halves: Y
        zero_acc<D>(acc[q]);
      }
    }
    __syncthreads();
    gemm_acc_quad<PPW>(acc, rA2, Wm, 0, i, g);  // Z = A2 Y
#pragma unroll
    for (int q = 0; q < PPW; ++q) load_half<D, float, true>(Wm[q] + D, e2[q], tid);  // right halves: A2^T
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);  // left halves: Z
    __syncthreads();
    {
      float rZ[PPW][C::RB][C::KS];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_aop_lds<D>(Wm[q], rZ[q], w, i, g);
        load_rows_global<D>(e2[q] + D * D, acc[q], w, i, g);  // G2
      }
      gemm_acc_quad<PPW>(acc, rZ, Wm, D, i, g);  // G = G2 + Z A2^T
#pragma unroll
      for (int q = 0; q < PPW; ++q)
        if (valid[q]) write_rows_global<D>(out[q] + D * D, acc[q], w, i, g);
    }
    __syncthreads();
  }
}

// one level of the down-sweep, four elements per wavefront: P <- H_e + A_e^T (I + P G_e)^{-1} P A_e into the element's H
__global__ void __launch_bounds__(64, 2) scan_apply16_kernel(const ScanArgs a) {
  constexpr int D = 16, PPW = SCAN16_PPW;
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  const SolveArgs& p = a.tv.s;
  const int st = a.stride;
  const long long per = (p.T - st + 2LL * st - 1) / (2LL * st);  // elements j + st per problem in this round
  const long long items = p.n * per;
  const long long nquads = (items + PPW - 1) / PPW;
  for (long long quad = blockIdx.x; quad < nquads; quad += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, i = lane & 15, g = lane >> 4;
    constexpr int w = 0;
    float* const Wmine = Wm[g & (PPW - 1)];
    bool valid[PPW];
    float* out[PPW];  // the element's H in the workspace
    const float* e[PPW];
    const float* gP[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      valid[q] = quad * PPW + q < items;
      const long long item = valid[q] ? quad * PPW + q : items - 1;
      const long long prob = item / per;
      const long long j = (item % per) * 2 * st;
      // an element whose range reaches the terminal cost is a constant map: its H is P already, nothing to write; it
      // goes through the arithmetic on its own (finite) matrices with its own H standing in for the value on its right
      const bool reaches_end = j + 2 * st >= p.T;
      valid[q] = valid[q] && !reaches_end;
      e[q] = a.ws + (prob * p.T + j + st) * 3 * D * D;
      out[q] = a.ws + ((prob * p.T + j + st) * 3 + 2) * D * D;
      gP[q] = reaches_end ? e[q] + 2 * D * D : a.ws + ((prob * p.T + j + 2 * st) * 3 + 2) * D * D;
    }
    floatx4 accY[PPW][C::RB][C::NT], accR[PPW][C::RB][C::NT];
    float rAT[PPW][C::RB][C::KS];
    {
      float rP[PPW][C::RB][C::KS];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_half<D, float, false>(Wm[q], e[q] + D * D, tid);  // G
        load_half<D, float, false>(Wm[q] + D, e[q], tid);      // A
        load_aop_global<D, float>(gP[q], rP[q], w, i, g);
        eye_acc<D>(accY[q], w, i, g);
        zero_acc<D>(accR[q]);
      }
      __syncthreads();
      gemm_acc_quad<PPW>(accY, rP, Wm, 0, i, g);  // I + P G
      gemm_acc_quad<PPW>(accR, rP, Wm, D, i, g);  // P A
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aopT_lds<D>(Wm[q] + D, rAT[q], w, i, g);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        store_rows<D>(Wm[q], accY[q], w, i, g);
        store_rows<D>(Wm[q] + D, accR[q], w, i, g);
      }
      __syncthreads();
    }
    const unsigned long long badm = __ballot(solve_rows16<true>(Wmine, lane) != 0);  // right halves: (I + P G)^{-1} P A
#pragma unroll
    for (int q = 0; q < PPW; ++q) load_rows_global<D>(e[q] + 2 * D * D, accY[q], w, i, g);
    gemm_acc_quad<PPW>(accY, rAT, Wm, D, i, g);
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      if ((badm >> (16 * q)) & 0xFFFFull) poison<D>(accY[q]);
      if (valid[q]) write_rows_global<D>(out[q], accY[q], w, i, g);
    }
    __syncthreads();
  }
}

}  // namespace ttc
