// Roll-out kernel of the time-invariant problem (Alg. 1, forward loop, r = 0).
#pragma once
#include "ttc_common.hpp"

namespace ttc {

// ------------------------------------------------------------------------------------------------

// y[r] = sum_c M[r][c] x[c] for the row r = tid / TPR of a row-major global d x d matrix; the TPR
// threads of a row (adjacent lanes) each take a share of the columns; all of them get the sum.
template <int D, typename TM>
__device__ __forceinline__ float matvec_row(const TM* M, const float* xs, int tid) {
  constexpr int TPR = Cfg<D>::NTHR / D;  // 2 or 4
  const int r = tid / TPR, part = tid % TPR;
  float s = 0.f;
#pragma unroll
  for (int c4 = part * (D / TPR); c4 < (part + 1) * (D / TPR); c4 += 4) {
    const floatx4 mv = ld4<TM>(M, (long)r * D + c4);
    s += mv[0] * xs[c4] + mv[1] * xs[c4 + 1] + mv[2] * xs[c4 + 2] + mv[3] * xs[c4 + 3];
  }
#pragma unroll
  for (int m = 1; m < TPR; m <<= 1) s += __shfl_xor(s, m, 64);
  return s;
}

// Roll-out kernel (Alg. 1 with r = 0).  Backward sweep: the value matrices P_T .. P_1 are produced
// one step at a time in the re-based form of the reverse symplectic factor (re-base every step):
//     M_t = (I + P_{t+1} G)^{-1} P_{t+1} A,   K_t = -(R^{-1} B^T) M_t,   P_t = Q + A^T M_t,
// the gains go to the workspace; forward sweep: u_t = K_t x_t, x_{t+1} = A x_t + B u_t and the cost.
template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) rollout_kernel(const RolloutArgs p) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  __shared__ float s_x[D], s_u[D], s_xn[D];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  float* const wsC = p.ws + (long)blockIdx.x * (p.T + 3) * D * D;  // G, X, A^T in register layout
  float* const wsK = wsC + 3 * D * D;                              // K_0 .. K_{T-1}, row-major

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* QTp = p.QT ? reinterpret_cast<const TIn*>(p.QT) + prob * p.sQT : Qp;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    int info = 0, nsolve = 0;
    floatx4 acc[C::RB][C::NT];

    // ---- setup: X = R^{-1} B^T, G = B X; row blocks of G, X, A^T to the workspace
    load_half<D, TIn, false>(WL, Rp, tid);
    load_half<D, TIn, false>(WR, Bp, tid);
    __syncthreads();
    symmetrise_half<D>(WL, tid);
    transpose_half<D>(WR, w, i, g);              // RHS = B^T
    ++nsolve;
    if (lds_solve<D, 7, false>(W, S, tid) && !info) info = nsolve;  // R is positive definite: no pivot search
    {
      float c[C::RB][C::KS];
      load_aop_lds<D>(WR, c, w, i, g);
      store_aop_ws<D>(wsC + 1 * D * D, c, tid);
      load_aop_global<D, TIn>(Bp, c, w, i, g);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, c, WR, i, g);
      store_rows<D>(WL, acc, w, i, g);
      __syncthreads();
      symmetrise_half<D>(WL, tid);
      __syncthreads();
      load_aop_lds<D>(WL, c, w, i, g);
      store_aop_ws<D>(wsC + 0 * D * D, c, tid);
#pragma unroll
      for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
        for (int k = 0; k < C::KS; ++k)
          c[rb][k] = ld1<TIn>(Ap, (long)(16 * (k / 4) + 4 * g + (k % 4)) * D + 16 * (C::RB * w + rb) + i);
      store_aop_ws<D>(wsC + 2 * D * D, c, tid);
    }
    __syncthreads();
    load_half<D, TIn, false>(WR, QTp, tid);
    __syncthreads();
    symmetrise_half<D>(WR, tid);
    __syncthreads();

    // ---- backward sweep (the constant row blocks stay in registers)
    float cG[C::RB][C::KS], cX[C::RB][C::KS], cAT[C::RB][C::KS];
    load_aop_ws<D>(wsC + 0 * D * D, cG, tid, 0);
    load_aop_ws<D>(wsC + 1 * D * D, cX, tid, 0);
    load_aop_ws<D>(wsC + 2 * D * D, cAT, tid, 0);
    for (int t = p.T - 1; t >= 0; --t) {
      eye_acc<D>(acc, w, i, g);
      gemm_acc<D>(acc, cG, WR, i, g);   // (I + P G)^T
      store_rows_T<D>(WL, acc, w, i, g);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cAT, WR, i, g);  // (P A)^T
      __syncthreads();
      store_rows_T<D>(WR, acc, w, i, g);
      __syncthreads();
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cX, WR, i, g);    // -K_t
#pragma unroll
      for (int rb = 0; rb < C::RB; ++rb) {
#pragma unroll
        for (int cc = 0; cc < C::NT; ++cc) acc[rb][cc] = -acc[rb][cc];
        write_rows_global<D>(wsK + (long)t * D * D, acc[rb], C::RB * w + rb, i, g);
      }
      if (t >= 1) {
#pragma unroll
        for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
          for (int cc = 0; cc < C::NT; ++cc)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const long row = 16 * (C::RB * w + rb) + 4 * g + v, col = tile_col<D>(cc, i);
              acc[rb][cc][v] = 0.5f * (ld1<TIn>(Qp, row * D + col) + ld1<TIn>(Qp, col * D + row));
            }
        gemm_acc<D>(acc, cAT, WR, i, g);  // P_t = Q + A^T M_t
        __syncthreads();
        store_rows<D>(WR, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WR, tid);
        __syncthreads();
      }
    }
    __syncthreads();  // gains visible to the whole workgroup

    // ---- forward sweep
    const int r = tid / (C::NTHR / D), part = tid % (C::NTHR / D);
    if (tid < D) s_x[tid] = ld1<TIn>(x0p, tid);
    __syncthreads();
    float cpart = 0.f;
    if (p.flags & TTC_FLAG_STAGE_COST_AT_X0) {
      const float qx = matvec_row<D, TIn>(Qp, s_x, tid);
      if (part == 0) cpart += s_x[r] * qx;
    }
    if (p.X && tid < D) p.X[prob * (long)(p.T + 1) * D + tid] = s_x[tid];
    for (int t = 0; t < p.T; ++t) {
      const float u = matvec_row<D, float>(wsK + (long)t * D * D, s_x, tid);
      if (part == 0) s_u[r] = u;
      __syncthreads();
      const float ru = matvec_row<D, TIn>(Rp, s_u, tid);
      const float xn = matvec_row<D, TIn>(Ap, s_x, tid) + matvec_row<D, TIn>(Bp, s_u, tid);
      if (part == 0) {
        cpart += s_u[r] * ru;
        s_xn[r] = xn;
        p.U[(prob * p.T + t) * (long)D + r] = info ? __builtin_nanf("") : u;
      }
      __syncthreads();
      const float qx = matvec_row<D, TIn>(t == p.T - 1 ? QTp : Qp, s_xn, tid);
      if (part == 0) {
        cpart += s_xn[r] * qx;
        s_x[r] = xn;
        if (p.X) p.X[(prob * (p.T + 1) + t + 1) * (long)D + r] = info ? __builtin_nanf("") : xn;
      }
      __syncthreads();
    }
    cpart = sum64(cpart);
    if (lane == 0) s_red[w] = cpart;
    __syncthreads();
    if (tid == 0) {
      float cst = 0.f;
      for (int ww = 0; ww < C::NW; ++ww) cst += s_red[ww];
      if (p.cost) p.cost[prob] = info ? __builtin_nanf("") : cst;
      if (p.info) p.info[prob] = info;
    }
    __syncthreads();
  }
}

}  // namespace ttc
