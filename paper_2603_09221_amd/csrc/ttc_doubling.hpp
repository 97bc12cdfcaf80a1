// Long-horizon path of the solver: the Riccati steps of a time-invariant problem composed by squaring.
//
// One backward step of Prop. 3.1, written with G = B R^{-1} B^T (the G of Thm 3.3), is the map
//     f_e(P) = H_e + A_e^T P (I + G_e P)^{-1} A_e          of the element e = (A_e, G_e, H_e) = (A, G, Q).
// These maps are the symplectic transfer matrices Sigma_t of Thm 3.3 in a parametrisation that needs
// no A^{-1}, and they are closed under composition: f_e o f_e = f_e' with
//     M = (I + G_e H_e)^{-1},   A' = A_e M A_e,   G' = G_e + A_e M G_e A_e^T,   H' = H_e + A_e^T H_e M A_e.
// The paper multiplies the T factors one after the other (Sec. 3.3, "sequential" product); with
// time-invariant parameters (its "Homo." setting) the product of 2^k equal factors is k squarings.
//
// Schedule for horizon T (host side: ttc_lqr_solve):
//   P_1 = f^(T-1)(Q_T); when Q_T is Q itself, Q = f(0) gives P_1 = f^T(0).  With m = T or T-1 the
//   number of maps to apply, the bits of m are visited from the lowest: a set bit k applies f_{e^(2^k)}
//   to P (one dense solve; free while P is still 0, since f_e(0) = H_e), and e is squared between bits.
//   The last step is taken on its own because it also yields the gain (Eq. "decode"):
//     M_1 = (I + P_1 G)^{-1} P_1 A,   P_0 = A^T M_1 (the paper's Q_0 = 0),   K_0 = -R^{-1} B^T M_1.
//
// Data flow: a product is (row blocks of the left matrix in registers) x (right matrix in one half of
// the LDS pair).  The element lives in the workgroup's workspace as plain row-major fp32 matrices
// (L2/Infinity-Cache resident, 64 KB each at d = 128) and is pulled into LDS or registers in the role
// each product needs; a wavefront only ever rewrites the rows it alone reads in that phase.
#pragma once
#include "ttc_common.hpp"

namespace ttc {

// one half of the LDS pair -> plain row-major global matrix
template <int D>
__device__ __forceinline__ void store_half_global(float* dst, const float* Wh, int tid) {
  using C = Cfg<D>;
  for (int idx = tid; idx < D * D / 4; idx += C::NTHR) {
    const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
    *reinterpret_cast<floatx4*>(dst + (long)r * D + c4) = *reinterpret_cast<const floatx4*>(Wh + r * C::PITCH + c4);
  }
}
// accumulator rows of this wavefront <- plain row-major global matrix (the mirror of write_rows_global)
template <int D>
__device__ __forceinline__ void load_rows_global(const float* src, floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT], int w, int i,
                                                 int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int h = 0; h < C::NH; ++h) {
        float t[C::VEC];
        lds_ldv<C::VEC>(src + (long)(16 * (C::RB * w + rb) + 4 * g + v) * D + 16 * C::VEC * h + C::VEC * i, t);
#pragma unroll
        for (int tp = 0; tp < C::VEC; ++tp) acc[rb][h * C::VEC + tp][v] = t[tp];
      }
}
template <int D>
__device__ __forceinline__ void write_rows_global(float* dst, const floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT], int w, int i,
                                                  int g) {
#pragma unroll
  for (int rb = 0; rb < Cfg<D>::RB; ++rb) write_rows_global<D>(dst, acc[rb], Cfg<D>::RB * w + rb, i, g);
}
// e <- e o e in the workspace (gA, gG, gH).  Returns the solve's breakdown flag.
// Global reads are started one product ahead of their use (issue_half / load_*_global into registers
// that are only consumed after the next product), so that their latency is covered by matrix work.
template <int D>
__device__ __forceinline__ int square_element(float* W, SolveScratch<D>& S, float* gA, float* gG, float* gH, int tid,
                                              PhaseTimers& tm) {
  using C = Cfg<D>;
  tid += opaque_zero();  // address arithmetic starts afresh here instead of living in registers from kernel entry
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  floatx4 acc[C::RB][C::NT];
  HalfRegs<D> hA;
  {
    float rG[C::RB][C::KS];
    load_half<D, float, false>(WR, gH, tid);
    load_aop_global<D, float>(gG, rG, w, i, g);
    __syncthreads();
    issue_half<D, float>(hA, gA, tid);  // wanted right after the solve
    eye_acc<D>(acc, w, i, g);
    gemm_acc<D>(acc, rG, WR, i, g);  // I + G H
    store_rows<D>(WL, acc, w, i, g);
    __syncthreads();
  }
  set_half_identity<D>(WR, tid);
  __syncthreads();
  tm.toc(2);
  const int flag = lds_solve<D>(W, S, tid);  // right half: M = (I + G H)^{-1}
  tm.toc(1);

  float rM[C::RB][C::KS], rA[C::RB][C::KS], rAT[C::RB][C::KS];
  floatx4 init[C::RB][C::NT];
  load_aop_lds<D>(WR, rM, w, i, g);
  commit_half<D, false>(WL, hA, tid);
  __syncthreads();
  {
    HalfRegs<D> hG;
    float rH[C::RB][C::KS];
    issue_half<D, float>(hG, gG, tid);  // G is the right operand of A G below; M is in registers now
    load_aop_global<D, float>(gH, rH, w, i, g);
    zero_acc<D>(acc);
    gemm_acc<D>(acc, rM, WL, i, g);  // X1 = M A
    commit_half<D, false>(WR, hG, tid);
    load_aop_lds<D>(WL, rA, w, i, g);
    load_aopT_lds<D>(WL, rAT, w, i, g);
    __syncthreads();
    store_rows<D>(WL, acc, w, i, g);
    __syncthreads();
    load_rows_global<D>(gH, init, w, i, g);  // for H' two products later
    zero_acc<D>(acc);
    gemm_acc<D>(acc, rA, WL, i, g);  // A' = A X1
    write_rows_global<D>(gA, acc, w, i, g);
    zero_acc<D>(acc);
    gemm_acc<D>(acc, rH, WL, i, g);  // V = H X1
  }
  __syncthreads();
  store_rows<D>(WL, acc, w, i, g);
  zero_acc<D>(acc);
  gemm_acc<D>(acc, rA, WR, i, g);  // A G
  __syncthreads();
  store_rows_T<D>(WR, acc, w, i, g);  // right half: G A^T
  gemm_acc<D>(init, rAT, WL, i, g);  // H' = H + A^T V
  write_rows_global<D>(gH, init, w, i, g);
  load_rows_global<D>(gG, init, w, i, g);  // for G' one product later
  __syncthreads();
  zero_acc<D>(acc);
  gemm_acc<D>(acc, rM, WR, i, g);  // X2 = M G A^T
  store_rows<D>(WL, acc, w, i, g);  // (every wavefront is past its reads of V)
  __syncthreads();
  gemm_acc<D>(init, rA, WL, i, g);  // G' = G + A X2
  write_rows_global<D>(gG, init, w, i, g);
  __syncthreads();
  tm.toc(2);
  return flag;
}

// gH <- H of e o e only (A and G of the square are not needed after the last squaring when P is still 0)
template <int D>
__device__ __forceinline__ int square_element_H(float* W, SolveScratch<D>& S, const float* gA, const float* gG, float* gH,
                                                int tid, PhaseTimers& tm) {
  using C = Cfg<D>;
  tid += opaque_zero();  // address arithmetic starts afresh here instead of living in registers from kernel entry
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  floatx4 acc[C::RB][C::NT];
  {
    float rG[C::RB][C::KS];
    load_half<D, float, false>(WR, gH, tid);
    load_aop_global<D, float>(gG, rG, w, i, g);
    __syncthreads();
    eye_acc<D>(acc, w, i, g);
    gemm_acc<D>(acc, rG, WR, i, g);  // I + G H
    store_rows<D>(WL, acc, w, i, g);
    __syncthreads();
  }
  float rAT[C::RB][C::KS];
  load_half<D, float, false>(WR, gA, tid);
  __syncthreads();
  load_aopT_lds<D>(WR, rAT, w, i, g);
  tm.toc(2);
  const int flag = lds_solve<D>(W, S, tid);  // right half: X1 = (I + G H)^{-1} A
  tm.toc(1);
  {
    float rH[C::RB][C::KS];
    load_aop_global<D, float>(gH, rH, w, i, g);
    zero_acc<D>(acc);
    gemm_acc<D>(acc, rH, WR, i, g);  // V = H X1
  }
  store_rows<D>(WL, acc, w, i, g);
  __syncthreads();
  load_rows_global<D>(gH, acc, w, i, g);
  gemm_acc<D>(acc, rAT, WL, i, g);  // H' = H + A^T V
  write_rows_global<D>(gH, acc, w, i, g);
  __syncthreads();
  tm.toc(2);
  return flag;
}

// Builds [I + P G | P A] in LDS and solves: afterwards the right half is (I + P G)^{-1} P A and rAT holds
// the wavefront's rows of A^T.
template <int D, typename TA>
__device__ __forceinline__ int mobius_solve(float* W, SolveScratch<D>& S, const TA* Asrc, const float* Gsrc,
                                            const float* Psrc, float (&rAT)[Cfg<D>::RB][Cfg<D>::KS], int tid,
                                            PhaseTimers& tm) {
  using C = Cfg<D>;
  tid += opaque_zero();  // address arithmetic starts afresh here instead of living in registers from kernel entry
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  {
    floatx4 accY[C::RB][C::NT], accR[C::RB][C::NT];
    float rP[C::RB][C::KS];
    load_half<D, float, false>(WL, Gsrc, tid);
    load_half<D, TA, false>(WR, Asrc, tid);
    load_aop_global<D, float>(Psrc, rP, w, i, g);
    __syncthreads();
    eye_acc<D>(accY, w, i, g);
    gemm_acc<D>(accY, rP, WL, i, g);  // I + P G
    zero_acc<D>(accR);
    gemm_acc<D>(accR, rP, WR, i, g);  // P A
    load_aopT_lds<D>(WR, rAT, w, i, g);
    __syncthreads();
    store_rows<D>(WL, accY, w, i, g);
    store_rows<D>(WR, accR, w, i, g);
    __syncthreads();
  }
  tm.toc(3);
  const int flag = lds_solve<D>(W, S, tid);
  tm.toc(1);
  return flag;
}


template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) doubling_kernel(const DoublingArgs da) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  const SolveArgs& p = da.s;

  float* const WL = W;
  float* const WR = W + D;
  float* const ws = p.ws + (long)blockIdx.x * DBL_SLOTS * D * D;
  float* const gA = ws + DBL_A * D * D;
  float* const gG = ws + DBL_G * D * D;
  float* const gH = ws + DBL_H * D * D;
  float* const gG0 = ws + DBL_G0 * D * D;
  float* const gP = ws + DBL_P * D * D;
  float* const gX = ws + DBL_X * D * D;  // rows of R^{-1} B^T in register layout

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    int info = 0, nsolve = 0;
    floatx4 acc[C::RB][C::NT];
    PhaseTimers tm;  // phases: 0 set-up, 1 dense solves, 2 squarings, 3 applications and last step, 4 outputs

    // ---- set-up: X = R^{-1} B^T, G = B X; the element e = (A, G, Q) goes to the workspace
    load_half<D, TIn, false>(WL, Rp, tid);
    load_half<D, TIn, false>(WR, Bp, tid);
    __syncthreads();
    symmetrise_half<D>(WL, tid);
    transpose_half<D>(WR, w, i, g);
    ++nsolve;
    tm.toc(0);
    if (lds_solve<D, 7, false>(W, S, tid) && !info) info = nsolve;  // R is positive definite: no pivot search
    tm.toc(1);
    {
      float c[C::RB][C::KS];
      load_aop_lds<D>(WR, c, w, i, g);
      store_aop_ws<D>(gX, c, tid);
      load_aop_global<D, TIn>(Bp, c, w, i, g);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, c, WR, i, g);  // rows of G = B X
      store_rows<D>(WL, acc, w, i, g);
      __syncthreads();
      symmetrise_half<D>(WL, tid);
      load_half<D, TIn, false>(WR, Qp, tid);
      __syncthreads();
      symmetrise_half<D>(WR, tid);
      store_half_global<D>(gG, WL, tid);
      store_half_global<D>(gG0, WL, tid);
      __syncthreads();
      store_half_global<D>(gH, WR, tid);
      load_half<D, TIn, false>(WL, Ap, tid);
      __syncthreads();
      store_half_global<D>(gA, WL, tid);
      if (da.p_from_qt) {
        load_half<D, TIn, false>(WR, reinterpret_cast<const TIn*>(p.QT) + prob * p.sQT, tid);
        __syncthreads();
        symmetrise_half<D>(WR, tid);
        __syncthreads();
        store_half_global<D>(gP, WR, tid);
      }
      __syncthreads();
    }

    tm.toc(0);
    // ---- P_1 by binary powering of the one-step map
    const float* Pcur = gP;
    bool have_p = da.p_from_qt != 0;
    for (int m = da.m; m;) {
      if (m & 1) {
        if (!have_p) {
          have_p = true;
          if (m == 1) {
            Pcur = gH;  // f_e(0) = H_e, and e is not touched again
          } else {
            load_half<D, float, false>(WL, gH, tid);
            __syncthreads();
            store_half_global<D>(gP, WL, tid);
            __syncthreads();
          }
        } else {
          float rAT[C::RB][C::KS];
          ++nsolve;
          if (mobius_solve<D, float>(W, S, gA, gG, gP, rAT, tid, tm) && !info) info = nsolve;
          load_rows_global<D>(gH, acc, w, i, g);
          gemm_acc<D>(acc, rAT, WR, i, g);  // P <- H_e + A_e^T (I + P G_e)^{-1} P A_e
          write_rows_global<D>(gP, acc, w, i, g);
          __syncthreads();
          tm.toc(3);
        }
      }
      m >>= 1;
      if (m) {
        ++nsolve;
        const int flag = (m == 1 && !have_p) ? square_element_H<D>(W, S, gA, gG, gH, tid, tm)
                                             : square_element<D>(W, S, gA, gG, gH, tid, tm);
        if (flag && !info) info = nsolve;
      }
    }

    // ---- last step with the problem's own (A, G): M_1, then P_0 = A^T M_1 and -K_0 = X M_1
    {
      float rAT[C::RB][C::KS];
      ++nsolve;
      if (mobius_solve<D, TIn>(W, S, Ap, gG0, Pcur, rAT, tid, tm) && !info) info = nsolve;
      zero_acc<D>(acc);
      gemm_acc<D>(acc, rAT, WR, i, g);
      store_rows<D>(WL, acc, w, i, g);
      __syncthreads();
      symmetrise_half<D>(WL, tid);
      __syncthreads();
    }
    {
      float c[C::RB][C::KS];
      load_aop_ws<D>(gX, c, tid, 0);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, c, WR, i, g);
    }
    tm.toc(3);
    emit_gain<D, TIn>(p, prob, acc, x0p, info, tid);
    emit_value<D, TIn>(p, prob, WL, Qp, x0p, info, s_red, tid);
    tm.toc(4);
    tm.dump(p);
  }
}

}  // namespace ttc
