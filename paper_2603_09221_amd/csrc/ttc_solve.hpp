// The solve kernel of d >= 32: reverse symplectic iteration in groups with re-basing (Thm 3.3, Alg. 4).
#pragma once
#include "ttc_common.hpp"
#include "ttc_tv.hpp"

#ifndef TTC_D64_WAVES
#define TTC_D64_WAVES 2  // d = 64: two wavefronts per SIMD (four workgroups per compute unit): one problem's dense solve overlaps another's products
#endif
namespace ttc {

// Solve kernel.  Persistent workgroups: workgroup b handles problems b, b + gridDim.x, ...
//
// Per problem the work is a sequence of phases, each "build [M | RHS] in LDS, dense solve, consume":
//   phase R  X = R^{-1} B^T, then G = B X (Thm 3.3's G).
//   phase A  A^{-1}; C_K = X A^{-T}; Z2 = Q_T, Z1 = I.
//   phase S  one group of reverse symplectic steps (Alg. 4 body), the last one leaving the
//            pair untransposed; the solve re-bases it, [Y1 Y2] <- [I, Y1^{-1} Y2].  Repeated until all
//            T factors Sigma_T .. Sigma_1 are applied; the last factor has Q_0 = 0, i.e. no "+ Y1 Q".
//   output   after the last solve the right half is P_0 = Y1^{-1} Y2 itself (Alg. 4), lambda_0 = P_0 x0,
//            and K_0 = -R^{-1} B^T A^{-T} P_0 = -C_K P_0 (Thm A.4: u_1 = -R^{-1} B^T A^{-T} lambda_0).
// The row blocks of G, A^T, Q and A^{-1} go from LDS straight into registers as they are produced and
// stay there to the end of the problem; only C_K, needed once at the very end, waits in the workspace.
// Global reads are started a phase ahead of their use where registers allow.
template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR, (D == 64 ? TTC_D64_WAVES : 1)) solve_kernel(const SolveArgs p) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  __shared__ float s_growth[C::NW];  // per wavefront: max |Y1| after the step just taken

  float* const WL = W;      // left half  (Z1 / Y1 / M of a dense solve)
  float* const WR = W + D;  // right half (Z2 / Y2 / RHS)
  // per-workgroup workspace: the row blocks of C_K in register layout
  float* const wsC = p.ws + (long)blockIdx.x * D * D;
  const bool pure = (p.flags & TTC_FLAG_PURE_SYMPLECTIC) != 0;

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    // (the opaque zero keeps the address arithmetic of a problem from being hoisted out of this loop and spilled)
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    TTC_TIMER_DECL
    int info = 0, nsolve = 0;
    floatx4 acc[C::RB][C::NT];
    int s = 1;          // next reverse step (1 .. T; step s applies Sigma_{T-s+1})
    int grp = 0;        // current group of steps
    bool fresh = true;  // Z1 = I, not materialised
    bool hard = false;  // the growth guard tripped: this problem goes to the Riccati recursion instead
    int plan_base = 0, plan_T = p.T, plan_ng = p.ngroups;  // grouping of the steps after plan_base
    // the constant row blocks, in registers from here to the end of the problem
    float cG[C::RB][C::KS], cAi[C::RB][C::KS], cAT[C::RB][C::KS], cQ[C::RB][C::KS];

    // ---------------------------------------------------------------- phase R: X = R^{-1} B^T, G = B X
    load_half<D, TIn, false>(WL, reinterpret_cast<const TIn*>(p.R) + prob * p.sR, tid);
    load_half<D, TIn, false>(WR, reinterpret_cast<const TIn*>(p.B) + prob * p.sB, tid);
    __syncthreads();
    symmetrise_half<D>(WL, tid);
    transpose_half<D>(WR, w, i, g);              // RHS = B^T
    {
      float cX[C::RB][C::KS];
      {
        float cB[C::RB][C::KS];
        load_aopT_lds<D>(WR, cB, w, i, g);       // rows of B = columns of B^T
        TTC_TOC(6)
        ++nsolve;
        if (lds_solve<D, 7, false>(W, S, tid) && !info) info = nsolve;  // R is positive definite: no pivot search
        TTC_TOC(1)
        zero_acc<D>(acc);
        gemm_acc<D>(acc, cB, WR, i, g);          // rows of G = B X
        load_aop_lds<D>(WR, cX, w, i, g);        // rows of X, for C_K
        store_rows<D>(WL, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WL, tid);             // G is symmetric up to rounding; make it exactly so
        __syncthreads();
        load_aop_lds<D>(WL, cG, w, i, g);
        __syncthreads();
        TTC_TOC(7)
        // ------------------------------------------------------------ phase A: A^{-1}, A^T, Q, C_K
        // (read here, one matrix after the other: started before the product above, the sixteen pieces a thread
        // holds of each matrix do not fit the registers next to its operands and are spilled one by one, each
        // read waited for on its own)
        load_half<D, TIn, false>(WL, Ap, tid + opaque_zero());
        load_half<D, TIn, false>(WR, Qp, tid + opaque_zero());
      }
      __syncthreads();
      symmetrise_half<D>(WR, tid);
      load_aopT_lds<D>(WL, cAT, w, i, g);        // rows of A^T = columns of A
      __syncthreads();
      load_aop_lds<D>(WR, cQ, w, i, g);          // rows of the symmetric part of Q
      __syncthreads();
      set_half_identity<D>(WR, tid);
      __syncthreads();
      TTC_TOC(0)
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;
      TTC_TOC(1)
      load_aop_lds<D>(WR, cAi, w, i, g);
      __syncthreads();
      transpose_half<D>(WR, w, i, g);            // A^{-T}
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cX, WR, i, g);            // rows of C_K = X A^{-T}
    }
    store_rows<D>(WL, acc, w, i, g);
    __syncthreads();
    {
      float c[C::RB][C::KS];
      load_aop_lds<D>(WL, c, w, i, g);
      store_aop_ws<D>(wsC, c, tid);
    }
    // initial pair [Y1 Y2] = [I Q_T]
    if (p.QT) {
      load_half<D, TIn, false>(WR, reinterpret_cast<const TIn*>(p.QT) + prob * p.sQT, tid);
      __syncthreads();
      symmetrise_half<D>(WR, tid);
    } else {
      store_aop_lds<D>(WR, cQ, w, i, g);         // Q_T = Q, already symmetric
    }
    __syncthreads();

    // ---------------------------------------------------------------- groups of steps, each ended by a re-base
    for (;;) {
      {
        TTC_TOC(2)
        const int tg = tid + opaque_zero(), lane = tg & 63, w = tg >> 6, i = lane & 15, g = lane >> 4;
        // last step of this group: the plan_T steps from plan_base on are cut into plan_ng groups whose lengths
        // differ by at most one, the longer groups first
        const int gend = plan_base + plan_T - (int)(((long long)(plan_ng - 1 - grp) * plan_T) / plan_ng);
        float g_prev = 1.f;  // max |Y1| before the step: the group starts from Y1 = I
        for (int k = 1;; ++s, ++k) {
          bool last = (s >= gend);
          if (fresh) eye_acc<D>(acc, w, i, g); else load_rows<D>(WL, acc, w, i, g);
          gemm_acc<D>(acc, cG, WR, i, g);    // Z1 + G Z2       (Y1 + Y2 G)
          store_rows<D>(WL, acc, w, i, g);
          __syncthreads();
          zero_acc<D>(acc);
          gemm_acc<D>(acc, cAi, WL, i, g);   // A^{-1} (.)      (... A^{-T})  = new Z1
          if (p.growth_limit > 0.f) {
            const float mx = wave_absmax<D>(acc);
            if (lane == 0) s_growth[w] = mx;
          }
          __syncthreads();
          store_rows<D>(WL, acc, w, i, g);
          __syncthreads();
          if (p.growth_limit > 0.f) {
            // Growth guard.  Y1 starts a group as the identity and its inverse stays of order one (it is the
            // closed-loop transition over the group), so max |Y1| tracks cond(Y1), which is what the float32
            // error of P = Y1^{-1} Y2 is proportional to.  A group that is about to pass the limit (the last
            // step's growth repeated) ends here, and the rest of the horizon is re-planned with groups no
            // longer than this one; a pair that has passed it takes the problem out of the symplectic
            // iteration, to the recursion of Prop. 3.1 in its printed form (below).
            float gm = s_growth[0];
#pragma unroll
            for (int ww = 1; ww < C::NW; ++ww) gm = fmaxf(gm, s_growth[ww]);
            if (!(gm <= p.growth_limit) && !info) {  // also true for NaN; every thread reads the same values
              // (a problem whose set-up broke down is NaN anyway and keeps its report)
              hard = true;
              break;
            }
            if (!last && k >= 2 && s < p.T && gm * (gm / g_prev) > p.growth_limit) {
              last = true;
              plan_base = s;
              plan_T = p.T - s;
              plan_ng = (plan_T + k - 1) / k;
              grp = -1;  // the next group is the first of the new plan
            }
            g_prev = gm;
          }
          zero_acc<D>(acc);
          gemm_acc<D>(acc, cAT, WR, i, g);   // A^T Z2          (Y2 A)
          if (s < p.T) gemm_acc<D>(acc, cQ, WL, i, g);  // + Q Z1 (+ Y1 Q_{t-1}); Q_0 = 0 for the last factor
          __syncthreads();
          fresh = false;
          if (!last) {
            store_rows<D>(WR, acc, w, i, g);
            __syncthreads();
            if (pure) {
              normalise_rows_zland<D>(W, tid);
              __syncthreads();
            }
          } else {
            // leave Z-land: [Y1 | Y2] untransposed for the solve Y1 P = Y2
            store_rows_T<D>(WR, acc, w, i, g);
            load_rows<D>(WL, acc, w, i, g);
            __syncthreads();
            store_rows_T<D>(WL, acc, w, i, g);
            __syncthreads();
            ++s;
            break;
          }
        }
      }
      if (hard) break;
      TTC_TOC(3)
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;
      TTC_TOC(4)
      symmetrise_half<D>(WR, tid);           // P is symmetric; also makes it its own Z-land image
      __syncthreads();
      fresh = true;
      ++grp;
      if (s > p.T) break;
    }

    if (hard) {
      // Prop. 3.1 as printed, from P_T: one positive definite solve per step, no A^{-1}, no accumulated factors
      // (what ttc_lqr_solve_tv runs, here with the same matrices in every step).  info: 2 + index of the step.
      __syncthreads();  // every wavefront has left the pair
      const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
      const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
      const TIn* QTp = p.QT ? reinterpret_cast<const TIn*>(p.QT) + prob * p.sQT : Qp;
      riccati_problem<D, TIn>(W, S, s_red, p, prob, p.T, Ap, Bp, Qp, Rp, 0, 0, 0, 0, QTp, nullptr, Qp, x0p, 2,
                              tid + opaque_zero());
      continue;
    }
    // ---- outputs: WR holds P_0 (paper convention, Q_0 = 0)
    {
      float c[C::RB][C::KS];
      load_aop_ws<D>(wsC, c, tid, opaque_zero());  // C_K; in flight while P_0 is written out
      emit_value<D, TIn>(p, prob, WR, Qp, x0p, info, s_red, tid);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, c, WR, i, g);               // -K_0 = C_K P_0
    }
    emit_gain<D, TIn>(p, prob, acc, x0p, info, tid);
    __syncthreads();                               // every wavefront is done with the pair
    TTC_TOC(5)
    TTC_TIMER_DUMP(p)
  }
}

}  // namespace ttc
