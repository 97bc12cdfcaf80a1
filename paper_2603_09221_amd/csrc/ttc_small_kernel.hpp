// The d = 16 solve kernel of the default path: four problems per wavefront (or one, for small batches), the
// device pieces of ttc_small.hpp, and the recursion of Prop. 3.1 (ttc_tv.hpp) for problems the growth guard
// takes out of the symplectic iteration.
#pragma once
#include "ttc_small.hpp"
#include "ttc_tv.hpp"

namespace ttc {

// PPW = problems per wavefront: 4 for batches that fill the chip, 1 for small ones (the four rows of 16 lanes
// then all hold the same problem and compute, and write, the same values; every per-problem loop runs once).
template <typename TIn, int PPW>
__global__ void __launch_bounds__(64, PPW == 4 ? 2 : 1) solve_small_kernel(const SolveArgs p) {
  constexpr int D = 16;
  using C = Cfg<D>;
  static_assert(PPW == 1 || PPW == 4, "one problem or four per wavefront");
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  __shared__ float s_red[C::NW];
  __shared__ __attribute__((aligned(16))) float s_x0[PPW][D];  // the problems' initial states, for the outputs
  const bool pure = (p.flags & TTC_FLAG_PURE_SYMPLECTIC) != 0;
  const long long nquads = (p.n + PPW - 1) / PPW;

  for (long long quad = blockIdx.x; quad < nquads; quad += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, i = lane & 15, g = lane >> 4;
    constexpr int w = 0;
    long long prob[PPW];  // a ragged last quad repeats the last problem; only valid ones are written out
    bool valid[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      valid[q] = quad * PPW + q < p.n;
      prob[q] = valid[q] ? quad * PPW + q : p.n - 1;
    }
    float* const Wmine = Wm[g & (PPW - 1)];  // the problem whose rows this lane holds during the dense solves
    int info[PPW] = {};
    int nsolve = 0;
    auto note = [&](int bad) {   // fold a dense solve's per-lane breakdown flags into the per-problem info
      ++nsolve;
      const unsigned long long m = __ballot(bad != 0);
#pragma unroll
      for (int q = 0; q < PPW; ++q)
        if (!info[q] && ((m >> (16 * q)) & 0xFFFFull)) info[q] = nsolve;
    };
    PhaseTimers tm;  // phases: 0 set-up, 1 dense solves, 2 steps, 3 outputs
    floatx4 acc[PPW][C::RB][C::NT];
    float cG[PPW][C::RB][C::KS], cAi[PPW][C::RB][C::KS], cAT[PPW][C::RB][C::KS], cQ[PPW][C::RB][C::KS];
    float cCK[PPW][C::RB][C::KS];

    // ---- phase R: X = R^{-1} B^T, G = B X
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      load_half<D, TIn, false>(Wm[q], reinterpret_cast<const TIn*>(p.R) + prob[q] * p.sR, tid);
      load_half<D, TIn, true>(Wm[q] + D, reinterpret_cast<const TIn*>(p.B) + prob[q] * p.sB, tid);  // RHS = B^T
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
    __syncthreads();
    {
      float cB[PPW][C::RB][C::KS], cX[PPW][C::RB][C::KS];
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aopT_lds<D>(Wm[q] + D, cB[q], w, i, g);  // rows of B = columns of B^T
      tm.toc(0);
      note(solve_rows16<false>(Wmine, lane));  // R is positive definite: no pivot search
      tm.toc(1);
#pragma unroll
      for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
      gemm_acc_quad<PPW>(acc, cB, Wm, D, i, g);  // rows of G = B X
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_aop_lds<D>(Wm[q] + D, cX[q], w, i, g);
        store_rows<D>(Wm[q], acc[q], w, i, g);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q], cG[q], w, i, g);
      __syncthreads();
      // ---- phase A: A^{-1}, A^T, Q, C_K = X A^{-T}
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_half<D, TIn, false>(Wm[q], reinterpret_cast<const TIn*>(p.A) + prob[q] * p.sA, tid);
        load_half<D, TIn, false>(Wm[q] + D, reinterpret_cast<const TIn*>(p.Q) + prob[q] * p.sQ, tid);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        symmetrise_half<D>(Wm[q] + D, tid);
        load_aopT_lds<D>(Wm[q], cAT[q], w, i, g);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q] + D, cQ[q], w, i, g);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) set_half_identity<D>(Wm[q] + D, tid);
      __syncthreads();
      tm.toc(0);
      note(solve_rows16<true>(Wmine, lane));
      tm.toc(1);
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_aop_lds<D>(Wm[q] + D, cAi[q], w, i, g);
        load_rows<D>(Wm[q] + D, acc[q], w, i, g);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows_T<D>(Wm[q] + D, acc[q], w, i, g);  // A^{-T}
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
      gemm_acc_quad<PPW>(acc, cX, Wm, D, i, g);  // rows of C_K = X A^{-T}
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q], cCK[q], w, i, g);
    }
    // initial pair [Y1 Y2] = [I Q_T]
    if (p.QT) {
#pragma unroll
      for (int q = 0; q < PPW; ++q)
        load_half<D, TIn, false>(Wm[q] + D, reinterpret_cast<const TIn*>(p.QT) + prob[q] * p.sQT, tid);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
    } else {
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_aop_lds<D>(Wm[q] + D, cQ[q], w, i, g);  // Q_T = Q, already symmetric
    }
    __syncthreads();

    tm.toc(0);
    // ---- groups of reverse symplectic steps, each ended by a re-base
    int s = 1;
    bool fresh = true;
    bool hard = false;  // the growth guard tripped
    int plan_base = 0, plan_T = p.T, plan_ng = p.ngroups;  // grouping of the steps after plan_base
    for (int grp = 0;; ++grp) {
      const int gend = plan_base + plan_T - (int)(((long long)(plan_ng - 1 - grp) * plan_T) / plan_ng);
      float g_prev = 1.f;  // max |Y1| before the step: a group starts from Y1 = I
      for (int k = 1;; ++s, ++k) {
        bool last = (s >= gend);
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          if (fresh) eye_acc<D>(acc[q], w, i, g); else load_rows<D>(Wm[q], acc[q], w, i, g);
        }
        gemm_acc_quad<PPW>(acc, cG, Wm, D, i, g);   // Z1 + G Z2
#pragma unroll
        for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
        gemm_acc_quad<PPW>(acc, cAi, Wm, 0, i, g);  // A^{-1} (.) = new Z1
        if (p.growth_limit > 0.f) {
          // Growth guard (see solve_kernel): max |Y1| over the wavefront's problems.  A group about to pass the
          // limit ends with this step and the rest of the horizon is re-planned with groups no longer than it;
          // beyond the limit all the wavefront's problems leave the symplectic iteration for the recursion of
          // Prop. 3.1 in its printed form (below).
          uint32_t m = 0;
#pragma unroll
          for (int q = 0; q < PPW; ++q) {
            if (info[q]) continue;  // a problem whose set-up broke down is NaN anyway and keeps its report
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const uint32_t b = __float_as_uint(acc[q][0][0][v]) & 0x7FFFFFFFu;
              m = b > m ? b : m;
            }
          }
          const float gm = __uint_as_float(wave_max_u32(m));
          if (!(gm <= p.growth_limit)) {  // wave-uniform; also true for NaN
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
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
        gemm_acc_quad<PPW>(acc, cAT, Wm, D, i, g);              // A^T Z2
        if (s < p.T) gemm_acc_quad<PPW>(acc, cQ, Wm, 0, i, g);  // + Q Z1; Q_0 = 0 for the last factor
        __syncthreads();
        fresh = false;
        if (!last) {
#pragma unroll
          for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q] + D, acc[q], w, i, g);
          __syncthreads();
          if (pure) {
#pragma unroll
            for (int q = 0; q < PPW; ++q) normalise_rows_zland<D>(Wm[q], tid);
            __syncthreads();
          }
        } else {
          // leave Z-land: [Y1 | Y2] untransposed for the solve Y1 P = Y2
          floatx4 z1[PPW][C::RB][C::NT];
#pragma unroll
          for (int q = 0; q < PPW; ++q) {
            store_rows_T<D>(Wm[q] + D, acc[q], w, i, g);
            load_rows<D>(Wm[q], z1[q], w, i, g);
          }
          __syncthreads();
#pragma unroll
          for (int q = 0; q < PPW; ++q) store_rows_T<D>(Wm[q], z1[q], w, i, g);
          __syncthreads();
          ++s;
          break;
        }
      }
      if (hard) break;
      tm.toc(2);
      note(solve_rows16<true>(Wmine, lane));
      tm.toc(1);
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
      __syncthreads();
      fresh = true;
      if (s > p.T) break;
    }
    if (hard) {
      // Prop. 3.1 as printed, from P_T, for the wavefront's problems (what ttc_lqr_solve_tv runs, here with the same
      // matrices in every step).  A problem whose set-up broke down keeps that report.
      __syncthreads();
      const TIn *Ap[PPW], *Bp[PPW], *Qp[PPW], *Rp[PPW], *PTp[PPW];
      bool keep[PPW];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        Ap[q] = reinterpret_cast<const TIn*>(p.A) + prob[q] * p.sA;
        Bp[q] = reinterpret_cast<const TIn*>(p.B) + prob[q] * p.sB;
        Qp[q] = reinterpret_cast<const TIn*>(p.Q) + prob[q] * p.sQ;
        Rp[q] = reinterpret_cast<const TIn*>(p.R) + prob[q] * p.sR;
        PTp[q] = p.QT ? reinterpret_cast<const TIn*>(p.QT) + prob[q] * p.sQT : Qp[q];
        keep[q] = valid[q] && !info[q];
      }
      riccati_quad<TIn, PPW>(Wm, s_red, p, prob, keep, p.T, Ap, Bp, Qp, Rp, PTp, 0, 0, 0, 0, 2, tid + opaque_zero());
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if (!(valid[q] && info[q])) continue;  // set-up breakdown: NaN outputs and its own code
        const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob[q] * p.sx0;
        zero_acc<D>(acc[q]);
        emit_gain<D, TIn>(p, prob[q], acc[q], x0p, info[q], tid);
        emit_value<D, TIn>(p, prob[q], Wm[q] + D, Qp[q], x0p, info[q], s_red, tid);
      }
      __syncthreads();
      continue;
    }

    tm.toc(2);
    // ---- outputs: the right halves hold P_0 (paper convention, Q_0 = 0)
    if (p.flags & TTC_FLAG_STAGE_COST_AT_X0) {  // P_0 + Q is assembled problem by problem
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if (!valid[q]) continue;  // uniform over the wavefront
        const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob[q] * p.sQ;
        const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob[q] * p.sx0;
        zero_acc<D>(acc[q]);
        gemm_acc<D>(acc[q], cCK[q], Wm[q] + D, i, g);  // -K_0 = C_K P_0
        emit_gain<D, TIn>(p, prob[q], acc[q], x0p, info[q], tid);
        emit_value<D, TIn>(p, prob[q], Wm[q] + D, Qp, x0p, info[q], s_red, tid);
      }
      __syncthreads();
    } else {
      // All the wavefront's problems at once: -K_0 = C_K P_0 on the matrix cores, K_0 to the left halves, then lane
      // (i, g) takes row i of its problem's K_0 and P_0 for u_0 = K_0 x_0 and value = x_0^T P_0 x_0; the matrices
      // leave as one 16-byte piece per lane and problem.
      const int gq = g & (PPW - 1);
      const long long pg = (quad * PPW + gq < p.n) ? quad * PPW + gq : p.n - 1;
      const float x0_m = ld1<TIn>(reinterpret_cast<const TIn*>(p.x0), pg * p.sx0 + i);
#pragma unroll
      for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
      gemm_acc_quad<PPW>(acc, cCK, Wm, D, i, g);
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[q][0][0][v] = -acc[q][0][0][v];
        store_rows<D>(Wm[q], acc[q], w, i, g);  // left halves: K_0, row-major
      }
      s_x0[gq][i] = x0_m;
      __syncthreads();
      const float nanv = __builtin_nanf("");
      float u = 0.f, pw = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const floatx4 kr = *reinterpret_cast<const floatx4*>(Wm[gq] + i * C::PITCH + 4 * c);
        const floatx4 pr = *reinterpret_cast<const floatx4*>(Wm[gq] + D + i * C::PITCH + 4 * c);
        const floatx4 xr = *reinterpret_cast<const floatx4*>(&s_x0[gq][4 * c]);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          u = __builtin_fmaf(kr[v], xr[v], u);
          pw = __builtin_fmaf(pr[v], xr[v], pw);
        }
      }
      const float val = sum16(x0_m * pw);
      int myinfo = info[0];
#pragma unroll
      for (int q = 1; q < PPW; ++q) myinfo = (gq == q) ? info[q] : myinfo;
      if (quad * PPW + gq < p.n && (PPW == 4 || g == 0)) {
        p.u0[pg * D + i] = myinfo ? nanv : u;
        if (i == 0) {
          if (p.value) p.value[pg] = myinfo ? nanv : val;
          if (p.info) p.info[pg] = myinfo;
        }
      }
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if (!valid[q]) continue;  // uniform over the wavefront
        const floatx4 nan4 = floatx4{nanv, nanv, nanv, nanv};
        if (p.K0)
          *reinterpret_cast<floatx4*>(p.K0 + prob[q] * (long)D * D + 4 * lane) =
              info[q] ? nan4 : *reinterpret_cast<const floatx4*>(Wm[q] + (lane >> 2) * C::PITCH + 4 * (lane & 3));
        if (p.P0)
          *reinterpret_cast<floatx4*>(p.P0 + prob[q] * (long)D * D + 4 * lane) =
              info[q] ? nan4 : *reinterpret_cast<const floatx4*>(Wm[q] + D + (lane >> 2) * C::PITCH + 4 * (lane & 3));
      }
      __syncthreads();
    }
    tm.toc(3);
    tm.dump(p);
  }
}

}  // namespace ttc
