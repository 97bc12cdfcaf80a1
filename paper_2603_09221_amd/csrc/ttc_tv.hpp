// Time-heterogeneous problems: A_t, B_t, Q_t, R_t vary over the horizon (the general statement of
// Prop. 3.1; the paper's "time-heterogeneous parameterization", Sec. 4).
// Included by ttc_lqr.hip after the helpers it shares with the other kernels.
//
// With every factor Sigma_t of Thm 3.3 different, nothing can be prepared once per problem, and each
// factor would need its own A_t^{-1}.  The kernel therefore re-bases after every factor, which turns a
// factor into one backward Riccati step in Moebius form and needs no A_t^{-1}:
//     X_s = R_s^{-1} B_s^T,  G_s = B_s X_s,
//     M_s = (I + P_{s+1} G_s)^{-1} P_{s+1} A_s,   P_s = Q[s-1] + A_s^T M_s   (P_T = Q[T-1], no Q on x_0),
//     K_0 = -X_0 M_0                                                         (Eq. "decode").
// Two dense solves and four products per step; the value matrix stays on chip for the whole horizon
// (in LDS as the right operand of the products, in registers while the pair serves the R_s solve),
// the step's matrices are streamed from HBM once each.
#pragma once

namespace ttc {

struct TvArgs {
  SolveArgs s;                 // n, T, A, B, Q, R, x0 and their problem strides, outputs (QT, ws, groups unused)
  long long tA, tB, tQ, tR;    // elements between consecutive steps
};

template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) solve_tv_kernel(const TvArgs ta) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  const SolveArgs& p = ta.s;
  float* const WL = W;
  float* const WR = W + D;

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    int info = 0, nsolve = 0;
    float cX[C::RB][C::KS];  // rows of X_0, for the gain

    {
      const int tid = threadIdx.x + opaque_zero();
      load_half<D, TIn, false>(WR, Qp + (long long)(p.T - 1) * ta.tQ, tid);  // P_T = Q_T
      __syncthreads();
      symmetrise_half<D>(WR, tid);
      __syncthreads();
    }
    for (int s = p.T - 1; s >= 0; --s) {
      // (address arithmetic local to the step: see opaque_zero)
      const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
      floatx4 acc[C::RB][C::NT];
      float cG[C::RB][C::KS], cAT[C::RB][C::KS];
      {
        floatx4 preg[C::RB][C::NT];
        load_rows<D>(WR, preg, w, i, g);  // P_{s+1} waits in registers while the pair serves the R_s solve
        __syncthreads();
        load_half<D, TIn, false>(WL, Rp + (long long)s * ta.tR, tid);
        load_half<D, TIn, true>(WR, Bp + (long long)s * ta.tB, tid);  // RHS = B_s^T
        __syncthreads();
        symmetrise_half<D>(WL, tid);
        float cB[C::RB][C::KS];
        load_aopT_lds<D>(WR, cB, w, i, g);  // rows of B_s = columns of B_s^T
        __syncthreads();
        ++nsolve;
        if (lds_solve<D, 7, false>(W, S, tid) && !info) info = nsolve;  // R_s is positive definite: no pivot search
        zero_acc<D>(acc);
        gemm_acc<D>(acc, cB, WR, i, g);  // rows of G_s = B_s X_s
        if (s == 0) load_aop_lds<D>(WR, cX, w, i, g);
        store_rows<D>(WL, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WL, tid);
        __syncthreads();
        load_aop_lds<D>(WL, cG, w, i, g);
        __syncthreads();
        store_rows<D>(WR, preg, w, i, g);  // P_{s+1} back as the right operand
      }
      load_half<D, TIn, false>(WL, Ap + (long long)s * ta.tA, tid);
      __syncthreads();
      load_aopT_lds<D>(WL, cAT, w, i, g);  // rows of A_s^T
      __syncthreads();
      eye_acc<D>(acc, w, i, g);
      gemm_acc<D>(acc, cG, WR, i, g);      // I + G_s P = (I + P G_s)^T
      store_rows_T<D>(WL, acc, w, i, g);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cAT, WR, i, g);     // A_s^T P = (P A_s)^T
      __syncthreads();
      store_rows_T<D>(WR, acc, w, i, g);
      __syncthreads();
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;  // right half: M_s
      if (s >= 1) {
        load_half<D, TIn, false>(WL, Qp + (long long)(s - 1) * ta.tQ, tid);  // the cost on x_s
        __syncthreads();
        symmetrise_half<D>(WL, tid);
        __syncthreads();
        load_rows<D>(WL, acc, w, i, g);
        gemm_acc<D>(acc, cAT, WR, i, g);   // P_s = Q[s-1] + A_s^T M_s
        __syncthreads();
        store_rows<D>(WR, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WR, tid);
        __syncthreads();
      } else {
        zero_acc<D>(acc);
        gemm_acc<D>(acc, cAT, WR, i, g);   // P_0 = A_0^T M_0
        store_rows<D>(WL, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WL, tid);
        __syncthreads();
        zero_acc<D>(acc);
        gemm_acc<D>(acc, cX, WR, i, g);    // -K_0 = X_0 M_0
        emit_gain<D, TIn>(p, prob, acc, x0p, info, tid);
        emit_value<D, TIn>(p, prob, WL, Qp, x0p, info, s_red, tid);
      }
    }
  }
}

struct TvRolloutArgs {
  RolloutArgs r;               // n, T, A, B, Q, R, x0 and their problem strides, U, X, cost, info, ws (QT unused)
  long long tA, tB, tQ, tR;    // elements between consecutive steps
};

// Roll-out of a time-heterogeneous problem (Alg. 1 with r = 0): the backward sweep of solve_tv_kernel
// keeping every gain K_s = -X_s M_s in the workspace, then the closed-loop forward sweep
// u_s = K_s x_s, x_{s+1} = A_s x_s + B_s u_s with the cost sum_s u_s^T R_s u_s + x_{s+1}^T Q[s] x_{s+1}.
template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) rollout_tv_kernel(const TvRolloutArgs ta) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  __shared__ float s_x[D], s_u[D], s_xn[D];
  const RolloutArgs& p = ta.r;
  float* const WL = W;
  float* const WR = W + D;
  float* const wsK = p.ws + (long)blockIdx.x * p.T * D * D;  // K_0 .. K_{T-1}, row-major

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    int info = 0, nsolve = 0;
    {
      const int tid = threadIdx.x + opaque_zero();
      load_half<D, TIn, false>(WR, Qp + (long long)(p.T - 1) * ta.tQ, tid);  // P_T = Q_T
      __syncthreads();
      symmetrise_half<D>(WR, tid);
      __syncthreads();
    }
    // ---- backward sweep
    for (int s = p.T - 1; s >= 0; --s) {
      const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
      floatx4 acc[C::RB][C::NT];
      float cG[C::RB][C::KS], cAT[C::RB][C::KS], cX[C::RB][C::KS];
      {
        floatx4 preg[C::RB][C::NT];
        load_rows<D>(WR, preg, w, i, g);
        __syncthreads();
        load_half<D, TIn, false>(WL, Rp + (long long)s * ta.tR, tid);
        load_half<D, TIn, true>(WR, Bp + (long long)s * ta.tB, tid);
        __syncthreads();
        symmetrise_half<D>(WL, tid);
        float cB[C::RB][C::KS];
        load_aopT_lds<D>(WR, cB, w, i, g);
        __syncthreads();
        ++nsolve;
        if (lds_solve<D, 7, false>(W, S, tid) && !info) info = nsolve;
        zero_acc<D>(acc);
        gemm_acc<D>(acc, cB, WR, i, g);  // rows of G_s
        load_aop_lds<D>(WR, cX, w, i, g);  // rows of X_s, for the gain
        store_rows<D>(WL, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WL, tid);
        __syncthreads();
        load_aop_lds<D>(WL, cG, w, i, g);
        __syncthreads();
        store_rows<D>(WR, preg, w, i, g);
      }
      load_half<D, TIn, false>(WL, Ap + (long long)s * ta.tA, tid);
      __syncthreads();
      load_aopT_lds<D>(WL, cAT, w, i, g);
      __syncthreads();
      eye_acc<D>(acc, w, i, g);
      gemm_acc<D>(acc, cG, WR, i, g);
      store_rows_T<D>(WL, acc, w, i, g);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cAT, WR, i, g);
      __syncthreads();
      store_rows_T<D>(WR, acc, w, i, g);
      __syncthreads();
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;  // right half: M_s
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cX, WR, i, g);  // -K_s
#pragma unroll
      for (int rb = 0; rb < C::RB; ++rb) {
#pragma unroll
        for (int cc = 0; cc < C::NT; ++cc) acc[rb][cc] = -acc[rb][cc];
        write_rows_global<D>(wsK + (long)s * D * D, acc[rb], C::RB * w + rb, i, g);
      }
      if (s >= 1) {
        load_half<D, TIn, false>(WL, Qp + (long long)(s - 1) * ta.tQ, tid);
        __syncthreads();
        symmetrise_half<D>(WL, tid);
        __syncthreads();
        load_rows<D>(WL, acc, w, i, g);
        gemm_acc<D>(acc, cAT, WR, i, g);  // P_s
        __syncthreads();
        store_rows<D>(WR, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WR, tid);
        __syncthreads();
      }
    }
    __syncthreads();  // gains visible to the whole workgroup

    // ---- forward sweep
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = tid / (C::NTHR / D), part = tid % (C::NTHR / D);
    if (tid < D) s_x[tid] = ld1<TIn>(x0p, tid);
    __syncthreads();
    float cpart = 0.f;
    if (p.X && tid < D) p.X[prob * (long)(p.T + 1) * D + tid] = s_x[tid];
    for (int t = 0; t < p.T; ++t) {
      const float u = matvec_row<D, float>(wsK + (long)t * D * D, s_x, tid);
      if (part == 0) s_u[r] = u;
      __syncthreads();
      const float ru = matvec_row<D, TIn>(Rp + (long long)t * ta.tR, s_u, tid);
      const float xn = matvec_row<D, TIn>(Ap + (long long)t * ta.tA, s_x, tid) +
                       matvec_row<D, TIn>(Bp + (long long)t * ta.tB, s_u, tid);
      if (part == 0) {
        cpart += s_u[r] * ru;
        s_xn[r] = xn;
        p.U[(prob * p.T + t) * (long)D + r] = info ? __builtin_nanf("") : u;
      }
      __syncthreads();
      const float qx = matvec_row<D, TIn>(Qp + (long long)t * ta.tQ, s_xn, tid);
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

// The same at d = 16 with four problems per wavefront (see ttc_small.hpp): products of the four problems
// interleaved on the matrix cores, their dense solves side by side with one row per lane.
template <typename TIn>
__global__ void __launch_bounds__(64) solve_tv_small_kernel(const TvArgs ta) {
  constexpr int D = 16;
  using C = Cfg<D>;
  constexpr int PPW = 4;
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  __shared__ float s_red[C::NW];
  const SolveArgs& p = ta.s;
  const long long nquads = (p.n + PPW - 1) / PPW;

  for (long long quad = blockIdx.x; quad < nquads; quad += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, i = lane & 15, g = lane >> 4;
    constexpr int w = 0;
    long long prob[PPW];  // a ragged last quad repeats the last problem; only valid ones are written out
    bool valid[PPW];
    const TIn *Ap[PPW], *Bp[PPW], *Qp[PPW], *Rp[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      valid[q] = quad * PPW + q < p.n;
      prob[q] = valid[q] ? quad * PPW + q : p.n - 1;
      Ap[q] = reinterpret_cast<const TIn*>(p.A) + prob[q] * p.sA;
      Bp[q] = reinterpret_cast<const TIn*>(p.B) + prob[q] * p.sB;
      Qp[q] = reinterpret_cast<const TIn*>(p.Q) + prob[q] * p.sQ;
      Rp[q] = reinterpret_cast<const TIn*>(p.R) + prob[q] * p.sR;
    }
    float* const Wmine = Wm[g];  // the problem whose rows this lane holds during the dense solves
    int info[PPW] = {0, 0, 0, 0};
    int nsolve = 0;
    auto note = [&](int bad) {
      ++nsolve;
      const unsigned long long m = __ballot(bad != 0);
#pragma unroll
      for (int q = 0; q < PPW; ++q)
        if (!info[q] && ((m >> (16 * q)) & 0xFFFFull)) info[q] = nsolve;
    };
    floatx4 acc[PPW][C::RB][C::NT];
    float cX[PPW][C::RB][C::KS];

#pragma unroll
    for (int q = 0; q < PPW; ++q) load_half<D, TIn, false>(Wm[q] + D, Qp[q] + (long long)(p.T - 1) * ta.tQ, tid);  // P_T = Q_T
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
    __syncthreads();
    for (int s = p.T - 1; s >= 0; --s) {
      float cG[PPW][C::RB][C::KS], cAT[PPW][C::RB][C::KS];
      {
        floatx4 preg[PPW][C::RB][C::NT];
        float cB[PPW][C::RB][C::KS];
#pragma unroll
        for (int q = 0; q < PPW; ++q) load_rows<D>(Wm[q] + D, preg[q], w, i, g);  // P_{s+1} waits in registers
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          load_half<D, TIn, false>(Wm[q], Rp[q] + (long long)s * ta.tR, tid);
          load_half<D, TIn, true>(Wm[q] + D, Bp[q] + (long long)s * ta.tB, tid);  // RHS = B_s^T
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          symmetrise_half<D>(Wm[q], tid);
          load_aopT_lds<D>(Wm[q] + D, cB[q], w, i, g);
        }
        __syncthreads();
        note(solve_rows16<false>(Wmine, lane));  // R_s is positive definite: no pivot search
#pragma unroll
        for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
        gemm_acc_quad(acc, cB, Wm, D, i, g);  // rows of G_s = B_s X_s
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          if (s == 0) load_aop_lds<D>(Wm[q] + D, cX[q], w, i, g);
          store_rows<D>(Wm[q], acc[q], w, i, g);
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q], cG[q], w, i, g);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          store_rows<D>(Wm[q] + D, preg[q], w, i, g);  // P_{s+1} back as the right operand
          load_half<D, TIn, false>(Wm[q], Ap[q] + (long long)s * ta.tA, tid);
        }
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aopT_lds<D>(Wm[q], cAT[q], w, i, g);  // rows of A_s^T
      __syncthreads();
      {
        floatx4 acc2[PPW][C::RB][C::NT];
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          eye_acc<D>(acc[q], w, i, g);
          zero_acc<D>(acc2[q]);
        }
        gemm_acc_quad(acc, cG, Wm, D, i, g);    // I + G_s P = (I + P G_s)^T
        gemm_acc_quad(acc2, cAT, Wm, D, i, g);  // A_s^T P = (P A_s)^T
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          store_rows_T<D>(Wm[q], acc[q], w, i, g);
          store_rows_T<D>(Wm[q] + D, acc2[q], w, i, g);
        }
      }
      __syncthreads();
      note(solve_rows16<true>(Wmine, lane));  // right halves: M_s
      if (s >= 1) {
#pragma unroll
        for (int q = 0; q < PPW; ++q) load_half<D, TIn, false>(Wm[q], Qp[q] + (long long)(s - 1) * ta.tQ, tid);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) load_rows<D>(Wm[q], acc[q], w, i, g);
        gemm_acc_quad(acc, cAT, Wm, D, i, g);  // P_s = Q[s-1] + A_s^T M_s
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q] + D, acc[q], w, i, g);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
        __syncthreads();
      } else {
#pragma unroll
        for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
        gemm_acc_quad(acc, cAT, Wm, D, i, g);  // P_0 = A_0^T M_0
#pragma unroll
        for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
        gemm_acc_quad(acc, cX, Wm, D, i, g);   // -K_0 = X_0 M_0
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          if (!valid[q]) continue;  // uniform over the wavefront
          const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob[q] * p.sx0;
          emit_gain<D, TIn>(p, prob[q], acc[q], x0p, info[q], tid);
          emit_value<D, TIn>(p, prob[q], Wm[q], Qp[q], x0p, info[q], s_red, tid);
        }
        __syncthreads();
      }
    }
  }
}

}  // namespace ttc
