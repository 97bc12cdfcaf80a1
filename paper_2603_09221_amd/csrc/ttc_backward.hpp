// Backward pass of the layer (Thm 3.2; appendix: Thm A.6): gradients of a loss of the output u_0 = u_1^* with
// respect to A_t, B_t, Q_t, R_t and the initial state, from dl/du_0.
//
// The gradients are outer products of two KKT solutions (states, controls, co-states): the layer's own problem
// (the "primal LQR") and the "dual LQR", the same dynamics and quadratic costs from the initial state 0 with the
// linear cost g^T ut_0 on the first control, g = dl/du_0.  Its affine terms (Prop. A.1) vanish after the first
// step, so the dual trajectory is the closed loop of the same gains started from ut_0 = -S_0^{-1} g:
//     ut_0 = -S_0^{-1} g,  xt_1 = B_0 ut_0,  ut_s = K_s xt_s,  xt_{s+1} = A_s xt_s + B_s ut_s      (s >= 1)
// beside the primal   u_0 = -S_0^{-1} (B_0^T P_1 A_0 x_0),  u_s = K_s x_s,  x_{s+1} = A_s x_s + B_s u_s,
// with S_0 = R_0 + B_0^T P_1 B_0.  Co-states by the recursion of Alg. 2 for both: lam_T = Q[T-1] x_T,
// lam_t = Q[t-1] x_t + A_t^T lam_{t+1}, and dl/dx_0 = lamt_0 = A_0^T lamt_1.  Then, per step s (the paper's t = s+1),
//     dl/dA_s = lam_{s+1} xt_s^T + lamt_{s+1} x_s^T          dl/dB_s = lam_{s+1} ut_s^T + lamt_{s+1} u_s^T
//     dl/dQ[s] = sym(xt_{s+1} x_{s+1}^T)                     dl/dR_s = sym(ut_s u_s^T).
// The paper's kernel (Alg. 5) runs the forward symplectic recursion from cached lam_0, LU(Y1) and Y3; that
// recursion multiplies by A_t^{-T} every step and loses all accuracy in float32 on dense problems, and caching the
// gains of the forward pass would cost T d^2 floats per problem.  Here the backward pass is self-contained: it
// repeats the backward recursion of Prop. 3.1 (the code of ttc_lqr_solve_tv), keeps the gains of the problem in
// flight in its workgroup's workspace slot, and rolls both closed loops forward.
//
// One workgroup per problem.  Workspace slot of a workgroup: K_1 .. K_{T-1} (d^2 floats each, slot s at
// (s-1) d^2) and six trajectories of (T+1) d floats: X, U, Xt, Ut, LAM, LAMt.
#pragma once
#include "ttc_common.hpp"
#include "ttc_rollout.hpp"
#include "ttc_tv.hpp"

namespace ttc {

// y[j] = sum_r M[r][j] x[r] (the transposed product) for a row-major global d x d matrix: thread (part, j) sums its
// share of the rows (consecutive threads read consecutive columns), the parts are added through LDS (red: TPR x D
// floats).  Contains two barriers; every thread gets y[tid % D].
template <int D, typename TM>
__device__ __forceinline__ float matvecT_row(const TM* M, const float* xs, float* red, int tid) {
  constexpr int TPR = Cfg<D>::NTHR / D;
  const int j = tid % D, part = tid / D;
  float s = 0.f;
#pragma unroll 8
  for (int r = part * (D / TPR); r < (part + 1) * (D / TPR); ++r) s += ld1<TM>(M, (long)r * D + j) * xs[r];
  red[part * D + j] = s;
  __syncthreads();
  float y = 0.f;
#pragma unroll
  for (int q = 0; q < TPR; ++q) y += red[q * D + j];
  __syncthreads();
  return y;
}

// the same products with the matrix in one half of the LDS pair (row r at Wh + r*PITCH)
template <int D>
__device__ __forceinline__ float matvec_lds(const float* Wh, const float* xs, int tid) {
  using C = Cfg<D>;
  constexpr int TPR = C::NTHR / D;
  const int r = tid / TPR, part = tid % TPR;
  float s = 0.f;
#pragma unroll
  for (int c4 = part * (D / TPR); c4 < (part + 1) * (D / TPR); c4 += 4) {
    const floatx4 mv = *reinterpret_cast<const floatx4*>(Wh + r * C::PITCH + c4);
    s += mv[0] * xs[c4] + mv[1] * xs[c4 + 1] + mv[2] * xs[c4 + 2] + mv[3] * xs[c4 + 3];
  }
#pragma unroll
  for (int m = 1; m < TPR; m <<= 1) s += __shfl_xor(s, m, 64);
  return s;
}
template <int D>
__device__ __forceinline__ float matvecT_lds(const float* Wh, const float* xs, float* red, int tid) {
  using C = Cfg<D>;
  constexpr int TPR = C::NTHR / D;
  const int j = tid % D, part = tid / D;
  float s = 0.f;
#pragma unroll 8
  for (int r = part * (D / TPR); r < (part + 1) * (D / TPR); ++r) s += Wh[r * C::PITCH + j] * xs[r];
  red[part * D + j] = s;
  __syncthreads();
  float y = 0.f;
#pragma unroll
  for (int q = 0; q < TPR; ++q) y += red[q * D + j];
  __syncthreads();
  return y;
}

// out (d x d, row-major, global) = or += a b^T + c e^T, vectors in LDS; each thread a share of the 16-byte pieces
template <int D, bool ACCUMULATE>
__device__ __forceinline__ void outer2_global(float* out, const float* a, const float* b, const float* c, const float* e,
                                              float scale, int tid) {
  using C = Cfg<D>;
  for (int idx = tid; idx < D * D / 4; idx += C::NTHR) {
    const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
    const float ar = scale * a[r], cr = scale * c[r];
    floatx4 v;
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = ar * b[c4 + k] + cr * e[c4 + k];
    floatx4* dst = reinterpret_cast<floatx4*>(out + (long)r * D + c4);
    if (ACCUMULATE) v += *dst;
    *dst = v;
  }
}

template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) backward_kernel(const BackwardArgs ba) {
  using C = Cfg<D>;
  constexpr int TPR = C::NTHR / D;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[TPR * D];
  __shared__ float s_v[8][D];  // working vectors
  const RolloutArgs& p = ba.r;
  float* const WL = W;
  float* const WR = W + D;
  const int T = p.T;
  float* const wsK = p.ws + (long)blockIdx.x * ((long)(T - 1) * D * D + 6L * (T + 1) * D);  // K_1 .. K_{T-1}
  float* const traj = wsK + (long)(T - 1) * D * D;
  float* const tX = traj;                                // (T+1) x d each
  float* const tU = traj + 1L * (T + 1) * D;
  float* const tXt = traj + 2L * (T + 1) * D;
  float* const tUt = traj + 3L * (T + 1) * D;
  float* const tL = traj + 4L * (T + 1) * D;
  float* const tLt = traj + 5L * (T + 1) * D;
  const float nanv = __builtin_nanf("");

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    // the terminal cost: a separate matrix for time-invariant problems that give one, else Q of the last step
    const TIn* QTp = p.QT ? reinterpret_cast<const TIn*>(p.QT) + prob * p.sQT : Qp + (long long)(T - 1) * ba.tQ;
    auto stage_cost = [&](int s) { return (s == T - 1) ? QTp : Qp + (long long)s * ba.tQ; };  // the cost on x_{s+1}
    const float* gp = ba.g + prob * ba.sg;
    int info = 0;

    // ---- backward recursion (Prop. 3.1): gains K_{T-1} .. K_1 to the workspace, P_1 left in the right half
    load_half<D, TIn, false>(WR, QTp, tid);
    __syncthreads();
    symmetrise_half<D>(WR, tid);
    __syncthreads();
    for (int s = T - 1; s >= 1; --s) {
      floatx4 pn[C::RB][C::NT];
      const int flag = riccati_step<D, TIn>(W, S, Ap + (long long)s * ba.tA, Bp + (long long)s * ba.tB,
                                            Rp + (long long)s * ba.tR, pn, tid);
      if (flag && !info) info = T - s;
      {
        floatx4 acc[C::RB][C::NT];
        load_rows<D>(WR, acc, w, i, g);
#pragma unroll
        for (int rb = 0; rb < C::RB; ++rb) {
#pragma unroll
          for (int cc = 0; cc < C::NT; ++cc) acc[rb][cc] = -acc[rb][cc];
          write_rows_global<D>(wsK + (long)(s - 1) * D * D, acc[rb], C::RB * w + rb, i, g);  // K_s
        }
      }
      __syncthreads();
      next_value_matrix<D, TIn>(W, stage_cost(s - 1), pn, tid);
    }

    // ---- step 0: S_0 = R_0 + B_0^T P_1 B_0 and the two right-hand sides F x_0 = B_0^T P_1 A_0 x_0 and g
    float* const v_x = s_v[0];
    float* const v_y = s_v[1];
    float* const v_z = s_v[2];
    float* const v_u = s_v[3];
    float* const v_ut = s_v[4];
    float* const v_xt = s_v[5];
    if (tid < D) v_x[tid] = ld1<TIn>(x0p, tid);
    __syncthreads();
    {
      const float y = matvec_row<D, TIn>(Ap, v_x, tid);  // A_0 x_0
      if (tid % TPR == 0) v_y[tid / TPR] = y;
    }
    __syncthreads();
    {
      const float z = matvec_lds<D>(WR, v_y, tid);  // P_1 A_0 x_0
      if (tid % TPR == 0) v_z[tid / TPR] = z;
    }
    __syncthreads();
    {
      float cP[C::RB][C::KS], cBT[C::RB][C::KS];
      floatx4 acc[C::RB][C::NT];
      load_aop_lds<D>(WR, cP, w, i, g);  // rows of P_1
      load_half<D, TIn, false>(WL, Bp, tid);
      __syncthreads();
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cP, WL, i, g);  // P_1 B_0
      load_aopT_lds<D>(WL, cBT, w, i, g);  // rows of B_0^T
      const float fx = matvecT_lds<D>(WL, v_z, s_red, tid);  // B_0^T P_1 A_0 x_0 (contains barriers)
      store_rows<D>(WR, acc, w, i, g);  // right half: P_1 B_0 (every wavefront holds its rows of P_1)
      __syncthreads();
      load_rows_input<D, TIn>(Rp, acc, w, i, g);
      gemm_acc<D>(acc, cBT, WR, i, g);  // S_0 = R_0 + B_0^T P_1 B_0
      __syncthreads();
      store_rows<D>(WL, acc, w, i, g);
      // right-hand sides: column 0 = F x_0, column 1 = g, the other columns zero
      for (int idx = tid; idx < D * D / 4; idx += C::NTHR) {
        const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
        *reinterpret_cast<floatx4*>(WR + r * C::PITCH + c4) = floatx4{0.f, 0.f, 0.f, 0.f};
      }
      __syncthreads();
      if (tid < D) {
        WR[tid * C::PITCH + 0] = fx;
        WR[tid * C::PITCH + 1] = gp[tid];
      }
      __syncthreads();
    }
    symmetrise_half<D>(WL, tid);  // R is read as its symmetric part
    __syncthreads();
    {
      const int flag = lds_solve<D, 7, false>(W, S, tid);
      if (flag && !info) info = T;
    }
    if (tid < D) {
      const float u = -WR[tid * C::PITCH + 0], ut = -WR[tid * C::PITCH + 1];
      v_u[tid] = u;
      v_ut[tid] = ut;
      v_xt[tid] = 0.f;
      tX[tid] = v_x[tid];
      tXt[tid] = 0.f;
    }
    __syncthreads();

    // ---- both closed loops forward (Alg. 1): states and controls of every step to the workspace
    for (int s = 0; s < T; ++s) {
      const TIn* As = Ap + (long long)s * ba.tA;
      const TIn* Bs = Bp + (long long)s * ba.tB;
      if (s >= 1) {
        const float* Ks = wsK + (long)(s - 1) * D * D;
        const float u = matvec_row<D, float>(Ks, v_x, tid);
        const float ut = matvec_row<D, float>(Ks, v_xt, tid);
        if (tid % TPR == 0) {
          v_u[tid / TPR] = u;
          v_ut[tid / TPR] = ut;
        }
        __syncthreads();
      }
      const float xn = matvec_row<D, TIn>(As, v_x, tid) + matvec_row<D, TIn>(Bs, v_u, tid);
      const float xtn = matvec_row<D, TIn>(As, v_xt, tid) + matvec_row<D, TIn>(Bs, v_ut, tid);
      if (tid < D) {
        tU[(long)s * D + tid] = v_u[tid];
        tUt[(long)s * D + tid] = v_ut[tid];
      }
      __syncthreads();  // every thread has read the old states
      if (tid % TPR == 0) {
        const int r = tid / TPR;
        v_x[r] = xn;
        v_xt[r] = xtn;
        tX[(long)(s + 1) * D + r] = xn;
        tXt[(long)(s + 1) * D + r] = xtn;
      }
      __syncthreads();
    }

    // ---- co-states backward (Alg. 2), for both trajectories; dl/dx_0 = lamt_0
    float* const v_l = s_v[6];
    float* const v_lt = s_v[7];
    {
      const float l = matvec_row<D, TIn>(stage_cost(T - 1), v_x, tid);  // lam_T = Q_T x_T (Q read as its symmetric
      const float lT = matvecT_row<D, TIn>(stage_cost(T - 1), v_x, s_red, tid);  // part: half of Q x + Q^T x)
      const float lt = matvec_row<D, TIn>(stage_cost(T - 1), v_xt, tid);
      const float ltT = matvecT_row<D, TIn>(stage_cost(T - 1), v_xt, s_red, tid);
      if (tid % TPR == 0) {
        v_y[tid / TPR] = 0.5f * l;
        v_z[tid / TPR] = 0.5f * lt;
      }
      __syncthreads();
      if (tid < D) {
        v_l[tid] = v_y[tid] + 0.5f * lT;
        v_lt[tid] = v_z[tid] + 0.5f * ltT;
        tL[(long)T * D + tid] = v_l[tid];
        tLt[(long)T * D + tid] = v_lt[tid];
      }
      __syncthreads();
    }
    for (int t = T - 1; t >= 0; --t) {
      // lam_t = Q[t-1] x_t + A_t^T lam_{t+1} (no state cost for t = 0)
      const TIn* At = Ap + (long long)t * ba.tA;
      float al = matvecT_row<D, TIn>(At, v_l, s_red, tid);
      float alt = matvecT_row<D, TIn>(At, v_lt, s_red, tid);
      if (t >= 1) {
        if (tid < D) {
          v_x[tid] = tX[(long)t * D + tid];
          v_xt[tid] = tXt[(long)t * D + tid];
        }
        __syncthreads();
        const TIn* Qt = stage_cost(t - 1);
        const float q1 = matvec_row<D, TIn>(Qt, v_x, tid), q2 = matvec_row<D, TIn>(Qt, v_xt, tid);
        const float q1T = matvecT_row<D, TIn>(Qt, v_x, s_red, tid), q2T = matvecT_row<D, TIn>(Qt, v_xt, s_red, tid);
        if (tid % TPR == 0) {
          v_y[tid / TPR] = 0.5f * q1;
          v_z[tid / TPR] = 0.5f * q2;
        }
        __syncthreads();
        al += 0.5f * q1T;
        alt += 0.5f * q2T;
        if (tid < D) {
          al += v_y[tid];
          alt += v_z[tid];
        }
      }
      __syncthreads();
      if (tid < D) {
        v_l[tid] = al;
        v_lt[tid] = alt;
        tL[(long)t * D + tid] = al;
        tLt[(long)t * D + tid] = alt;
      }
      __syncthreads();
    }
    if (tid < D) ba.gx0[prob * D + tid] = info ? nanv : v_lt[tid];
    if (tid == 0 && p.info) p.info[prob] = info;

    // ---- gradients: per step, or summed over the steps for time-invariant parameters
    for (int s = 0; s < T; ++s) {
      __syncthreads();
      if (tid < D) {
        s_v[0][tid] = info ? nanv : tL[(long)(s + 1) * D + tid];
        s_v[1][tid] = tLt[(long)(s + 1) * D + tid];
        s_v[2][tid] = tX[(long)s * D + tid];
        s_v[3][tid] = tXt[(long)s * D + tid];
        s_v[4][tid] = info ? nanv : tU[(long)s * D + tid];
        s_v[5][tid] = tUt[(long)s * D + tid];
        s_v[6][tid] = info ? nanv : tX[(long)(s + 1) * D + tid];
        s_v[7][tid] = tXt[(long)(s + 1) * D + tid];
      }
      __syncthreads();
      const long long mat = (long long)D * D;
      if (ba.sum_steps) {
        const long long o = prob * mat;
        const bool lastq = (s == T - 1) && ba.gQT;  // a terminal cost that is its own matrix has its own gradient
        if (s == 0) {
          outer2_global<D, false>(ba.gA + o, s_v[0], s_v[3], s_v[1], s_v[2], 1.f, tid);
          outer2_global<D, false>(ba.gB + o, s_v[0], s_v[5], s_v[1], s_v[4], 1.f, tid);
          outer2_global<D, false>(ba.gR + o, s_v[5], s_v[4], s_v[4], s_v[5], 0.5f, tid);
          if (lastq) {  // T = 1: nothing is charged at Q
            outer2_global<D, false>(ba.gQT + o, s_v[7], s_v[6], s_v[6], s_v[7], 0.5f, tid);
            outer2_global<D, false>(ba.gQ + o, s_v[7], s_v[6], s_v[6], s_v[7], 0.f, tid);
          } else {
            outer2_global<D, false>(ba.gQ + o, s_v[7], s_v[6], s_v[6], s_v[7], 0.5f, tid);
          }
        } else {
          outer2_global<D, true>(ba.gA + o, s_v[0], s_v[3], s_v[1], s_v[2], 1.f, tid);
          outer2_global<D, true>(ba.gB + o, s_v[0], s_v[5], s_v[1], s_v[4], 1.f, tid);
          outer2_global<D, true>(ba.gR + o, s_v[5], s_v[4], s_v[4], s_v[5], 0.5f, tid);
          if (lastq) outer2_global<D, false>(ba.gQT + o, s_v[7], s_v[6], s_v[6], s_v[7], 0.5f, tid);
          else outer2_global<D, true>(ba.gQ + o, s_v[7], s_v[6], s_v[6], s_v[7], 0.5f, tid);
        }
      } else {
        const long long o = (prob * T + s) * mat;
        outer2_global<D, false>(ba.gA + o, s_v[0], s_v[3], s_v[1], s_v[2], 1.f, tid);
        outer2_global<D, false>(ba.gB + o, s_v[0], s_v[5], s_v[1], s_v[4], 1.f, tid);
        outer2_global<D, false>(ba.gQ + o, s_v[7], s_v[6], s_v[6], s_v[7], 0.5f, tid);
        outer2_global<D, false>(ba.gR + o, s_v[5], s_v[4], s_v[4], s_v[5], 0.5f, tid);
      }
    }
    __syncthreads();
  }
}

}  // namespace ttc
