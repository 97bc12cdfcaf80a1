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

// Two matrix-vector products at once (the primal and the dual trajectory always need the same matrix): for the
// row r = tid / TPR of a row-major d x d matrix, ya = sum_c M[r][c] xa[c] and yb likewise; the TPR threads of a
// row each take a share of the columns and all of them get the sums.  MatLoad(r, c4) returns M[r][c4 .. c4+3].
template <int D, typename MatLoad>
__device__ __forceinline__ void matvec2(MatLoad&& row4, const float* xa, const float* xb, int tid, float& ya, float& yb) {
  constexpr int TPR = Cfg<D>::NTHR / D;  // 2 or 4
  const int r = tid / TPR, part = tid % TPR;
  float sa = 0.f, sb = 0.f;
#pragma unroll
  for (int c4 = part * (D / TPR); c4 < (part + 1) * (D / TPR); c4 += 4) {
    const floatx4 mv = row4(r, c4);
    sa += mv[0] * xa[c4] + mv[1] * xa[c4 + 1] + mv[2] * xa[c4 + 2] + mv[3] * xa[c4 + 3];
    sb += mv[0] * xb[c4] + mv[1] * xb[c4 + 1] + mv[2] * xb[c4 + 2] + mv[3] * xb[c4 + 3];
  }
#pragma unroll
  for (int m = 1; m < TPR; m <<= 1) {
    sa += __shfl_xor(sa, m, 64);
    sb += __shfl_xor(sb, m, 64);
  }
  ya = sa;
  yb = sb;
}
// The transposed products ya[j] = sum_r M[r][j] xa[r], yb likewise: thread (part, j) sums its share of the rows
// (consecutive threads read consecutive columns), the parts are added through LDS (red: 2 x TPR x D floats).
// Contains two barriers; every thread gets the sums for j = tid % D.  MatLoad1(r, j) returns M[r][j].
template <int D, typename MatLoad1>
__device__ __forceinline__ void matvecT2(MatLoad1&& elem, const float* xa, const float* xb, float* red, int tid, float& ya,
                                         float& yb) {
  constexpr int TPR = Cfg<D>::NTHR / D;
  const int j = tid % D, part = tid / D;
  float sa = 0.f, sb = 0.f;
#pragma unroll 8
  for (int r = part * (D / TPR); r < (part + 1) * (D / TPR); ++r) {
    const float mv = elem(r, j);
    sa += mv * xa[r];
    sb += mv * xb[r];
  }
  red[part * D + j] = sa;
  red[(TPR + part) * D + j] = sb;
  __syncthreads();
  float a = 0.f, b = 0.f;
#pragma unroll
  for (int q = 0; q < TPR; ++q) {
    a += red[q * D + j];
    b += red[(TPR + q) * D + j];
  }
  __syncthreads();
  ya = a;
  yb = b;
}

// out (d x d, row-major, global) = scale (a b^T + c e^T), vectors in LDS; each thread a share of the 16-byte pieces
template <int D>
__device__ __forceinline__ void outer2_global(float* out, const float* a, const float* b, const float* c, const float* e,
                                              float scale, int tid) {
  using C = Cfg<D>;
  for (int idx = tid; idx < D * D / 4; idx += C::NTHR) {
    const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
    const float ar = scale * a[r], cr = scale * c[r];
    floatx4 v;
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = ar * b[c4 + k] + cr * e[c4 + k];
    *reinterpret_cast<floatx4*>(out + (long)r * D + c4) = v;
  }
}

template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) backward_kernel(const BackwardArgs ba) {
  using C = Cfg<D>;
  constexpr int TPR = C::NTHR / D;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[2 * TPR * D];
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
    float* const v_xt = s_v[1];
    float* const v_u = s_v[2];
    float* const v_ut = s_v[3];
    float* const v_l = s_v[4];
    float* const v_lt = s_v[5];
    float* const v_y = s_v[6];
    float* const v_z = s_v[7];
    auto glob4 = [](const TIn* M) { return [M](int r, int c4) { return ld4<TIn>(M, (long)r * D + c4); }; };
    auto glob1 = [](const TIn* M) { return [M](int r, int j) { return ld1<TIn>(M, (long)r * D + j); }; };
    auto lds4 = [](const float* Wh) {
      return [Wh](int r, int c4) { return *reinterpret_cast<const floatx4*>(Wh + r * C::PITCH + c4); };
    };
    auto lds1 = [](const float* Wh) { return [Wh](int r, int j) { return Wh[r * C::PITCH + j]; }; };
    const bool lead = (tid % TPR == 0);  // one thread of each row's group
    const int row = tid / TPR;
    if (tid < D) {
      v_x[tid] = ld1<TIn>(x0p, tid);
      v_xt[tid] = 0.f;
    }
    __syncthreads();
    {
      float y, dummy;
      matvec2<D>(glob4(Ap), v_x, v_xt, tid, y, dummy);  // A_0 x_0
      if (lead) v_y[row] = y;
    }
    __syncthreads();
    {
      float z, dummy;
      matvec2<D>(lds4(WR), v_y, v_xt, tid, z, dummy);  // P_1 A_0 x_0
      if (lead) v_z[row] = z;
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
      float fx, dummy;
      matvecT2<D>(lds1(WL), v_z, v_xt, s_red, tid, fx, dummy);  // B_0^T P_1 A_0 x_0 (contains barriers)
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
      v_u[tid] = -WR[tid * C::PITCH + 0];
      v_ut[tid] = -WR[tid * C::PITCH + 1];
      tX[tid] = v_x[tid];
      tXt[tid] = 0.f;
    }
    __syncthreads();
    // Time-invariant parameters: A and B stay in the two halves of the pair (free from here on) for the closed
    // loops and the co-states, so that only the gains are read from memory in the loops below.
    const bool resident = ba.sum_steps != 0;
    if (resident) {
      load_half<D, TIn, false>(WL, Ap, tid);
      load_half<D, TIn, false>(WR, Bp, tid);
      __syncthreads();
    }

    // ---- both closed loops forward (Alg. 1): states and controls of every step to the workspace
    for (int s = 0; s < T; ++s) {
      const TIn* As = Ap + (long long)s * ba.tA;
      const TIn* Bs = Bp + (long long)s * ba.tB;
      if (s >= 1) {
        const float* Ks = wsK + (long)(s - 1) * D * D;
        float u, ut;
        matvec2<D>([Ks](int r, int c4) { return *reinterpret_cast<const floatx4*>(Ks + (long)r * D + c4); }, v_x, v_xt,
                   tid, u, ut);
        if (lead) {
          v_u[row] = u;
          v_ut[row] = ut;
        }
        __syncthreads();
      }
      float ax, axt, bu, but;
      if (resident) {
        matvec2<D>(lds4(WL), v_x, v_xt, tid, ax, axt);
        matvec2<D>(lds4(WR), v_u, v_ut, tid, bu, but);
      } else {
        matvec2<D>(glob4(As), v_x, v_xt, tid, ax, axt);
        matvec2<D>(glob4(Bs), v_u, v_ut, tid, bu, but);
      }
      if (tid < D) {
        tU[(long)s * D + tid] = v_u[tid];
        tUt[(long)s * D + tid] = v_ut[tid];
      }
      __syncthreads();  // every thread has read the old states
      if (lead) {
        v_x[row] = ax + bu;
        v_xt[row] = axt + but;
        tX[(long)(s + 1) * D + row] = ax + bu;
        tXt[(long)(s + 1) * D + row] = axt + but;
      }
      __syncthreads();
    }

    // ---- co-states backward (Alg. 2), for both trajectories; dl/dx_0 = lamt_0.  A cost matrix is read as its
    // symmetric part: half of Q x + Q^T x from memory, or the symmetrised copy when it stays in LDS.
    auto sym_cost_times = [&](const TIn* Qm, float& qa, float& qb) {  // for j = tid < D: (sym(Q) v_x)[j], (sym(Q) v_xt)[j]
      float r1, r2, c1, c2;
      matvec2<D>(glob4(Qm), v_x, v_xt, tid, r1, r2);
      matvecT2<D>(glob1(Qm), v_x, v_xt, s_red, tid, c1, c2);
      if (lead) {
        v_y[row] = r1;
        v_z[row] = r2;
      }
      __syncthreads();
      qa = qb = 0.f;
      if (tid < D) {
        qa = 0.5f * (v_y[tid] + c1);
        qb = 0.5f * (v_z[tid] + c2);
      }
      __syncthreads();
    };
    {
      float qa, qb;
      sym_cost_times(stage_cost(T - 1), qa, qb);  // lam_T = Q_T x_T
      if (tid < D) {
        v_l[tid] = qa;
        v_lt[tid] = qb;
        tL[(long)T * D + tid] = qa;
        tLt[(long)T * D + tid] = qb;
      }
      __syncthreads();
    }
    if (resident && T >= 2) {  // the stage cost Q, symmetrised, takes B's place
      load_half<D, TIn, false>(WR, Qp, tid);
      __syncthreads();
      symmetrise_half<D>(WR, tid);
      __syncthreads();
    }
    for (int t = T - 1; t >= 0; --t) {
      // lam_t = Q[t-1] x_t + A_t^T lam_{t+1} (no state cost for t = 0)
      const TIn* At = Ap + (long long)t * ba.tA;
      float al, alt;
      if (resident) matvecT2<D>(lds1(WL), v_l, v_lt, s_red, tid, al, alt);
      else matvecT2<D>(glob1(At), v_l, v_lt, s_red, tid, al, alt);
      if (t >= 1) {
        if (tid < D) {
          v_x[tid] = tX[(long)t * D + tid];
          v_xt[tid] = tXt[(long)t * D + tid];
        }
        __syncthreads();
        float qa, qb;
        if (resident) {
          float r1, r2;
          matvec2<D>(lds4(WR), v_x, v_xt, tid, r1, r2);
          if (lead) {
            v_y[row] = r1;
            v_z[row] = r2;
          }
          __syncthreads();
          qa = tid < D ? v_y[tid] : 0.f;
          qb = tid < D ? v_z[tid] : 0.f;
        } else {
          sym_cost_times(stage_cost(t - 1), qa, qb);
        }
        al += qa;
        alt += qb;
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

    // ---- gradients: per step, or summed over the steps (in registers) for time-invariant parameters
    auto stage_vectors = [&](int s) {  // lam, lamt of s+1; x, xt, u, ut of s; x, xt of s+1
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
    };
    const long long mat = (long long)D * D;
    if (ba.sum_steps) {
      constexpr int NV = (D * D / 4 + C::NTHR - 1) / C::NTHR;  // 16-byte pieces of a matrix per thread
      const long long o = prob * mat;
      auto put = [&](float* dst, const floatx4 (&v)[NV]) {
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          const int idx = tid + k * C::NTHR;
          if (idx < D * D / 4)
            *reinterpret_cast<floatx4*>(dst + o + (long long)(idx / (D / 4)) * D + (idx % (D / 4)) * 4) = v[k];
        }
      };
      {  // first pass over the steps: dl/dA and dl/dB (two passes keep the accumulators within the register file)
        floatx4 sA[NV], sB[NV];
#pragma unroll
        for (int k = 0; k < NV; ++k) sA[k] = sB[k] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < T; ++s) {
          stage_vectors(s);
#pragma unroll
          for (int k = 0; k < NV; ++k) {
            const int idx = tid + k * C::NTHR;
            if (idx < D * D / 4) {
              const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
              const float l = s_v[0][r], lt = s_v[1][r];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                sA[k][e] += l * s_v[3][c4 + e] + lt * s_v[2][c4 + e];
                sB[k][e] += l * s_v[5][c4 + e] + lt * s_v[4][c4 + e];
              }
            }
          }
        }
        put(ba.gA, sA);
        put(ba.gB, sB);
      }
      {  // second pass: dl/dR, dl/dQ and the terminal cost's own gradient
        floatx4 sQ[NV], sR[NV], sQT[NV];
#pragma unroll
        for (int k = 0; k < NV; ++k) sQ[k] = sR[k] = sQT[k] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < T; ++s) {
          stage_vectors(s);
          const bool terminal_own = (s == T - 1) && ba.gQT;  // a terminal cost that is its own matrix
#pragma unroll
          for (int k = 0; k < NV; ++k) {
            const int idx = tid + k * C::NTHR;
            if (idx < D * D / 4) {
              const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
              const float ur = 0.5f * s_v[4][r], utr = 0.5f * s_v[5][r], xr = 0.5f * s_v[6][r], xtr = 0.5f * s_v[7][r];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                sR[k][e] += utr * s_v[4][c4 + e] + ur * s_v[5][c4 + e];
                const float q = xtr * s_v[6][c4 + e] + xr * s_v[7][c4 + e];
                if (terminal_own) sQT[k][e] += q; else sQ[k][e] += q;
              }
            }
          }
        }
        put(ba.gQ, sQ);
        put(ba.gR, sR);
        if (ba.gQT) put(ba.gQT, sQT);
      }
    } else {
      for (int s = 0; s < T; ++s) {
        stage_vectors(s);
        const long long o = (prob * T + s) * mat;
        outer2_global<D>(ba.gA + o, s_v[0], s_v[3], s_v[1], s_v[2], 1.f, tid);
        outer2_global<D>(ba.gB + o, s_v[0], s_v[5], s_v[1], s_v[4], 1.f, tid);
        outer2_global<D>(ba.gQ + o, s_v[7], s_v[6], s_v[6], s_v[7], 0.5f, tid);
        outer2_global<D>(ba.gR + o, s_v[5], s_v[4], s_v[4], s_v[5], 0.5f, tid);
      }
    }
    __syncthreads();
  }
}

}  // namespace ttc
