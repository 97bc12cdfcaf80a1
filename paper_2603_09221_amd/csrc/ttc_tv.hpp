// Time-heterogeneous problems: A_t, B_t, Q_t, R_t vary over the horizon (the general statement of
// Prop. 3.1; the paper's "time-heterogeneous parameterization", Sec. 4).
//
// With every factor Sigma_t of Thm 3.3 different, nothing can be prepared once per problem: each factor
// would need its own A_t^{-1} and G_t = B_t R_t^{-1} B_t^T, two dense solves before the factor is even
// applied, and a re-base on top.  Re-basing after every factor turns the iteration into the backward
// recursion of Prop. 3.1 itself, and its printed form needs one solve per step, with a positive
// definite matrix (no pivot search):
//     S_s = R_s + B_s^T P_{s+1} B_s,   W_s = S_s^{-1} B_s^T P_{s+1} A_s,   K_s = -W_s        (Eq. "decode")
//     P_s = Q[s-1] + A_s^T P_{s+1} A_s - (B_s^T P_{s+1} A_s)^T W_s   (P_T = Q[T-1], no Q on x_0)  (Eq. "riccati")
// Six products and one dense solve per step; the value matrix stays on chip for the whole horizon, the
// step's matrices are streamed from HBM once each.
#pragma once
#include "ttc_common.hpp"
#include "ttc_small.hpp"
#include "ttc_rollout.hpp"

namespace ttc {


// accumulator rows of this wavefront <- row-major global matrix of input element type
template <int D, typename TIn>
__device__ __forceinline__ void load_rows_input(const TIn* src, floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int h = 0; h < C::NH; ++h) {
        const long off = (long)(16 * (C::RB * w + rb) + 4 * g + v) * D + 16 * C::VEC * h + C::VEC * i;
        if constexpr (C::VEC == 4) {
          const floatx4 t = ld4<TIn>(src, off);
#pragma unroll
          for (int tp = 0; tp < 4; ++tp) acc[rb][h * 4 + tp][v] = t[tp];
        } else {
#pragma unroll
          for (int tp = 0; tp < C::VEC; ++tp) acc[rb][h * C::VEC + tp][v] = ld1<TIn>(src, off + tp);
        }
      }
}

// One backward step of Prop. 3.1 with the matrices of one step.  On entry the right half of the pair
// holds P_{s+1} (symmetric); on exit it holds W = S^{-1} B^T P A = -K_s, S = R + B^T P B, and pn holds this
// wavefront's rows of A^T P A - (B^T P A)^T W, which is P_s up to the stage cost.  Six products and one
// unpivoted solve (S is positive definite).  Returns the solve's breakdown flag.
template <int D, typename TIn>
__device__ __forceinline__ int riccati_step(float* W, SolveScratch<D>& S, const TIn* As, const TIn* Bs, const TIn* Rs,
                                            floatx4 (&pn)[Cfg<D>::RB][Cfg<D>::NT], int tid) {
  using C = Cfg<D>;
  tid += opaque_zero();
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  float cFT[C::RB][C::KS];
  {
    float cAT[C::RB][C::KS], cBT[C::RB][C::KS];
    {
      floatx4 accPA[C::RB][C::NT], accPB[C::RB][C::NT];
      {
        float cP[C::RB][C::KS];
        load_aop_lds<D>(WR, cP, w, i, g);  // rows of P (symmetric)
        load_half<D, TIn, false>(WL, As, tid);
        __syncthreads();
        load_half<D, TIn, false>(WR, Bs, tid);  // P is in registers now
        zero_acc<D>(accPA);
        gemm_acc<D>(accPA, cP, WL, i, g);  // P A
        __syncthreads();
        zero_acc<D>(accPB);
        gemm_acc<D>(accPB, cP, WR, i, g);  // P B
      }
      load_aopT_lds<D>(WL, cAT, w, i, g);  // rows of A^T
      load_aopT_lds<D>(WR, cBT, w, i, g);  // rows of B^T
      __syncthreads();
      store_rows<D>(WL, accPA, w, i, g);
      store_rows<D>(WR, accPB, w, i, g);
      __syncthreads();
    }
    floatx4 accS[C::RB][C::NT], accF[C::RB][C::NT];
    load_rows_input<D, TIn>(Rs, accS, w, i, g);
    gemm_acc<D>(accS, cBT, WR, i, g);  // S = R + B^T P B
    zero_acc<D>(accF);
    gemm_acc<D>(accF, cBT, WL, i, g);  // F = B^T P A
    zero_acc<D>(pn);
    gemm_acc<D>(pn, cAT, WL, i, g);    // A^T P A
    __syncthreads();
    store_rows<D>(WL, accS, w, i, g);
    store_rows<D>(WR, accF, w, i, g);
    __syncthreads();
  }
  symmetrise_half<D>(WL, tid);  // R is read as its symmetric part
  load_aopT_lds<D>(WR, cFT, w, i, g);  // rows of F^T
  __syncthreads();
  const int flag = lds_solve<D, 7, false>(W, S, tid);  // right half: W = S^{-1} F
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int k = 0; k < C::KS; ++k) cFT[rb][k] = -cFT[rb][k];
  gemm_acc<D>(pn, cFT, WR, i, g);  // - F^T W
  return flag;
}

// pn += the symmetric part of the stage cost Qs (staged through the left half), then P_s = pn goes to the
// right half, exactly symmetric.  Contains the barriers it needs; the right half must no longer be read.
template <int D, typename TIn>
__device__ __forceinline__ void next_value_matrix(float* W, const TIn* Qs, floatx4 (&pn)[Cfg<D>::RB][Cfg<D>::NT], int tid) {
  using C = Cfg<D>;
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  load_half<D, TIn, false>(WL, Qs, tid);
  __syncthreads();
  symmetrise_half<D>(WL, tid);
  __syncthreads();
  floatx4 q[C::RB][C::NT];
  load_rows<D>(WL, q, w, i, g);
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int c = 0; c < C::NT; ++c) pn[rb][c] += q[rb][c];
  store_rows<D>(WR, pn, w, i, g);
  __syncthreads();
  symmetrise_half<D>(WR, tid);
  __syncthreads();
}

// The whole backward recursion of one problem by one workgroup, from P_T to the outputs P_0, K_0, u_0, value and
// info: T calls of riccati_step.  Step s reads A, B, R at As + s*tA, Bs + s*tB, Rs + s*tR and the stage cost on
// the state it starts from at Qs + (s-1)*tQ (none for s = 0); zero strides give the time-invariant problem.
// The terminal value matrix is PTf (float32) if given, else PT (input element type).  info_base is added to the
// index (1 = the step taken first, s = T-1) of the step whose solve broke down.  All threads must call it.
template <int D, typename TIn>
__device__ __forceinline__ void riccati_problem(float* W, SolveScratch<D>& S, float* s_red, const SolveArgs& p,
                                                long long prob, int T, const TIn* As, const TIn* Bs, const TIn* Qs,
                                                const TIn* Rs, long long tA, long long tB, long long tQ, long long tR,
                                                const TIn* PT, const float* PTf, const TIn* Qflag, const TIn* x0p,
                                                int info_base, int tid) {
  using C = Cfg<D>;
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  int info = 0;
  if (PTf) load_half<D, float, false>(WR, PTf, tid);
  else load_half<D, TIn, false>(WR, PT, tid);
  __syncthreads();
  symmetrise_half<D>(WR, tid);
  __syncthreads();
  for (int s = T - 1; s >= 0; --s) {
    floatx4 pn[C::RB][C::NT];
    const int flag = riccati_step<D, TIn>(W, S, As + (long long)s * tA, Bs + (long long)s * tB, Rs + (long long)s * tR,
                                          pn, tid);
    if (flag && !info) info = info_base + T - s;
    if (s >= 1) {
      __syncthreads();  // every wavefront is done reading W = -K_s
      next_value_matrix<D, TIn>(W, Qs + (long long)(s - 1) * tQ, pn, tid);
    } else {
      store_rows<D>(WL, pn, w, i, g);  // P_0 (no cost on x_0)
      __syncthreads();
      symmetrise_half<D>(WL, tid);
      __syncthreads();
      floatx4 acc[C::RB][C::NT];
      load_rows<D>(WR, acc, w, i, g);  // rows of -K_0
      emit_gain<D, TIn>(p, prob, acc, x0p, info, tid);
      emit_value<D, TIn>(p, prob, WL, Qflag, x0p, info, s_red, tid);
    }
  }
}

template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) solve_tv_kernel(const TvArgs ta) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  const SolveArgs& p = ta.s;

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero();
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    riccati_problem<D, TIn>(W, S, s_red, p, prob, p.T, Ap, Bp, Qp, Rp, ta.tA, ta.tB, ta.tQ, ta.tR,
                            Qp + (long long)(p.T - 1) * ta.tQ, ta.PT ? ta.PT + prob * ta.sPT : nullptr, Qp, x0p, 0, tid);
  }
}

// Roll-out of a time-heterogeneous problem (Alg. 1 with r = 0): the backward sweep of solve_tv_kernel
// keeping every gain K_s in the workspace, then the closed-loop forward sweep
// u_s = K_s x_s, x_{s+1} = A_s x_s + B_s u_s with the cost sum_s u_s^T R_s u_s + x_{s+1}^T Q[s] x_{s+1}.
template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) rollout_tv_kernel(const TvRolloutArgs ta) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  __shared__ float s_x[D], s_u[D], s_xn[D];
  const RolloutArgs& p = ta.r;
  float* const WR = W + D;
  float* const wsK = p.ws + (long)blockIdx.x * p.T * D * D;  // K_0 .. K_{T-1}, row-major

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    int info = 0;
    {
      const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
      load_half<D, TIn, false>(WR, Qp + (long long)(p.T - 1) * ta.tQ, tid);  // P_T = Q_T
      __syncthreads();
      symmetrise_half<D>(WR, tid);
      __syncthreads();
      // ---- backward sweep
      for (int s = p.T - 1; s >= 0; --s) {
        floatx4 pn[C::RB][C::NT];
        const int flag = riccati_step<D, TIn>(W, S, Ap + (long long)s * ta.tA, Bp + (long long)s * ta.tB,
                                              Rp + (long long)s * ta.tR, pn, tid);
        if (flag && !info) info = p.T - s;
        {
          floatx4 acc[C::RB][C::NT];
          load_rows<D>(WR, acc, w, i, g);
#pragma unroll
          for (int rb = 0; rb < C::RB; ++rb) {
#pragma unroll
            for (int cc = 0; cc < C::NT; ++cc) acc[rb][cc] = -acc[rb][cc];
            write_rows_global<D>(wsK + (long)s * D * D, acc[rb], C::RB * w + rb, i, g);  // K_s
          }
        }
        __syncthreads();
        if (s >= 1) next_value_matrix<D, TIn>(W, Qp + (long long)(s - 1) * ta.tQ, pn, tid);
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
// PPW = problems per wavefront: 4 for batches that fill the chip, 1 for small ones (the four rows of 16 lanes
// then all hold the same problem; every per-problem loop runs once).
//
// riccati_quad: the whole backward recursion of the wavefront's PPW problems, from their terminal value matrices
// (PTp[q], input element type) to the outputs.  Step s of problem q reads A, B, R at Ap[q] + s*tA, ... and the
// stage cost on the state it starts from at Qp[q] + (s-1)*tQ; zero strides give the time-invariant problem.
// info = info_base + the index (1 = the step taken first) of the step whose solve broke down.
template <typename TIn, int PPW>
__device__ __forceinline__ void riccati_quad(float (*Wm)[16 * Cfg<16>::PITCH], float* s_red, const SolveArgs& p,
                                             const long long (&prob)[PPW], const bool (&valid)[PPW], int T,
                                             const TIn* const (&Ap)[PPW], const TIn* const (&Bp)[PPW],
                                             const TIn* const (&Qp)[PPW], const TIn* const (&Rp)[PPW],
                                             const TIn* const (&PTp)[PPW], long long tA, long long tB, long long tQ,
                                             long long tR, int info_base, int tid) {
  constexpr int D = 16;
  using C = Cfg<D>;
  constexpr int w = 0;
  const int lane = tid & 63, i = lane & 15, g = lane >> 4;
  float* const Wmine = Wm[g & (PPW - 1)];  // the problem whose rows this lane holds during the dense solves
  int info[PPW] = {};
  int nsolve = 0;
  auto note = [&](int bad) {
    ++nsolve;
    const unsigned long long m = __ballot(bad != 0);
#pragma unroll
    for (int q = 0; q < PPW; ++q)
      if (!info[q] && ((m >> (16 * q)) & 0xFFFFull)) info[q] = nsolve;
  };
  // One problem per wavefront is the shape of small batches, where nothing else hides a step's reads of its matrices:
  // there they are requested one step ahead (PF), into registers, and handed to LDS when their turn comes.
  constexpr bool PF = PPW == 1;
  HalfRegs<D> hA[PPW], hB[PPW], hQ[PPW];
  floatx4 rR[PPW][C::RB][C::NT];
  auto fetch_abr = [&](int s) {
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      issue_half<D, TIn>(hA[q], Ap[q] + (long long)s * tA, tid);
      issue_half<D, TIn>(hB[q], Bp[q] + (long long)s * tB, tid);
      load_rows_input<D, TIn>(Rp[q] + (long long)s * tR, rR[q], w, i, g);
    }
  };
  auto fetch_q = [&](int s) {  // the stage cost on the state step s starts from
#pragma unroll
    for (int q = 0; q < PPW; ++q) issue_half<D, TIn>(hQ[q], Qp[q] + (long long)(s - 1) * tQ, tid);
  };
  if (PF) {
    fetch_abr(T - 1);
    if (T >= 2) fetch_q(T - 1);
  }
#pragma unroll
  for (int q = 0; q < PPW; ++q) load_half<D, TIn, false>(Wm[q] + D, PTp[q], tid);  // P_T = Q_T
  wave_lds_sync();
#pragma unroll
  for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
  wave_lds_sync();
  for (int s = T - 1; s >= 0; --s) {
    // the step of riccati_step, for four problems at once
    floatx4 pn[PPW][C::RB][C::NT], accF[PPW][C::RB][C::NT], accW[PPW][C::RB][C::NT];
    {
      float cAT[PPW][C::RB][C::KS], cBT[PPW][C::RB][C::KS];
      {
        floatx4 accPA[PPW][C::RB][C::NT], accPB[PPW][C::RB][C::NT];
        {
          float cP[PPW][C::RB][C::KS];
#pragma unroll
          for (int q = 0; q < PPW; ++q) {
            load_aop_lds<D>(Wm[q] + D, cP[q], w, i, g);  // rows of P
            if (PF) commit_half<D, false>(Wm[q], hA[q], tid);
            else load_half<D, TIn, false>(Wm[q], Ap[q] + (long long)s * tA, tid);
          }
          wave_lds_sync();
#pragma unroll
          for (int q = 0; q < PPW; ++q) {
            if (PF) commit_half<D, false>(Wm[q] + D, hB[q], tid);  // P is in registers now
            else load_half<D, TIn, false>(Wm[q] + D, Bp[q] + (long long)s * tB, tid);
            zero_acc<D>(accPA[q]);
            zero_acc<D>(accPB[q]);
          }
          gemm_acc_quad<PPW>(accPA, cP, Wm, 0, i, g);  // P A
          wave_lds_sync();
          gemm_acc_quad<PPW>(accPB, cP, Wm, D, i, g);  // P B
        }
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          load_aopT_lds<D>(Wm[q], cAT[q], w, i, g);      // rows of A^T
          load_aopT_lds<D>(Wm[q] + D, cBT[q], w, i, g);  // rows of B^T
        }
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          store_rows<D>(Wm[q], accPA[q], w, i, g);
          store_rows<D>(Wm[q] + D, accPB[q], w, i, g);
        }
        wave_lds_sync();
      }
      floatx4 accS[PPW][C::RB][C::NT];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if (PF) accS[q][0][0] = rR[q][0][0];
        else load_rows_input<D, TIn>(Rp[q] + (long long)s * tR, accS[q], w, i, g);
        zero_acc<D>(accF[q]);
        zero_acc<D>(pn[q]);
      }
      if (PF && s >= 1) fetch_abr(s - 1);  // the next step's matrices, while this step computes
      gemm_acc_quad<PPW>(accS, cBT, Wm, D, i, g);  // S = R + B^T P B
      gemm_acc_quad<PPW>(accF, cBT, Wm, 0, i, g);  // F = B^T P A
      gemm_acc_quad<PPW>(pn, cAT, Wm, 0, i, g);    // A^T P A
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], accS[q], w, i, g);
      wave_lds_sync();
    }
#pragma unroll
    for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);  // R is read as its symmetric part
    wave_lds_sync();
    float cS[PPW][C::RB][C::KS];
#pragma unroll
    for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q], cS[q], w, i, g);  // rows of S, for the refinement below
    note(invert_rows16<false, true>(Wmine, lane));  // left halves: S^{-1}
    {
      // At d = 16 the accumulator layout of F is both the B operand of F and the A operand of F^T.
      float cSi[PPW][C::RB][C::KS];
      floatx4 res[PPW];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_aop_lds<D>(Wm[q], cSi[q], w, i, g);  // rows of S^{-1}
        zero_acc<D>(accW[q]);
        res[q] = accF[q][0][0];
      }
#pragma unroll
      for (int t = 0; t < 4; ++t)  // W = S^{-1} F = -K_s
#pragma unroll
        for (int q = 0; q < PPW; ++q)
          accW[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(cSi[q][0][t], accF[q][0][0][t], accW[q][0][0], 0, 0, 0);
      // One step of refinement, W += S^{-1} (F - S W): an explicitly formed inverse leaves an error proportional
      // to cond(S) in W, which the cancellation in A^T P A - F^T W magnifies when control is cheap; the corrected
      // W is as good as a factor-and-solve.
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int q = 0; q < PPW; ++q)
          res[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(-cS[q][0][t], accW[q][0][0][t], res[q], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int q = 0; q < PPW; ++q)
          accW[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(cSi[q][0][t], res[q][t], accW[q][0][0], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < 4; ++t)  // - F^T W
#pragma unroll
        for (int q = 0; q < PPW; ++q)
          pn[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(-accF[q][0][0][t], accW[q][0][0][t], pn[q][0][0], 0, 0, 0);
    }
    wave_lds_sync();
    if (s >= 1) {
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if (PF) commit_half<D, false>(Wm[q], hQ[q], tid);
        else load_half<D, TIn, false>(Wm[q], Qp[q] + (long long)(s - 1) * tQ, tid);
      }
      if (PF && s >= 2) fetch_q(s - 1);
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        floatx4 qs[C::RB][C::NT];
        load_rows<D>(Wm[q], qs, w, i, g);
        pn[q][0][0] += qs[0][0];
        store_rows<D>(Wm[q] + D, pn[q], w, i, g);  // P_s
      }
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
      wave_lds_sync();
    } else {
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], pn[q], w, i, g);  // P_0 (no cost on x_0)
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if (!valid[q]) continue;  // uniform over the wavefront
        const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob[q] * p.sx0;
        emit_gain<D, TIn>(p, prob[q], accW[q], x0p, info[q], tid);  // rows of -K_0
        emit_value<D, TIn>(p, prob[q], Wm[q], Qp[q], x0p, info[q] ? info_base + info[q] : 0, s_red, tid);
      }
      __syncthreads();
    }
  }
}

template <typename TIn, int PPW>
__global__ void __launch_bounds__(64, 2) solve_tv_small_kernel(const TvArgs ta) {
  constexpr int D = 16;
  using C = Cfg<D>;
  static_assert(PPW == 1 || PPW == 4, "one problem or four per wavefront");
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  __shared__ float s_red[C::NW];
  const SolveArgs& p = ta.s;
  const long long nquads = (p.n + PPW - 1) / PPW;

  for (long long quad = blockIdx.x; quad < nquads; quad += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero();
    long long prob[PPW];  // a ragged last quad repeats the last problem; only valid ones are written out
    bool valid[PPW];
    const TIn *Ap[PPW], *Bp[PPW], *Qp[PPW], *Rp[PPW], *PTp[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      valid[q] = quad * PPW + q < p.n;
      prob[q] = valid[q] ? quad * PPW + q : p.n - 1;
      Ap[q] = reinterpret_cast<const TIn*>(p.A) + prob[q] * p.sA;
      Bp[q] = reinterpret_cast<const TIn*>(p.B) + prob[q] * p.sB;
      Qp[q] = reinterpret_cast<const TIn*>(p.Q) + prob[q] * p.sQ;
      Rp[q] = reinterpret_cast<const TIn*>(p.R) + prob[q] * p.sR;
      PTp[q] = Qp[q] + (long long)(p.T - 1) * ta.tQ;  // P_T = Q_T
    }
    riccati_quad<TIn, PPW>(Wm, s_red, p, prob, valid, p.T, Ap, Bp, Qp, Rp, PTp, ta.tA, ta.tB, ta.tQ, ta.tR, 0, tid);
  }
}

}  // namespace ttc
