// Structured, contextualised problems (Sec. 4, "Contextualization" and "Parameterization"; Sec. 3.3,
// "Structured Parameterization"), d = 16: the T steps of a problem are never stored; the kernel builds
// them from a few per-problem vectors and two shared groups of r basis matrices,
//     A_t = I + Gamma_A^t diag(s_A),   B_t = Bbar Gamma_B^t,   Q_t = Gamma_Q^t Qbar Gamma_Q^t  (t < T),
//     Q_T = sum_i s_Qf[i] Qbasis[i],   R_t = diag(1 / rinv),   Gamma_X^t = diag(exp(-t lg_X)),
//     Bbar = sum_i s_B[i] Bbasis[i],   Qbar = sum_i s_Q[i] Qbasis[i],
// and runs the Riccati step of Prop. 3.1 on them.  A diagonal A_t turns two of the step's products into
// scalings:  with V = P B_t (P = P_{t}, symmetric) and a = diag(A_t),
//     S = R + B_t^T V,   F = B_t^T P A_t = V^T diag(a),   A_t^T P A_t = diag(a) P diag(a),
//     W = S^{-1} F = -K,   P_{t-1} = Q_{t-1} + diag(a) P diag(a) - F^T W,
// three products and one positive definite solve per step.  Four problems share a wavefront, as in the
// other d = 16 kernels.  At d = 16 the accumulator layout of a matrix (lane (i, g): column i, rows
// 4g..4g+3) is the A-operand layout of its transpose, which is what lets Bbar, V and P be used in both
// roles without a trip through LDS.
#pragma once

namespace ttc {

constexpr int CXT_RMAX = 64;  // most basis matrices per group

struct CxtArgs {
  SolveArgs s;  // n, T, x0 (stride 16), outputs; flags = 0; the matrix inputs are unused
  int r;
  const void *sA, *sB, *sQ, *sQf, *rinv, *lgA, *lgB, *lgQ;  // (n,16) vectors, (n,r) coefficients
  const void *Bbasis, *Qbasis;                              // (r,16,16), shared by all problems
};

template <typename TIn>
__global__ void __launch_bounds__(64) solve_cxt_kernel(const CxtArgs ca) {
  constexpr int D = 16;
  using C = Cfg<D>;
  constexpr int PPW = 4;
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  __shared__ __attribute__((aligned(16))) float vec[PPW][4][D];         // a_t, gamma_B^t, gamma_Q^(t-1), 1/rinv
  __shared__ __attribute__((aligned(16))) float coef[PPW][3][CXT_RMAX];  // s_B, s_Q, s_Qf
  __shared__ float s_red[C::NW];
  const SolveArgs& p = ca.s;
  const int r = ca.r;
  const long long nquads = (p.n + PPW - 1) / PPW;
  const TIn* const Bbasis = reinterpret_cast<const TIn*>(ca.Bbasis);
  const TIn* const Qbasis = reinterpret_cast<const TIn*>(ca.Qbasis);

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

    // ---- per-problem vectors: lane (i, g) keeps entry i of problem g's
    const long long pg = (quad * PPW + g < p.n) ? quad * PPW + g : p.n - 1;
    const float sA_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.sA), pg * D + i);
    const float lgA_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgA), pg * D + i);
    const float lgB_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgB), pg * D + i);
    const float lgQ_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgQ), pg * D + i);
    vec[g][3][i] = 1.f / ld1<TIn>(reinterpret_cast<const TIn*>(ca.rinv), pg * D + i);
    for (int k = i; k < r; k += 16) {
      coef[g][0][k] = ld1<TIn>(reinterpret_cast<const TIn*>(ca.sB), pg * r + k);
      coef[g][1][k] = ld1<TIn>(reinterpret_cast<const TIn*>(ca.sQ), pg * r + k);
      coef[g][2][k] = ld1<TIn>(reinterpret_cast<const TIn*>(ca.sQf), pg * r + k);
    }
    __syncthreads();

    // ---- Bbar, Qbar, Q_T in the accumulator layout: element (4g+v, i) of each of the four problems
    floatx4 Bbar[PPW], Qbar[PPW];
    float rI[PPW];
    {
      floatx4 Qf[PPW];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        Bbar[q] = floatx4{0.f, 0.f, 0.f, 0.f};
        Qbar[q] = Bbar[q];
        Qf[q] = Bbar[q];
        rI[q] = vec[q][3][i];
      }
#pragma unroll 2
      for (int k = 0; k < r; ++k) {
        floatx4 bb, qb;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          bb[v] = ld1<TIn>(Bbasis, (long)k * D * D + (4 * g + v) * D + i);
          qb[v] = ld1<TIn>(Qbasis, (long)k * D * D + (4 * g + v) * D + i);
        }
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          const float cb = coef[q][0][k], cq = coef[q][1][k], cf = coef[q][2][k];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            Bbar[q][v] += cb * bb[v];
            Qbar[q][v] += cq * qb[v];
            Qf[q][v] += cf * qb[v];
          }
        }
      }
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q] + D, reinterpret_cast<floatx4(&)[1]>(Qf[q]), w, i, g);  // P_T = Q_T
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
    __syncthreads();

    for (int s = p.T - 1; s >= 0; --s) {  // step s is the paper's t = s + 1; it turns P_t into P_{t-1}
      const float tf = (float)(s + 1);
      vec[g][0][i] = 1.f + expf(-tf * lgA_m) * sA_m;
      vec[g][1][i] = expf(-tf * lgB_m);
      vec[g][2][i] = expf(-(float)s * lgQ_m);  // for Q_{t-1}
      float cP[PPW][C::RB][C::KS];
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q] + D, cP[q], w, i, g);  // rows of P
      __syncthreads();
      float aI[PPW], qI[PPW];
      floatx4 aG[PPW], qG[PPW];
      floatx4 pn[PPW][C::RB][C::NT];
      float cBT[PPW][C::RB][C::KS];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        aI[q] = vec[q][0][i];
        qI[q] = vec[q][2][i];
        aG[q] = *reinterpret_cast<const floatx4*>(&vec[q][0][4 * g]);
        qG[q] = *reinterpret_cast<const floatx4*>(&vec[q][2][4 * g]);
        const float bI = vec[q][1][i];
        floatx4 bt[1];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          bt[0][v] = Bbar[q][v] * bI;                    // B_t: column i scaled
          cBT[q][0][v] = bt[0][v];                       // = rows of B_t^T as the A operand
          pn[q][0][0][v] = aG[q][v] * cP[q][0][v] * aI[q];  // diag(a) P diag(a): P is symmetric
        }
        store_rows<D>(Wm[q], bt, w, i, g);
      }
      __syncthreads();
      floatx4 accV[PPW][C::RB][C::NT];
#pragma unroll
      for (int q = 0; q < PPW; ++q) zero_acc<D>(accV[q]);
      gemm_acc_quad(accV, cP, Wm, 0, i, g);  // V = P B_t
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q] + D, accV[q], w, i, g);  // every lane has its rows of P
      __syncthreads();
      float cFT[PPW][C::RB][C::KS];
      {
        floatx4 accS[PPW][C::RB][C::NT];
        float Fa[PPW][C::RB][C::KS];
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          load_aop_lds<D>(Wm[q] + D, cFT[q], w, i, g);  // rows of V
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            cFT[q][0][v] *= -aI[q];                     // rows of -F^T = -diag(a) V
            Fa[q][0][v] = accV[q][0][0][v] * aG[q][v];  // rows of F = V^T diag(a)
            accS[q][0][0][v] = (4 * g + v == i) ? rI[q] : 0.f;
          }
        }
        gemm_acc_quad(accS, cBT, Wm, D, i, g);  // S = R + B_t^T V
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          store_rows<D>(Wm[q], accS[q], w, i, g);
          store_aop_lds<D>(Wm[q] + D, Fa[q], w, i, g);
        }
        __syncthreads();
      }
      note(solve_rows16<false>(Wmine, lane));  // right halves: W = S^{-1} F = -K
      gemm_acc_quad(pn, cFT, Wm, D, i, g);     // - F^T W
      __syncthreads();
      if (s >= 1) {
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
#pragma unroll
          for (int v = 0; v < 4; ++v) pn[q][0][0][v] += qG[q][v] * Qbar[q][v] * qI[q];  // + Q_{t-1}
          store_rows<D>(Wm[q] + D, pn[q], w, i, g);
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
        __syncthreads();
      } else {
#pragma unroll
        for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], pn[q], w, i, g);  // P_0 (no cost on x_0)
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          if (!valid[q]) continue;  // uniform over the wavefront
          const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob[q] * p.sx0;
          floatx4 acc[C::RB][C::NT];
          load_rows<D>(Wm[q] + D, acc, w, i, g);  // rows of -K_0
          emit_gain<D, TIn>(p, prob[q], acc, x0p, info[q], tid);
          emit_value<D, TIn>(p, prob[q], Wm[q], static_cast<const TIn*>(nullptr), x0p, info[q], s_red, tid);
        }
        __syncthreads();
      }
    }
  }
}

}  // namespace ttc
