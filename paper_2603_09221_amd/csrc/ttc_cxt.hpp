// Structured, contextualised problems (Sec. 4, "Contextualization" and "Parameterization"; Sec. 3.3,
// "Structured Parameterization"), d = 16: the T steps of a problem are never stored; the kernel builds
// them from a few per-problem vectors and two shared groups of r basis matrices,
//     A_t = I + Gamma_A^t diag(s_A),   B_t = Bbar Gamma_B^t,   Q_t = Gamma_Q^t Qbar Gamma_Q^t  (t < T),
//     Q_T = sum_i s_Qf[i] Qbasis[i],   R_t = diag(1 / rinv),   Gamma_X^t = diag(exp(-t lg_X)),
//     Bbar = sum_i s_B[i] Bbasis[i],   Qbar = sum_i s_Q[i] Qbasis[i],
// and runs the Riccati step of Prop. 3.1 on them.  A diagonal A_t turns two of the step's products into
// scalings:  with V = P B_t (P = P_{t}, symmetric) and a = diag(A_t),
//     S = R + B_t^T V,   F = B_t^T P A_t = V^T diag(a),   A_t^T P A_t = diag(a) P diag(a),
//     K = -S^{-1} F,   P_{t-1} = Q_{t-1} + diag(a) P diag(a) + F^T K,
// four products and one inverse of a positive definite matrix per step (S^{-1} is formed in place, negated, half
// the eliminations of a solve with sixteen right-hand sides; the product S^{-1} F goes to the matrix cores).  Four problems share a wavefront, as in the
// other d = 16 kernels.  At d = 16 the accumulator layout of a matrix (lane (i, g): column i, rows
// 4g..4g+3) is the A-operand layout of its transpose, which is what lets Bbar, V and P be used in both
// roles without a trip through LDS.
#pragma once
#include "ttc_common.hpp"
#include "ttc_small.hpp"

namespace ttc {


#ifndef TTC_CXT_WAVES
#define TTC_CXT_WAVES 2  // wavefronts per SIMD the register allocation aims at
#endif
// The workgroup is one wavefront: its lanes exchange data through LDS with wave_lds_sync(), which leaves the stores
// of the roll-out's gains in flight (a workgroup barrier would wait for each of them).
// PPW = problems per wavefront: 4 for batches that fill the chip; 1 for small batches, where a wavefront's
// latency is what counts: the four rows of 16 lanes then all hold the same problem (they compute, and
// write, the same values), and every per-problem loop below runs once instead of four times.
template <typename TIn, int PPW>
__global__ void __launch_bounds__(64, TTC_CXT_WAVES) solve_cxt_kernel(const CxtArgs ca) {
  constexpr int D = 16;
  using C = Cfg<D>;
  static_assert(PPW == 1 || PPW == 4, "one problem or four per wavefront");
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  // Wm[q]: left half S and then S^{-1} (at the end P_0), right half the value matrix between steps
  constexpr int PT = D + 4;                                              // row pitch of Vt
  __shared__ __attribute__((aligned(16))) float Vt[PPW][D * PT];         // V^T; during set-up: s_B, s_Q, s_Qf
  static_assert(PPW * D * PT >= PPW * 3 * CXT_RMAX, "the coefficients are staged in Vt");
  float (*const coef)[3][CXT_RMAX] = reinterpret_cast<float (*)[3][CXT_RMAX]>(&Vt[0][0]);
  __shared__ __attribute__((aligned(16))) float vecs[2][PPW][4][D];      // a_t, gamma_B^t, gamma_Q^(t-1), 1/rinv;
                                                                         // steps alternate between the two copies
  const SolveArgs& p = ca.s;
  const int r = ca.r;
  const long long slots = ca.roll_slots ? ca.roll_slots : p.T + 3;  // matrices per problem in roll_ws
  const long long nquads = (p.n + PPW - 1) / PPW;
  const TIn* const Bbasis = reinterpret_cast<const TIn*>(ca.Bbasis);
  const TIn* const Qbasis = reinterpret_cast<const TIn*>(ca.Qbasis);

  for (long long quad = blockIdx.x; quad < nquads; quad += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, i = lane & 15, g = lane >> 4;
    const int gq = g & (PPW - 1);  // the problem, among the wavefront's, that this lane's row of 16 lanes works on
    constexpr int w = 0;
    long long prob[PPW];  // a ragged last quad repeats the last problem; only valid ones are written out
    bool valid[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      valid[q] = quad * PPW + q < p.n;
      prob[q] = valid[q] ? quad * PPW + q : p.n - 1;
    }
    float* const Wmine = Wm[gq];  // the problem whose rows this lane holds during the dense solves
    int info[PPW] = {};
    int nsolve = 0;
    auto note = [&](int bad) {
      ++nsolve;
      const unsigned long long m = __ballot(bad != 0);
#pragma unroll
      for (int q = 0; q < PPW; ++q)
        if (!info[q] && ((m >> (16 * q)) & 0xFFFFull)) info[q] = nsolve;
    };

    PhaseTimers tm;  // phases: 0 set-up, 1 dense solves, 2 products and scalings, 3 outputs
    // ---- per-problem vectors: lane (i, g) keeps entry i of problem g's
    const long long pg = (quad * PPW + gq < p.n) ? quad * PPW + gq : p.n - 1;
    const float sA_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.sA), pg * D + i);
    const float lgA_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgA), pg * D + i);
    const float lgB_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgB), pg * D + i);
    const float lgQ_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgQ), pg * D + i);
    vecs[0][gq][3][i] = 1.f / ld1<TIn>(reinterpret_cast<const TIn*>(ca.rinv), pg * D + i);
    const float x0_m = ca.roll_ws ? 0.f : ld1<TIn>(reinterpret_cast<const TIn*>(p.x0), pg * p.sx0 + i);  // for the outputs
    const float g_m = ca.dual_g ? ca.dual_g[pg * D + i] : 0.f;
    const int r4 = (r + 3) & ~3;  // the coefficients are read four at a time: zeros past r
    for (int k = i; k < r4; k += 16) {
      coef[gq][0][k] = k < r ? ld1<TIn>(reinterpret_cast<const TIn*>(ca.sB), pg * r + k) : 0.f;
      coef[gq][1][k] = k < r ? ld1<TIn>(reinterpret_cast<const TIn*>(ca.sQ), pg * r + k) : 0.f;
      coef[gq][2][k] = k < r ? ld1<TIn>(reinterpret_cast<const TIn*>(ca.sQf), pg * r + k) : 0.f;
    }
    wave_lds_sync();

    // ---- Bbar, Qbar, Q_T in the accumulator layout: element (4g+v, i) of each of the four problems
    floatx4 Bbar[PPW], Qbar[PPW], pn[PPW][C::RB][C::NT];
    float rI[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      Bbar[q] = floatx4{0.f, 0.f, 0.f, 0.f};
      Qbar[q] = Bbar[q];
      pn[q][0][0] = Bbar[q];
      rI[q] = vecs[0][q][3][i];
    }
    for (int k0 = 0; k0 < r4; k0 += 4) {
      floatx4 cb[PPW], cq[PPW], cf[PPW];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        cb[q] = *reinterpret_cast<const floatx4*>(&coef[q][0][k0]);
        cq[q] = *reinterpret_cast<const floatx4*>(&coef[q][1][k0]);
        cf[q] = *reinterpret_cast<const floatx4*>(&coef[q][2][k0]);
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int k = k0 + kk < r ? k0 + kk : r - 1;  // past r: any matrix, its coefficients are zero
        floatx4 bb, qb;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          bb[v] = ld1<TIn>(Bbasis, (long)k * D * D + (4 * g + v) * D + i);
          qb[v] = ld1<TIn>(Qbasis, (long)k * D * D + (4 * g + v) * D + i);
        }
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            Bbar[q][v] += cb[q][kk] * bb[v];
            Qbar[q][v] += cq[q][kk] * qb[v];
            pn[q][0][0][v] += cf[q][kk] * qb[v];  // P_T = Q_T
          }
        }
      }
    }
    if (ca.roll_ws) {
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        if (!valid[q]) continue;
        float* const e = ca.roll_ws + prob[q] * slots * D * D;
        write_rows_global<D>(e, reinterpret_cast<const floatx4(&)[1]>(Bbar[q]), 0, i, g);
        write_rows_global<D>(e + D * D, reinterpret_cast<const floatx4(&)[1]>(Qbar[q]), 0, i, g);
        write_rows_global<D>(e + 2 * D * D, pn[q][0], 0, i, g);
      }
    }
    // the modulation of step s (the paper's t = s + 1), entry i of problem g: a_t, gamma_B^t, gamma_Q^(t-1)
    auto write_vec = [&](int s) {
      // exp(-t lg) = 2^(-t lg log2(e)) on the hardware's base-2 exponential: the rounding of the exponent
      // costs a relative error of about 4e-8 |t lg|, at most 6e-6 before the result underflows
      const float tf = -1.44269504f * (float)(s + 1), sf = -1.44269504f * (float)s;
      float (*vec)[4][D] = vecs[s & 1];
      vec[gq][0][i] = 1.f + __builtin_amdgcn_exp2f(tf * lgA_m) * sA_m;
      vec[gq][1][i] = __builtin_amdgcn_exp2f(tf * lgB_m);
      vec[gq][2][i] = __builtin_amdgcn_exp2f(sf * lgQ_m);
    };
    // a 16 x 16 matrix in LDS: written from the accumulator layout, read back a row
    // per lane, which is the accumulator layout of the transpose
    auto put_acc = [&](float* M, int pitch, const floatx4& x) {
#pragma unroll
      for (int v = 0; v < 4; ++v) M[(4 * g + v) * pitch + i] = x[v];
    };
    auto get_row = [&](const float* M, int pitch) { return *reinterpret_cast<const floatx4*>(M + i * pitch + 4 * g); };
#pragma unroll
    for (int q = 0; q < PPW; ++q) put_acc(Wm[q] + D, C::PITCH, pn[q][0][0]);
    write_vec(p.T - 1);
    wave_lds_sync();
    tm.toc(0);

    for (int s = p.T - 1; s >= 0; --s) {  // step s turns P_t (pn, also in LDS) into P_{t-1}
      const float (*vec)[4][D] = vecs[s & 1];
      float cP[PPW][C::RB][C::KS], cBT[PPW][C::RB][C::KS], cFT[PPW][C::RB][C::KS];
      floatx4 aG[PPW];
      floatx4 accVT[PPW][C::RB][C::NT];
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        const floatx4 pt = get_row(Wm[q] + D, C::PITCH);  // P[i][4g+v]; pn holds P[4g+v][i]
        const float aI = vec[q][0][i], bI = vec[q][1][i];
        aG[q] = *reinterpret_cast<const floatx4*>(&vec[q][0][4 * g]);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          cP[q][0][v] = 0.5f * (pn[q][0][0][v] + pt[v]);   // symmetric part: both the rows of P as the A
                                                          // operand and P in the accumulator layout
          cBT[q][0][v] = Bbar[q][v] * bI;                  // B_t (column i scaled) = rows of B_t^T as the A operand
          pn[q][0][0][v] = aG[q][v] * cP[q][0][v] * aI;    // diag(a) P diag(a)
        }
        zero_acc<D>(accVT[q]);
      }
#pragma unroll
      for (int t = 0; t < 4; ++t)  // V^T = B_t^T P; P symmetric: its B operand is cP itself
#pragma unroll
        for (int q = 0; q < PPW; ++q)
          accVT[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(cBT[q][0][t], cP[q][0][t], accVT[q][0][0], 0, 0, 0);
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        const float aI = vec[q][0][i];
        put_acc(Vt[q], PT, accVT[q][0][0]);  // V^T[4g+v][i] = V[i][4g+v]
#pragma unroll
        for (int v = 0; v < 4; ++v) cFT[q][0][v] = aI * accVT[q][0][0][v];  // rows of F^T = diag(a) V
      }
      wave_lds_sync();
      floatx4 accW[PPW][C::RB][C::NT];
      {
        floatx4 accS[PPW][C::RB][C::NT];
        floatx4 bV[PPW];
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          bV[q] = get_row(Vt[q], PT);  // V[4g+t][i]
#pragma unroll
          for (int v = 0; v < 4; ++v) accS[q][0][0][v] = (4 * g + v == i) ? rI[q] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)  // S = R + B_t^T V
#pragma unroll
          for (int q = 0; q < PPW; ++q)
            accS[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(cBT[q][0][t], bV[q][t], accS[q][0][0], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          store_rows<D>(Wm[q], accS[q], w, i, g);
          if (s == 0 && ca.dual_g) put_acc(Vt[q], PT, accS[q][0][0]);  // S_0 once more below (V^T has been read)
        }
      }
      wave_lds_sync();
      tm.toc(2);
      note(invert_rows16<true, true>(Wmine, lane));  // left halves: -S^{-1}, so that the next product is the gain itself
      tm.toc(1);
      if (s == 0 && ca.dual_g) {
        // The dual problem of the backward pass starts from ut_0 = -S_0^{-1} g: y = S_0^{-1} g, refined once with the
        // residual g - S_0 y.  Lane (i, g) takes row i of its problem's -S_0^{-1} (Wm) and S_0 (Vt).
        float (*dv)[D] = vecs[1][gq];  // the other step's copy is free at s = 0: g, y, residual
        dv[0][i] = g_m;
        wave_lds_sync();
        auto row_dot = [&](const float* M, int pitch, const float* v) {
          float acc = 0.f;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const floatx4 m = *reinterpret_cast<const floatx4*>(M + i * pitch + 4 * c);
            const floatx4 x = *reinterpret_cast<const floatx4*>(v + 4 * c);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = __builtin_fmaf(m[e], x[e], acc);
          }
          return acc;
        };
        const float y = -row_dot(Wm[gq], C::PITCH, dv[0]);
        dv[1][i] = y;
        wave_lds_sync();
        dv[2][i] = g_m - row_dot(Vt[gq], PT, dv[1]);
        wave_lds_sync();
        const float ut0 = -(y - row_dot(Wm[gq], C::PITCH, dv[2]));
        if (quad * PPW + gq < p.n && (PPW == 4 || g == 0)) ca.roll_ws[(pg * slots + p.T + 3) * D * D + i] = ut0;
      }
      {
        float cSi[PPW][C::RB][C::KS];
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          load_aop_lds<D>(Wm[q], cSi[q], w, i, g);  // rows of -S^{-1}
          zero_acc<D>(accW[q]);
        }
        // cFT holds F^T in the A-operand layout, which is the accumulator layout of F: B operand of the gain
#pragma unroll
        for (int t = 0; t < 4; ++t)  // K = (-S^{-1}) F
#pragma unroll
          for (int q = 0; q < PPW; ++q)
            accW[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(cSi[q][0][t], cFT[q][0][t], accW[q][0][0], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t)  // P += F^T K: the accumulator layout of K is its B operand
#pragma unroll
          for (int q = 0; q < PPW; ++q)
            pn[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(cFT[q][0][t], accW[q][0][0][t], pn[q][0][0], 0, 0, 0);
      }
      if (ca.roll_ws) {  // the gain K_s of this step, for the forward sweep
#pragma unroll
        for (int q = 0; q < PPW; ++q)
          if (valid[q])
            write_rows_global<D>(ca.roll_ws + (prob[q] * slots + 3 + s) * D * D, accW[q][0], 0, i, g);
      }
      if (s >= 1) {
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          const float qI = vec[q][2][i];
          const floatx4 qG = *reinterpret_cast<const floatx4*>(&vec[q][2][4 * g]);
#pragma unroll
          for (int v = 0; v < 4; ++v) pn[q][0][0][v] += qG[v] * Qbar[q][v] * qI;  // + Q_{t-1}
          put_acc(Wm[q] + D, C::PITCH, pn[q][0][0]);
        }
        write_vec(s - 1);
        wave_lds_sync();
        tm.toc(2);
      } else {
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          put_acc(Wm[q] + D, C::PITCH, pn[q][0][0]);  // P_0 (no cost on x_0)
          put_acc(Vt[q], PT, accW[q][0][0]);          // K_0, row-major
        }
        vecs[1][gq][0][i] = x0_m;
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          const floatx4 pt = get_row(Wm[q] + D, C::PITCH);
#pragma unroll
          for (int v = 0; v < 4; ++v) pn[q][0][0][v] = 0.5f * (pn[q][0][0][v] + pt[v]);
          store_rows<D>(Wm[q], pn[q], w, i, g);  // symmetric P_0
        }
        wave_lds_sync();
        if (ca.roll_ws) {  // the roll-out wants the gains (written above) and info only
#pragma unroll
          for (int q = 0; q < PPW; ++q)
            if (valid[q] && tid == 0 && p.info) p.info[prob[q]] = info[q];
        } else {
          // All the wavefront's problems at once: lane (i, g) takes row i of its problem's K_0 and P_0 for
          // u_0 = K_0 x_0 and value = x_0^T P_0 x_0; the matrices leave as one 16-byte piece per lane and problem.
          const float nanv = __builtin_nanf("");
          const float* const xv = vecs[1][gq][0];
          float u = 0.f, pw = 0.f;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const floatx4 kr = *reinterpret_cast<const floatx4*>(Vt[gq] + i * PT + 4 * c);
            const floatx4 pr = *reinterpret_cast<const floatx4*>(Wm[gq] + i * C::PITCH + 4 * c);
            const floatx4 xr = *reinterpret_cast<const floatx4*>(xv + 4 * c);
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
                  info[q] ? nan4 : *reinterpret_cast<const floatx4*>(Vt[q] + (lane >> 2) * PT + 4 * (lane & 3));
            if (p.P0)
              *reinterpret_cast<floatx4*>(p.P0 + prob[q] * (long)D * D + 4 * lane) =
                  info[q] ? nan4 : *reinterpret_cast<const floatx4*>(Wm[q] + (lane >> 2) * C::PITCH + 4 * (lane & 3));
          }
        }
        wave_lds_sync();
        tm.toc(3);
      }
    }
    if (quad + gridDim.x >= nquads) tm.dump(p);
  }
}


// Closed-loop forward sweep of the structured problems (Alg. 1, forward loop, r = 0), 16 lanes per problem,
// lane i owning entry i of the state and of the control:  u_s = K_s x_s,  x_{s+1} = a_t x_s + Bbar (gamma_B^t u_s)
// (t = s + 1),  cost += u_s^T R u_s + x_{s+1}^T Q_t x_{s+1}  with  Q_t = Gamma_Q^t Qbar Gamma_Q^t  for t < T and Q_T.
template <typename TIn>
__global__ void __launch_bounds__(64) rollout_cxt_forward_kernel(const CxtRolloutArgs ra) {
  constexpr int D = 16;
  __shared__ float xs[4][D], us[4][D];
  const CxtArgs& ca = ra.c;
  const SolveArgs& p = ca.s;
  const int lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
  const long long ngroups = (p.n + 3) / 4;
  const float nanv = __builtin_nanf("");
  auto row_dot = [&](const float* M, const float* v) {  // sum_j M[i][j] v[j], M row-major in global memory
    float acc = 0.f;
#pragma unroll
    for (int j4 = 0; j4 < D; j4 += 4) {
      const floatx4 m = *reinterpret_cast<const floatx4*>(M + i * D + j4);
      acc += m[0] * v[j4] + m[1] * v[j4 + 1] + m[2] * v[j4 + 2] + m[3] * v[j4 + 3];
    }
    return acc;
  };
  for (long long grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
    const bool valid = grp * 4 + g < p.n;
    const long long prob = valid ? grp * 4 + g : p.n - 1;
    const float* const e = ca.roll_ws + prob * (long long)(ca.roll_slots ? ca.roll_slots : p.T + 3) * D * D;
    const float sA_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.sA), prob * D + i);
    const float lgA_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgA), prob * D + i);
    const float lgB_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgB), prob * D + i);
    const float lgQ_m = ld1<TIn>(reinterpret_cast<const TIn*>(ca.lgQ), prob * D + i);
    const float r_m = 1.f / ld1<TIn>(reinterpret_cast<const TIn*>(ca.rinv), prob * D + i);
    const bool bad = p.info && p.info[prob] != 0;
    float x = ld1<TIn>(reinterpret_cast<const TIn*>(p.x0), prob * p.sx0 + i);
    float cost = 0.f;
    if (valid && ra.X) ra.X[prob * (long long)(p.T + 1) * D + i] = bad ? nanv : x;
    for (int s = 0; s < p.T; ++s) {
      const float tf = -1.44269504f * (float)(s + 1);
      __syncthreads();  // the previous step's reads of xs, us are done
      xs[g][i] = x;
      __syncthreads();
      const float u = row_dot(e + (long long)(3 + s) * D * D, xs[g]);
      us[g][i] = __builtin_amdgcn_exp2f(tf * lgB_m) * u;
      __syncthreads();
      const float a = 1.f + __builtin_amdgcn_exp2f(tf * lgA_m) * sA_m;
      x = a * x + row_dot(e, us[g]);
      __syncthreads();  // reads of xs are done
      const bool last = (s == p.T - 1);
      const float y = last ? x : __builtin_amdgcn_exp2f(tf * lgQ_m) * x;
      xs[g][i] = y;
      __syncthreads();
      const float qy = row_dot(last ? e + 2 * D * D : e + D * D, xs[g]);
      cost += sum16(u * u * r_m + y * qy);
      if (valid) {
        ra.U[(prob * (long long)p.T + s) * D + i] = bad ? nanv : u;
        if (ra.X) ra.X[(prob * (long long)(p.T + 1) + s + 1) * D + i] = bad ? nanv : x;
      }
    }
    if (valid && i == 0 && ra.cost) ra.cost[prob] = bad ? nanv : cost;
    __syncthreads();
  }
}

}  // namespace ttc
