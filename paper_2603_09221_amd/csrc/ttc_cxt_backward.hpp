// Backward pass of the structured, contextualised problems (ttc_lqr_backward_cxt; Thm 3.2 and Sec. 4,
// "Contextualization", "Parameterization"): the gradients of a loss of u_0 with respect to the per-problem vectors
// (the log-scale modulation coefficients and the diagonal of R^{-1} among them), x0 and the shared basis matrices.
//
// Three launches per chunk of problems:
//   solve_cxt_kernel         the backward recursion of the forward pass again (ttc_cxt.hpp), leaving per problem
//                            Bbar, Qbar, Q_T, every gain K_s and the dual problem's first control in the workspace
//   backward_cxt_vec_kernel  both closed loops, both co-state recursions and the gradients, on vectors (below)
//   cxt_basis_kernel         the bases' gradients: sums over the problems of the chunk, added to the caller's arrays
// With t = 1..T, gam_X^t = exp(-t lg_X), Bbar = sum_k sB_k B^(k), Qbar = sum_k sQ_k Q^(k), and the per-step gradients
// of Thm 3.2, gA_t = lam_t xt_{t-1}^T + lamt_t x_{t-1}^T, gB_t = lam_t ut_t^T + lamt_t u_t^T, gQ_t = sym(xt_t x_t^T),
// gR_t = sym(ut_t u_t^T) (primal x, u, lam; dual xt, ut, lamt):
//   A_t = I + diag(gam_A^t sA):            dsA_i = sum_t gam_A,i^t gA_t[i,i],   dlgA_i = sum_t -t gam_A,i^t sA_i gA_t[i,i]
//   B_t = Bbar diag(gam_B^t):              dBbar = sum_t gB_t diag(gam_B^t),    dlgB_j = sum_t -t gam_B,j^t sum_i Bbar[i,j] gB_t[i,j]
//   Q_t = diag(gam_Q^t) Qbar diag(gam_Q^t) (t < T):  dQbar = sum_t diag(gam_Q^t) gQ_t diag(gam_Q^t),
//                                          dlgQ_i = sum_t -2 t sum_j Q_t[i,j] gQ_t[i,j]   (both symmetric)
//   Q_T = sum_k sQf_k Q^(k):               dQ_T = gQ_T;      R_t = diag(1/rinv):  drinv_i = -sum_t gR_t[i,i] / rinv_i^2
//   dsB_k = <B^(k), dBbar>, dsQ_k = <Q^(k), dQbar>, dsQf_k = <Q^(k), dQ_T>;
//   dB^(k) = sum_p sB_k dBbar,  dQ^(k) = sum_p (sQ_k dQbar + sQf_k dQ_T).
#pragma once
#include "ttc_common.hpp"

namespace ttc {

// Row i (sixteen numbers) of a row-major 16 x 16 matrix in global memory.
struct Row16 {
  floatx4 v[4];
};
template <typename T>
__device__ __forceinline__ Row16 load_row16(const T* M, int i) {
  Row16 r;
#pragma unroll
  for (int c = 0; c < 4; ++c) r.v[c] = ld4<T>(M, (long)i * 16 + 4 * c);
  return r;
}
// <row, v> and <row, w> for two vectors in LDS
__device__ __forceinline__ void row_dot2(const Row16& m, const float* va, const float* vc, float& ya, float& yc) {
  float sa = 0.f, sc = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sa = __builtin_fmaf(m.v[c][e], va[4 * c + e], sa);
      sc = __builtin_fmaf(m.v[c][e], vc[4 * c + e], sc);
    }
  }
  ya = sa;
  yc = sc;
}
__device__ __forceinline__ float row_dot(const Row16& m, const float* va) {
  float sa = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) sa = __builtin_fmaf(m.v[c][e], va[4 * c + e], sa);
  }
  return sa;
}

// The backward pass proper, on vectors: sixteen lanes per problem (four problems per wavefront), lane i owning entry
// i of every vector and row i of every 16 x 16 matrix it accumulates.  solve_cxt_kernel has left, per problem,
// Bbar, Qbar, Q_T, the gains K_0 .. K_{T-1} and ut_0.  Forward: both closed loops (Alg. 1; the dual one starts from
// the state 0 with ut_0 = -S_0^{-1} g), states and scaled controls to the workspace, or to LDS when the horizon is
// short (a.traj_in_lds).  Backward: the co-states of both (Alg. 2) with A_t diagonal and Q_t = Gamma^t Qbar Gamma^t,
// and in the same sweep the gradients of Thm 3.2 contracted straight onto the parameterisation: no per-step gradient
// matrix is ever formed.  Every step is a short chain of dependent operations: gains are requested four steps at a
// time, and the lanes of a problem exchange vectors through LDS with an ordering point that does not wait for loads
// in flight.  The four wavefronts of a workgroup work independently (each on its own groups of four problems, with
// its own LDS areas); what they share is a copy of the basis matrices in LDS (a.basis_in_lds: r <= 16), which the
// inner products at the end read instead of going to memory once per problem.
constexpr int CXT_BWD_LDS_R = 16;  // most basis matrices per group kept in LDS
constexpr int CXT_BWD_LDS_T = 8;   // longest horizon whose trajectories stay in LDS
template <typename TIn>
__global__ void __launch_bounds__(256, 2) backward_cxt_vec_kernel(const CxtBackwardArgs a) {
  constexpr int D = 16;
  __shared__ __attribute__((aligned(16))) float vb_all[4][4][4][D];  // per wavefront and problem: vectors every lane of the problem reads
  __shared__ __attribute__((aligned(16))) float traj_all[4][4 * 4 * (CXT_BWD_LDS_T + 1) * D];
  __shared__ __attribute__((aligned(16))) float basis_lds[2 * CXT_BWD_LDS_R * D * D];  // Bbasis, then Qbasis
  const SolveArgs& p = a.c.s;
  const int T = p.T, r = a.c.r;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
  const long long slots = T + 4;
  const long long ngroups = (a.count + 3) / 4;
  const float nanv = __builtin_nanf("");
  const TIn* const Bb = reinterpret_cast<const TIn*>(a.c.Bbasis);
  const TIn* const Qb = reinterpret_cast<const TIn*>(a.c.Qbasis);
  if (a.basis_in_lds) {
    for (int k = threadIdx.x; k < r * D * D; k += 256) {
      basis_lds[k] = ld1<TIn>(Bb, k);
      basis_lds[r * D * D + k] = ld1<TIn>(Qb, k);
    }
  }
  __syncthreads();  // the only barrier: from here on a wavefront touches its own LDS areas and reads the bases
  float (*const vb)[4][D] = vb_all[w];
  float* const traj_lds = traj_all[w];
  float* const v0 = vb[g][0];
  float* const v1 = vb[g][1];
  float* const v2 = vb[g][2];
  float* const v3 = vb[g][3];
  PhaseTimers tm;  // phases: 4 first loads and step 0, 5 forward, 6 backward, 7 outputs (0..3 belong to the solve kernel)
  for (long long grp = blockIdx.x * 4LL + w; grp < ngroups; grp += gridDim.x * 4LL) {
    const bool valid = grp * 4 + g < a.count;
    const long long q = valid ? grp * 4 + g : a.count - 1;  // within the chunk
    const long long prob = a.first + q;                      // within the batch
    const float* const e = a.roll + q * slots * D * D;
    float* const tX = a.traj_in_lds ? traj_lds + g * 4 * (T + 1) * D : a.traj + q * 4 * (long long)(T + 1) * D;
    float* const tXt = tX + (long long)(T + 1) * D;
    float* const tU = tXt + (long long)(T + 1) * D;
    float* const tUt = tU + (long long)(T + 1) * D;
    // everything the first steps need is requested at once
    const Row16 bbr = load_row16(e, i);                                   // Bbar
    float ut = e[(long long)(T + 3) * D * D + i];                         // ut_0
    const float sA_m = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sA), prob * D + i);
    const float lgA_m = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgA), prob * D + i);
    const float lgB_m = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgB), prob * D + i);
    const float lgQ_m = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgQ), prob * D + i);
    const float rinv_m = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.rinv), prob * D + i);
    float x = ld1<TIn>(reinterpret_cast<const TIn*>(p.x0), prob * D + i), xt = 0.f;
    const bool bad = a.info && a.info[prob] != 0;
    float bb[D];  // row i of Bbar
#pragma unroll
    for (int j = 0; j < D; ++j) bb[j] = bbr.v[j >> 2][j & 3];

    // ---- forward: both closed loops
    // Four steps' gains are requested together (one wait per four steps instead of one per step); with the last
    // ones come the rows of Q_T and Qbar for the co-states.
    float u = 0.f, dR = 0.f;
    Row16 qtr = bbr, qqr = bbr;
    for (int s0 = 0; s0 < T; s0 += 4) {
      Row16 kb[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int sk = s0 + k < T ? s0 + k : T - 1;
        kb[k] = load_row16(e + (long long)(3 + sk) * D * D, i);
      }
      if (s0 + 4 >= T) {
        qtr = load_row16(e + 2 * D * D, i);
        qqr = load_row16(e + D * D, i);
      }
      if (s0 == 0) tm.toc(4);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int s = s0 + k;
        if (s >= T) break;
        const float tf = -1.44269504f * (float)(s + 1);
        wave_lds_sync();
        v0[i] = x;
        v1[i] = xt;
        wave_lds_sync();
        if (s > 0) row_dot2(kb[k], v0, v1, u, ut);  // u_s = K_s x_s, both loops
        else u = row_dot(kb[k], v0);               // u_0 = K_0 x_0 (ut_0 came with the matrices)
        const float gb = __builtin_amdgcn_exp2f(tf * lgB_m);
        const float us = gb * u, uts = gb * ut;  // the controls as B_t sees them, gamma_B^t u: also what dl/dBbar needs
        dR = __builtin_fmaf(ut, u, dR);          // dl/dR_t [i][i]
        tX[(long long)s * D + i] = x;
        tXt[(long long)s * D + i] = xt;
        tU[(long long)s * D + i] = us;
        tUt[(long long)s * D + i] = uts;
        wave_lds_sync();
        v2[i] = us;
        v3[i] = uts;
        wave_lds_sync();
        const float am = 1.f + __builtin_amdgcn_exp2f(tf * lgA_m) * sA_m;
        float bu = 0.f, but = 0.f;
#pragma unroll
        for (int j = 0; j < D; ++j) {
          bu = __builtin_fmaf(bb[j], v2[j], bu);
          but = __builtin_fmaf(bb[j], v3[j], but);
        }
        x = am * x + bu;
        xt = am * xt + but;
      }
    }
    tX[(long long)T * D + i] = x;
    tXt[(long long)T * D + i] = xt;
    tm.toc(5);

    // ---- backward: co-states, and the gradients of every step as they become available.  Iteration t (the paper's
    // step t, s = t - 1) takes lam_t and, in one exchange of four vectors, the scaled controls gamma_B^t u_s (for
    // dl/dB_t) and the scaled states gamma_Q^s x_s (for dl/dQ_s and for lam_s = Q_s x_s + a_t lam_t); with
    // B_t = Bbar Gamma_B^t and Q_s = Gamma_Q^s Qbar Gamma_Q^s the modulation factors are then already in place:
    //   dBbar[i][j] += lam_i ut'_j + lamt_i u'_j =: incB,   dlgB_j += -t Bbar[i][j] incB   (summed over i at the end)
    //   2 dQbar[i][j] += xt'_i x'_j + x'_i xt'_j =: incQ,   dlgQ_i += -s sum_j Qbar[i][j] incQ
    float nxs = tX[(long long)(T - 1) * D + i], nxts = tXt[(long long)(T - 1) * D + i];
    float nus = tU[(long long)(T - 1) * D + i], nuts = tUt[(long long)(T - 1) * D + i];
    float lam, lamt;
    wave_lds_sync();
    v0[i] = x;
    v1[i] = xt;
    wave_lds_sync();
    row_dot2(qtr, v0, v1, lam, lamt);  // lam_T = Q_T x_T
    float qq[D];
#pragma unroll
    for (int j = 0; j < D; ++j) qq[j] = qqr.v[j >> 2][j & 3];
    float dsA = 0.f, dlgA = 0.f, dlgQ = 0.f;
    float dB[D], dQ[D], dQf[D], cB[D];  // dQ holds twice dl/dQbar, cB holds dl/dlgB's terms without their Bbar[i][j]
#pragma unroll
    for (int j = 0; j < D; ++j) {
      dB[j] = dQ[j] = cB[j] = 0.f;
      dQf[j] = 0.5f * (xt * v0[j] + x * v1[j]);  // dl/dQ_T [i][j], symmetric
    }
    for (int t = T; t >= 1; --t) {
      const int s = t - 1;
      const float tf = -1.44269504f * (float)t, tt = (float)t;
      const float xs = nxs, xts = nxts, us = nus, uts = nuts;
      if (s >= 1) {  // the stored step before, for the next iteration
        nxs = tX[(long long)(s - 1) * D + i];
        nxts = tXt[(long long)(s - 1) * D + i];
        nus = tU[(long long)(s - 1) * D + i];
        nuts = tUt[(long long)(s - 1) * D + i];
      }
      const float gamA = __builtin_amdgcn_exp2f(tf * lgA_m);
      const float gq1 = __builtin_amdgcn_exp2f(-1.44269504f * (float)s * lgQ_m);
      const float xq = gq1 * xs, xtq = gq1 * xts;  // gamma_Q^s x_s
      wave_lds_sync();
      v0[i] = us;
      v1[i] = uts;
      v2[i] = xq;
      v3[i] = xtq;
      wave_lds_sync();
      const float gAii = lam * xts + lamt * xs;
      dsA = __builtin_fmaf(gamA, gAii, dsA);
      dlgA = __builtin_fmaf(-tt * gamA * sA_m, gAii, dlgA);
      const float am = 1.f + gamA * sA_m;
      if (s >= 1) {
        float hq = 0.f, qa = 0.f, qc = 0.f;
#pragma unroll
        for (int j = 0; j < D; ++j) {
          const float incB = __builtin_fmaf(lam, v1[j], lamt * v0[j]);
          dB[j] += incB;
          cB[j] = __builtin_fmaf(-tt, incB, cB[j]);
          const float incQ = __builtin_fmaf(xtq, v2[j], xq * v3[j]);
          dQ[j] += incQ;
          hq = __builtin_fmaf(qq[j], incQ, hq);
          qa = __builtin_fmaf(qq[j], v2[j], qa);
          qc = __builtin_fmaf(qq[j], v3[j], qc);
        }
        dlgQ = __builtin_fmaf(-(float)s, hq, dlgQ);
        lam = gq1 * qa + am * lam;  // lam_s = Q_s x_s + a_t lam_t
        lamt = gq1 * qc + am * lamt;
      } else {  // s = 0: no cost on x_0; lamt_0 = a_1 lamt_1 is dl/dx_0
#pragma unroll
        for (int j = 0; j < D; ++j) {
          const float incB = __builtin_fmaf(lam, v1[j], lamt * v0[j]);
          dB[j] += incB;
          cB[j] = __builtin_fmaf(-tt, incB, cB[j]);
        }
        lamt = am * lamt;
      }
    }
#pragma unroll
    for (int j = 0; j < D; ++j) {
      dQ[j] *= 0.5f;
      cB[j] *= bb[j];
    }
    tm.toc(6);
    // ---- outputs
    if (valid) {
      a.gx0[prob * D + i] = bad ? nanv : lamt;
      a.gsA[prob * D + i] = bad ? nanv : dsA;
      a.glgA[prob * D + i] = bad ? nanv : dlgA;
      a.glgQ[prob * D + i] = bad ? nanv : dlgQ;
      a.grinv[prob * D + i] = bad ? nanv : -dR / (rinv_m * rinv_m);
    }
    {  // dl/dlgB_j: the column sums of cB over the problem's lanes
      float mine = 0.f;
#pragma unroll
      for (int j = 0; j < D; ++j) {
        const float sj = sum16(cB[j]);
        mine = (i == j) ? sj : mine;
      }
      if (valid) a.glgB[prob * D + i] = bad ? nanv : mine;
    }
    if (valid) {  // rows of dl/dBbar, dl/dQbar, dl/dQ_T for the bases' sums
      float* const keep = a.keep + q * 768;
#pragma unroll
      for (int j4 = 0; j4 < D; j4 += 4) {
        const float f = bad ? nanv : 1.f;
        *reinterpret_cast<floatx4*>(keep + i * D + j4) = floatx4{dB[j4] * f, dB[j4 + 1] * f, dB[j4 + 2] * f, dB[j4 + 3] * f};
        *reinterpret_cast<floatx4*>(keep + 256 + i * D + j4) = floatx4{dQ[j4] * f, dQ[j4 + 1] * f, dQ[j4 + 2] * f, dQ[j4 + 3] * f};
        *reinterpret_cast<floatx4*>(keep + 512 + i * D + j4) = floatx4{dQf[j4] * f, dQf[j4 + 1] * f, dQf[j4 + 2] * f, dQf[j4 + 3] * f};
      }
    }
    float msb = 0.f, msq = 0.f, msf = 0.f;
    for (int k0 = 0; k0 < r; k0 += 4) {  // the inner products with the basis matrices, four matrices' rows per wait
      Row16 bk[4], qk[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int k = k0 + kk < r ? k0 + kk : r - 1;
        if (a.basis_in_lds) {
          bk[kk] = load_row16(basis_lds + k * 256, i);
          qk[kk] = load_row16(basis_lds + (r + k) * 256, i);
        } else {
          bk[kk] = load_row16(Bb + (long)k * 256, i);
          qk[kk] = load_row16(Qb + (long)k * 256, i);
        }
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int k = k0 + kk;
        if (k >= r) break;
        float sb = 0.f, sq = 0.f, sf = 0.f;
#pragma unroll
        for (int j = 0; j < D; ++j) {
          sb = __builtin_fmaf(bk[kk].v[j >> 2][j & 3], dB[j], sb);
          sq = __builtin_fmaf(qk[kk].v[j >> 2][j & 3], dQ[j], sq);
          sf = __builtin_fmaf(qk[kk].v[j >> 2][j & 3], dQf[j], sf);
        }
        sb = sum16(sb);
        sq = sum16(sq);
        sf = sum16(sf);
        // lane k mod 16 keeps the three numbers of matrix k; sixteen matrices leave with one store per array
        const bool mine = (k & 15) == i;
        msb = mine ? sb : msb;
        msq = mine ? sq : msq;
        msf = mine ? sf : msf;
        if ((k & 15) == 15 || k == r - 1) {
          if (valid && i <= (k & 15)) {
            const long long o = prob * r + (k & ~15) + i;
            a.gsB[o] = bad ? nanv : msb;
            a.gsQ[o] = bad ? nanv : msq;
            a.gsQf[o] = bad ? nanv : msf;
          }
        }
      }
    }
    wave_lds_sync();
    tm.toc(7);
  }
  tm.dump(p);
}

// gBbasis[k] += sum_p sB[p][k] dBbar[p], gQbasis[k] += sum_p (sQ[p][k] dQbar[p] + sQf[p][k] dQ_T[p]) over a slab of
// a.basis_slab of the chunk's problems per workgroup; thread e owns entry e of every basis matrix, the sums of a slab are added to the
// caller's arrays with one atomic addition per entry (the order of the slabs, and with it the last bits, may vary).
template <typename TIn>
__global__ void __launch_bounds__(256) cxt_basis_kernel(const CxtBackwardArgs a) {
  const int e = threadIdx.x;
  const int r = a.c.r;
  const long long q0 = (long long)blockIdx.x * a.basis_slab;
  long long q1 = q0 + a.basis_slab;
  q1 = q1 < a.count ? q1 : a.count;
  for (int k0 = 0; k0 < r; k0 += 16) {  // sixteen basis matrices of each group at a time (registers)
    float sb[16], sq[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) sb[k] = sq[k] = 0.f;
    // Lane 16 g + k of every wavefront reads coefficient k0 + k of group g (sB, sQ, sQf) with one load per problem
    // and the others take it from that lane; the next problem's values are fetched while this one's products are
    // formed.
    const int lane = threadIdx.x & 63, grp = lane >> 4, kk = k0 + (lane & 15);
    const TIn* const cbase = reinterpret_cast<const TIn*>(grp == 0 ? a.c.sB : grp == 1 ? a.c.sQ : a.c.sQf);
    const bool cread = grp < 3 && kk < r;
    float nB = 0.f, nQ = 0.f, nF = 0.f, nC = 0.f;
    if (q0 < q1) {
      const float* keep = a.keep + q0 * 768;
      nB = keep[e]; nQ = keep[256 + e]; nF = keep[512 + e];
      if (cread) nC = ld1<TIn>(cbase, (a.first + q0) * r + kk);
    }
    for (long long q = q0; q < q1; ++q) {
      const float dBbar = nB, dQbar = nQ, dQf = nF, cv = nC;
      if (q + 1 < q1) {
        const float* keep = a.keep + (q + 1) * 768;
        nB = keep[e]; nQ = keep[256 + e]; nF = keep[512 + e];
        if (cread) nC = ld1<TIn>(cbase, (a.first + q + 1) * r + kk);
      }
#pragma unroll
      for (int k = 0; k < 16; ++k) {  // coefficients past r were read as zero
        sb[k] = __builtin_fmaf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cv), k)), dBbar, sb[k]);
        sq[k] = __builtin_fmaf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cv), 16 + k)), dQbar, sq[k]);
        sq[k] = __builtin_fmaf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cv), 32 + k)), dQf, sq[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      if (k0 + k < r) {
        atomicAdd(a.gBbasis + (long)(k0 + k) * 256 + e, sb[k]);
        atomicAdd(a.gQbasis + (long)(k0 + k) * 256 + e, sq[k]);
      }
    }
  }
}

__global__ void __launch_bounds__(256) zero_floats_kernel(float* dst, long long n) {
  for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < n; k += (long long)gridDim.x * 256) dst[k] = 0.f;
}

}  // namespace ttc
