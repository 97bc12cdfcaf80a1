// Backward pass of the structured, contextualised problems (ttc_lqr_backward_cxt; Thm 3.2 and Sec. 4,
// "Contextualization", "Parameterization"): the gradients of a loss of u_0 with respect to the per-problem vectors
// (the log-scale modulation coefficients and the diagonal of R^{-1} among them), x0 and the shared basis matrices.
//
// The per-step gradients are those of the time-heterogeneous backward kernel (ttc_backward.hpp), which this path
// runs on the problems' steps written out densely, a chunk of problems at a time, between two small kernels:
//   cxt_expand_kernel    the T steps (A_t, B_t, Q_t, R_t) of every problem of the chunk, float32, into the workspace
//   backward_kernel<16>  gA_t, gB_t, gQ_t, gR_t of every step into the workspace; gx0, info straight to the caller
//   cxt_contract_kernel  the chain rule from the steps to the problem's vectors; dl/dBbar, dl/dQbar, dl/dQ_T kept
//   cxt_basis_kernel     the bases' gradients: sums over the problems of the chunk, added to the caller's arrays
// With t = 1..T, gam_X^t = exp(-t lg_X), Bbar = sum_k sB_k B^(k), Qbar = sum_k sQ_k Q^(k):
//   A_t = I + diag(gam_A^t sA):            dsA_i = sum_t gam_A,i^t gA_t[i,i],   dlgA_i = sum_t -t gam_A,i^t sA_i gA_t[i,i]
//   B_t = Bbar diag(gam_B^t):              dBbar = sum_t gB_t diag(gam_B^t),    dlgB_j = sum_t -t gam_B,j^t sum_i Bbar[i,j] gB_t[i,j]
//   Q_t = diag(gam_Q^t) Qbar diag(gam_Q^t) (t < T):  dQbar = sum_t diag(gam_Q^t) gQ_t diag(gam_Q^t),
//                                          dlgQ_i = sum_t -t (row i + column i sums of Q_t o gQ_t)
//   Q_T = sum_k sQf_k Q^(k):               dQ_T = gQ_T;      R_t = diag(1/rinv):  drinv_i = -sum_t gR_t[i,i] / rinv_i^2
//   dsB_k = <B^(k), dBbar>, dsQ_k = <Q^(k), dQbar>, dsQf_k = <Q^(k), dQ_T>;
//   dB^(k) = sum_p sB_k dBbar,  dQ^(k) = sum_p (sQ_k dQbar + sQf_k dQ_T).
#pragma once
#include "ttc_common.hpp"

namespace ttc {

// a workgroup of 256 threads per problem, thread e = 16 i + j owning entry (i, j) of every matrix
template <typename TIn>
__global__ void __launch_bounds__(256) cxt_expand_kernel(const CxtBackwardArgs a) {
  const int e = threadIdx.x, i = e >> 4, j = e & 15;
  const int r = a.c.r, T = a.c.s.T;
  const TIn* const Bb = reinterpret_cast<const TIn*>(a.c.Bbasis);
  const TIn* const Qb = reinterpret_cast<const TIn*>(a.c.Qbasis);
  for (long long q = blockIdx.x; q < a.count; q += gridDim.x) {
    const long long p = a.first + q;
    float bbar = 0.f, qbar = 0.f, qf = 0.f;
    for (int k = 0; k < r; ++k) {
      const float bk = ld1<TIn>(Bb, (long)k * 256 + e), qk = ld1<TIn>(Qb, (long)k * 256 + e);
      bbar = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sB), p * r + k), bk, bbar);
      qbar = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sQ), p * r + k), qk, qbar);
      qf = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sQf), p * r + k), qk, qf);
    }
    const float sA_i = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sA), p * 16 + i);
    const float lgA_i = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgA), p * 16 + i);
    const float lgB_j = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgB), p * 16 + j);
    const float lgQ_i = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgQ), p * 16 + i);
    const float lgQ_j = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgQ), p * 16 + j);
    const float rdiag = 1.f / ld1<TIn>(reinterpret_cast<const TIn*>(a.c.rinv), p * 16 + i);
    if (e < 16) a.x0f[q * 16 + e] = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.s.x0), p * 16 + e);
    for (int t = 1; t <= T; ++t) {
      const long long at = (q * T + (t - 1)) * 256 + e;
      a.dA[at] = i == j ? 1.f + expf(-(float)t * lgA_i) * sA_i : 0.f;
      a.dB[at] = bbar * expf(-(float)t * lgB_j);
      a.dQ[at] = t == T ? qf : expf(-(float)t * lgQ_i) * qbar * expf(-(float)t * lgQ_j);
      a.dR[at] = i == j ? rdiag : 0.f;
    }
  }
}

template <typename TIn>
__global__ void __launch_bounds__(256) cxt_contract_kernel(const CxtBackwardArgs a) {
  __shared__ float M[3][256];     // reductions over rows or columns; then dl/dBbar, dl/dQbar, dl/dQ_T
  const int e = threadIdx.x, i = e >> 4, j = e & 15;
  const int r = a.c.r, T = a.c.s.T;
  const TIn* const Bb = reinterpret_cast<const TIn*>(a.c.Bbasis);
  const TIn* const Qb = reinterpret_cast<const TIn*>(a.c.Qbasis);
  for (long long q = blockIdx.x; q < a.count; q += gridDim.x) {
    const long long p = a.first + q;
    float bbar = 0.f, qbar = 0.f;
    for (int k = 0; k < r; ++k) {
      bbar = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sB), p * r + k), ld1<TIn>(Bb, (long)k * 256 + e), bbar);
      qbar = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sQ), p * r + k), ld1<TIn>(Qb, (long)k * 256 + e), qbar);
    }
    const float sA_i = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sA), p * 16 + i);
    const float lgA_i = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgA), p * 16 + i);
    const float lgB_j = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgB), p * 16 + j);
    const float lgQ_i = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgQ), p * 16 + i);
    const float lgQ_j = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.lgQ), p * 16 + j);
    const float rinv_i = ld1<TIn>(reinterpret_cast<const TIn*>(a.c.rinv), p * 16 + i);
    float dsA = 0.f, dlgA = 0.f, dR = 0.f;      // used by the diagonal threads
    float dBbar = 0.f, dQbar = 0.f, dQf = 0.f;  // entry (i, j)
    float colB = 0.f, hadQ = 0.f;               // entry (i, j) of the sums that are reduced below
    for (int t = 1; t <= T; ++t) {
      const long long at = (q * T + (t - 1)) * 256 + e;
      const float ga = a.gA[at], gb = a.gB[at], gq = a.gQ[at], gr = a.gR[at];
      const float tf = (float)t;
      const float gamA = expf(-tf * lgA_i), gamB = expf(-tf * lgB_j), gamQ = expf(-tf * lgQ_i) * expf(-tf * lgQ_j);
      dsA = __builtin_fmaf(gamA, ga, dsA);
      dlgA = __builtin_fmaf(-tf * gamA * sA_i, ga, dlgA);
      dR += gr;
      dBbar = __builtin_fmaf(gamB, gb, dBbar);
      colB = __builtin_fmaf(-tf * gamB * bbar, gb, colB);
      if (t < T) {
        dQbar = __builtin_fmaf(gamQ, gq, dQbar);
        hadQ = __builtin_fmaf(-tf * gamQ * qbar, gq, hadQ);
      } else {
        dQf = gq;
      }
    }
    if (i == j) {
      a.gsA[p * 16 + i] = dsA;
      a.glgA[p * 16 + i] = dlgA;
      a.grinv[p * 16 + i] = -dR / (rinv_i * rinv_i);
    }
    __syncthreads();  // M is free (the previous problem's readers are done)
    M[0][e] = colB;
    M[1][e] = hadQ;
    __syncthreads();
    if (e < 16) {          // dlgB_j: column sums
      float s = 0.f;
#pragma unroll
      for (int ii = 0; ii < 16; ++ii) s += M[0][16 * ii + e];
      a.glgB[p * 16 + e] = s;
    } else if (e < 32) {   // dlgQ_i: row i plus column i
      const int c = e - 16;
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < 16; ++k) s += M[1][16 * c + k] + M[1][16 * k + c];
      a.glgQ[p * 16 + c] = s;
    }
    __syncthreads();
    M[0][e] = dBbar;
    M[1][e] = dQbar;
    M[2][e] = dQf;
    float* const keep = a.keep + q * 768;
    keep[e] = dBbar;
    keep[256 + e] = dQbar;
    keep[512 + e] = dQf;
    __syncthreads();
    // the 3 r inner products with the basis matrices: a wavefront per product, four entries per lane
    for (int o = e >> 6; o < 3 * r; o += 4) {
      const int which = o / r, k = o % r, lane = e & 63;
      const TIn* basis = which == 0 ? Bb : Qb;
      float s = 0.f;
#pragma unroll
      for (int x = 0; x < 4; ++x) s = __builtin_fmaf(ld1<TIn>(basis, (long)k * 256 + lane + 64 * x), M[which][lane + 64 * x], s);
#pragma unroll
      for (int sh = 1; sh < 64; sh <<= 1) s += __shfl_xor(s, sh, 64);
      float* dst = which == 0 ? a.gsB : which == 1 ? a.gsQ : a.gsQf;
      if (lane == 0) dst[p * r + k] = s;
    }
  }
}

// gBbasis[k] += sum_p sB[p][k] dBbar[p], gQbasis[k] += sum_p (sQ[p][k] dQbar[p] + sQf[p][k] dQ_T[p]) over a slab of
// the chunk's problems per workgroup; thread e owns entry e of every basis matrix, the sums of a slab are added to the
// caller's arrays with one atomic addition per entry (the order of the slabs, and with it the last bits, may vary).
constexpr int CXT_BASIS_SLAB = 32;
template <typename TIn>
__global__ void __launch_bounds__(256) cxt_basis_kernel(const CxtBackwardArgs a) {
  const int e = threadIdx.x;
  const int r = a.c.r;
  const long long q0 = (long long)blockIdx.x * CXT_BASIS_SLAB;
  long long q1 = q0 + CXT_BASIS_SLAB;
  q1 = q1 < a.count ? q1 : a.count;
  for (int k0 = 0; k0 < r; k0 += 16) {  // sixteen basis matrices of each group at a time (registers)
    float sb[16], sq[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) sb[k] = sq[k] = 0.f;
    for (long long q = q0; q < q1; ++q) {
      const long long p = a.first + q;
      const float* keep = a.keep + q * 768;
      const float dBbar = keep[e], dQbar = keep[256 + e], dQf = keep[512 + e];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        if (k0 + k < r) {
          sb[k] = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sB), p * r + k0 + k), dBbar, sb[k]);
          sq[k] = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sQ), p * r + k0 + k), dQbar, sq[k]);
          sq[k] = __builtin_fmaf(ld1<TIn>(reinterpret_cast<const TIn*>(a.c.sQf), p * r + k0 + k), dQf, sq[k]);
        }
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
