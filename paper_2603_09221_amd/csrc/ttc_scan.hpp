// Time-heterogeneous problems with the backward recursion taken as a tree over the horizon.
//
// One backward step of Prop. 3.1, with G_s = B_s R_s^{-1} B_s^T (the G_t of Thm 3.3), is the map
//     f_e(P) = H_e + A_e^T P (I + G_e P)^{-1} A_e        of the element e = (A_e, G_e, H_e) = (A_s, G_s, Q_{s-1}),
// the symplectic transfer matrix Sigma_t of Thm 3.3 in a form that needs no A^{-1}.  The maps are closed
// under composition: with e1 the earlier step, f_{e1} o f_{e2} = f_e for
//     M = (I + G_1 H_2)^{-1},   A = A_2 M A_1,   G = G_2 + A_2 M G_1 A_2^T,   H = H_1 + A_1^T H_2 M A_1,
// and composition is associative, so the product of the T factors, which the paper forms one factor
// after the other (Sec. 3.3), can be formed pairwise in ceil(log2 T) rounds, every round one launch over
// all pairs of all problems.  The terminal cost enters as one more element, the constant map
// (0, 0, Q_T): composed on the right of the steps s = 1..T-1 it leaves H = P_1 in the first element.
// The step s = 0, which also yields the gain, is then taken as printed (riccati_step).
//
// Elements live in the workspace as plain row-major fp32 matrices, element k of problem p at
// ws + ((p*T + k)*3) d^2: A, G, H; k = 0..T-2 is step s = k+1, k = T-1 the terminal element.
// A round with stride st rewrites element j (j a multiple of 2 st) as e_j o e_{j+st}; no other element
// is written in that round.  A breakdown (R_s not positive definite, I + G_1 H_2 singular) poisons the H it
// produces with NaN, which the last step turns into info = 1 and NaN outputs for that problem alone.
#pragma once
#include "ttc_common.hpp"
#include "ttc_doubling.hpp"
#include "ttc_tv.hpp"

namespace ttc {


template <int D>
__device__ __forceinline__ void poison(floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT]) {
  const float nanv = __builtin_nanf("");
#pragma unroll
  for (int rb = 0; rb < Cfg<D>::RB; ++rb)
#pragma unroll
    for (int c = 0; c < Cfg<D>::NT; ++c) acc[rb][c] = floatx4{nanv, nanv, nanv, nanv};
}

// the elements of every step of every problem
template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) scan_leaf_kernel(const ScanArgs a) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  const SolveArgs& p = a.tv.s;
  float* const WL = W;
  float* const WR = W + D;
  const long long items = p.n * p.T;
  for (long long item = blockIdx.x; item < items; item += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
    const long long prob = item / p.T;
    const int k = (int)(item % p.T);
    float* const gA = a.ws + item * 3 * D * D;
    float* const gG = gA + D * D;
    float* const gH = gG + D * D;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ + (long long)k * a.tv.tQ;  // Q[k] = Q_{s-1}, s = k+1
    floatx4 acc[C::RB][C::NT];
    load_half<D, TIn, false>(WL, Qp, tid);
    __syncthreads();
    symmetrise_half<D>(WL, tid);
    __syncthreads();
    store_half_global<D>(gH, WL, tid);
    if (k == p.T - 1) {  // the terminal element (0, 0, Q_T)
      zero_acc<D>(acc);
      write_rows_global<D>(gA, acc, w, i, g);
      write_rows_global<D>(gG, acc, w, i, g);
      __syncthreads();
      continue;
    }
    const int s = k + 1;
    const TIn* As = reinterpret_cast<const TIn*>(p.A) + prob * p.sA + (long long)s * a.tv.tA;
    const TIn* Bs = reinterpret_cast<const TIn*>(p.B) + prob * p.sB + (long long)s * a.tv.tB;
    const TIn* Rs = reinterpret_cast<const TIn*>(p.R) + prob * p.sR + (long long)s * a.tv.tR;
    load_rows_input<D, TIn>(As, acc, w, i, g);
    write_rows_global<D>(gA, acc, w, i, g);
    __syncthreads();  // H has left the left half
    load_half<D, TIn, false>(WL, Rs, tid);
    load_half<D, TIn, true>(WR, Bs, tid);  // right-hand sides: B^T
    __syncthreads();
    symmetrise_half<D>(WL, tid);
    float rB[C::RB][C::KS];
    load_aopT_lds<D>(WR, rB, w, i, g);  // rows of B = columns of B^T
    __syncthreads();
    const int flag = lds_solve<D, 7, false>(W, S, tid);  // right half: X = R^{-1} B^T
    zero_acc<D>(acc);
    gemm_acc<D>(acc, rB, WR, i, g);  // G = B X
    if (flag) poison<D>(acc);
    write_rows_global<D>(gG, acc, w, i, g);
    if (flag) {  // make sure the breakdown reaches P_1 whatever the other elements are
      poison<D>(acc);
      write_rows_global<D>(gH, acc, w, i, g);
    }
    __syncthreads();
  }
}

// e1 <- e1 o e2 for one pair of elements in the workspace, by the Cfg<D>::NTHR threads of a workgroup (tid = the
// thread's index).  Ends with the results written but no barrier.
template <int D>
__device__ __forceinline__ void scan_compose(float* W, SolveScratch<D>& S, float* St, float* e1, const float* e2,
                                             int tid) {
  using C = Cfg<D>;
  float* const WL = W;
  float* const WR = W + D;
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const oA = e1;  // the composition replaces the first element
  float* const oG = e1 + D * D;
  float* const oH = e1 + 2 * D * D;
  const float *A1 = e1, *G1 = e1 + D * D, *H1 = e1 + 2 * D * D;
  const float *A2 = e2, *G2 = e2 + D * D, *H2 = e2 + 2 * D * D;
  if constexpr (D == 16) {
    // a matrix is one 16-byte piece per lane: all six are requested at once and kept in LDS, one trip to memory
    // for the whole composition instead of one per use (a round with few items is bound by these trips)
    floatx4 v[6];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      v[k] = *reinterpret_cast<const floatx4*>(e1 + k * D * D + 4 * lane);
      v[3 + k] = *reinterpret_cast<const floatx4*>(e2 + k * D * D + 4 * lane);
    }
#pragma unroll
    for (int k = 0; k < 6; ++k) *reinterpret_cast<floatx4*>(&St[k * D * D + 4 * lane]) = v[k];
    __syncthreads();
    A1 = St; G1 = St + D * D; H1 = St + 2 * D * D;
    A2 = St + 3 * D * D; G2 = St + 4 * D * D; H2 = St + 5 * D * D;
  }
  floatx4 acc[C::RB][C::NT], accY[C::RB][C::NT];
  float rM[C::RB][C::KS], rA1T[C::RB][C::KS], rA2[C::RB][C::KS];
  {
    float rG1[C::RB][C::KS];
    load_half<D, float, false>(WR, H2, tid);
    load_aop_global<D, float>(G1, rG1, w, i, g);
    __syncthreads();
    eye_acc<D>(acc, w, i, g);
    gemm_acc<D>(acc, rG1, WR, i, g);  // I + G1 H2
    store_rows<D>(WL, acc, w, i, g);
    __syncthreads();
  }
  set_half_identity<D>(WR, tid);
  __syncthreads();
  const int flag = lds_solve<D>(W, S, tid);  // right half: M = (I + G1 H2)^{-1}
  load_aop_lds<D>(WR, rM, w, i, g);
  load_half<D, float, false>(WL, A1, tid);
  __syncthreads();
  zero_acc<D>(acc);
  gemm_acc<D>(acc, rM, WL, i, g);  // X1 = M A1
  load_aopT_lds<D>(WL, rA1T, w, i, g);
  load_half<D, float, false>(WR, G1, tid);  // M is in registers
  __syncthreads();
  store_rows<D>(WL, acc, w, i, g);  // left half: X1
  zero_acc<D>(accY);
  gemm_acc<D>(accY, rM, WR, i, g);  // Y = M G1
  __syncthreads();
  load_aop_global<D, float>(A2, rA2, w, i, g);
  zero_acc<D>(acc);
  gemm_acc<D>(acc, rA2, WL, i, g);  // A = A2 X1
  write_rows_global<D>(oA, acc, w, i, g);
  {
    float rH2[C::RB][C::KS];
    load_aop_global<D, float>(H2, rH2, w, i, g);
    zero_acc<D>(acc);
    gemm_acc<D>(acc, rH2, WL, i, g);  // V = H2 X1
  }
  store_rows<D>(WR, acc, w, i, g);  // right half: V
  __syncthreads();
  load_rows_global<D>(H1, acc, w, i, g);
  gemm_acc<D>(acc, rA1T, WR, i, g);  // H = H1 + A1^T V
  if (flag) poison<D>(acc);
  write_rows_global<D>(oH, acc, w, i, g);
  store_rows<D>(WL, accY, w, i, g);  // left half: Y
  __syncthreads();
  zero_acc<D>(acc);
  gemm_acc<D>(acc, rA2, WL, i, g);  // Z = A2 Y
  load_half<D, float, true>(WR, A2, tid);  // right half: A2^T
  __syncthreads();
  store_rows<D>(WL, acc, w, i, g);  // left half: Z
  __syncthreads();
  {
    float rZ[C::RB][C::KS];
    load_aop_lds<D>(WL, rZ, w, i, g);
    load_rows_global<D>(G2, acc, w, i, g);
    gemm_acc<D>(acc, rZ, WR, i, g);  // G = G2 + Z A2^T
    write_rows_global<D>(oG, acc, w, i, g);
  }
}

// one round of pairwise compositions
template <int D>
__global__ void __launch_bounds__(Cfg<D>::NTHR) scan_combine_kernel(const ScanArgs a) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ __attribute__((aligned(16))) float St[D == 16 ? 6 * D * D : 4];  // d = 16: the two elements, as read
  const SolveArgs& p = a.tv.s;
  const int st = a.stride;
  const long long per = (p.T - st + 2LL * st - 1) / (2LL * st);  // pairs per problem in this round
  const long long items = p.n * per;
  for (long long item = blockIdx.x; item < items; item += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero();
    const long long prob = item / per;
    const long long j = (item % per) * 2 * st;
    scan_compose<D>(W, S, St, a.ws + (prob * p.T + j) * 3 * D * D, a.ws + (prob * p.T + j + st) * 3 * D * D, tid);
    __syncthreads();
  }
}

// Down-sweep of the tree: after the rounds of scan_combine_kernel element j + st (st the round's stride, j a
// multiple of 2 st) still holds the composition of the steps [j + st, j + 2 st), and the value entering it from
// the right, P after the step of element j + 2 st, is final (it was produced one level up, or that element's range
// reaches the terminal cost and its map is constant).  One level of the down-sweep applies every such element to
// the value on its right, P <- H_e + A_e^T (I + P G_e)^{-1} P A_e, and leaves the result in the element's H slot;
// levels run from the largest stride down to 1, after which the H slot of element k holds P after step k + 1,
// P_{k+1} in the paper's numbering, for every k.  Elements whose range reaches the terminal cost are constant maps
// (A_e = G_e = 0): their H is final as it stands.  A round writes only H slots of odd multiples of st and reads
// only those of even multiples.
template <int D>
__global__ void __launch_bounds__(Cfg<D>::NTHR) scan_apply_kernel(const ScanArgs a) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ __attribute__((aligned(16))) float St[D == 16 ? 4 * D * D : 4];  // d = 16: A, G, H, P as read
  const SolveArgs& p = a.tv.s;
  float* const WR = W + D;
  const int st = a.stride;
  const long long per = (p.T - st + 2LL * st - 1) / (2LL * st);  // elements j + st per problem in this round
  const long long items = p.n * per;
  PhaseTimers tm;
  for (long long item = blockIdx.x; item < items; item += gridDim.x) {
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
    const long long prob = item / per;
    const long long j = (item % per) * 2 * st;
    if (j + 2 * st >= p.T) continue;  // the element's range reaches the terminal cost: its H is P already (uniform)
    float* const e = a.ws + (prob * p.T + j + st) * 3 * D * D;
    const float* gP = a.ws + ((prob * p.T + j + 2 * st) * 3 + 2) * D * D;
    const float *eA = e, *eG = e + D * D, *eH = e + 2 * D * D;
    if constexpr (D == 16) {  // as in scan_combine_kernel: the four matrices in one trip
      floatx4 v[4];
#pragma unroll
      for (int k = 0; k < 3; ++k) v[k] = *reinterpret_cast<const floatx4*>(e + k * D * D + 4 * lane);
      v[3] = *reinterpret_cast<const floatx4*>(gP + 4 * lane);
#pragma unroll
      for (int k = 0; k < 4; ++k) *reinterpret_cast<floatx4*>(&St[k * D * D + 4 * lane]) = v[k];
      __syncthreads();
      eA = St; eG = St + D * D; eH = St + 2 * D * D; gP = St + 3 * D * D;
    }
    floatx4 acc[C::RB][C::NT];
    float rAT[C::RB][C::KS];
    const int flag = mobius_solve<D, float>(W, S, eA, eG, gP, rAT, tid, tm);  // right half: (I + P G)^{-1} P A
    load_rows_global<D>(eH, acc, w, i, g);
    gemm_acc<D>(acc, rAT, WR, i, g);
    if (flag) poison<D>(acc);
    write_rows_global<D>(e + 2 * D * D, acc, w, i, g);
    __syncthreads();
  }
}

// the H slots of all elements, P_1 .. P_T of every problem, as one (n, T, d, d) array (symmetric parts)
template <int D>
__global__ void __launch_bounds__(Cfg<D>::NTHR) scan_gather_kernel(const ScanArgs a, float* __restrict__ P) {
  using C = Cfg<D>;
  const long long items = a.tv.s.n * a.tv.s.T;
  for (long long item = blockIdx.x; item < items; item += gridDim.x) {
    const float* src = a.ws + (item * 3 + 2) * D * D;
    float* dst = P + item * D * D;
    for (int idx = threadIdx.x; idx < D * D; idx += C::NTHR) {
      const int r = idx / D, c = idx % D;
      dst[idx] = 0.5f * (src[idx] + src[c * D + r]);
    }
  }
}

}  // namespace ttc
