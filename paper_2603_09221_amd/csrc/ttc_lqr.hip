// C-ABI entry points and kernels of the batched finite-horizon LQR solver (see include/ttc_lqr.h).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/ttc_lqr.h"
#include "ttc_device.hpp"

namespace ttc {

// Development aid: with -DTTC_PHASE_TIMERS, workgroup 0 accumulates s_memtime ticks per phase and
// writes them to the end of its workspace slot (read back by a profiling script); otherwise no code.
#ifdef TTC_PHASE_TIMERS
#define TTC_TIMER_DECL long long tt_[8] = {0, 0, 0, 0, 0, 0, 0, 0}; long long tt0_ = __builtin_amdgcn_s_memtime();
#define TTC_TOC(k) { const long long now_ = __builtin_amdgcn_s_memtime(); tt_[k] += now_ - tt0_; tt0_ = now_; }
#define TTC_TIMER_DUMP(ptr) if (threadIdx.x == 0 && blockIdx.x == 0) { for (int k_ = 0; k_ < 8; ++k_) (ptr)[k_] += tt_[k_]; }
#else
#define TTC_TIMER_DECL
#define TTC_TOC(k)
#define TTC_TIMER_DUMP(ptr)
#endif

// The same aid as an object, for code split over several functions.
struct PhaseTimers {
#ifdef TTC_PHASE_TIMERS
  long long t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  long long t0 = __builtin_amdgcn_s_memtime();
  __device__ __forceinline__ void toc(int k) {
    const long long now = __builtin_amdgcn_s_memtime();
    t[k] += now - t0;
    t0 = now;
  }
  __device__ __forceinline__ void dump(long long* dst) const {
    if (threadIdx.x == 0 && blockIdx.x == 0)
      for (int k = 0; k < 8; ++k) dst[k] += t[k];
  }
#else
  __device__ __forceinline__ void toc(int) {}
  __device__ __forceinline__ void dump(long long*) const {}
#endif
};

#define TTC_MAX_GROUPS 64  // explicit group lengths (development override) only; the default schedule has no limit

struct SolveArgs {
  long long n;
  int T, flags, ngroups;  // the T factors are applied in ngroups groups, one dense solve each
  int explicit_groups;       // 0: group g ends at step T - floor((ngroups-1-g) T / ngroups); 1: at gend[g]
  int gend[TTC_MAX_GROUPS];  // gend[g] = last step (1-based) of group g; gend[ngroups-1] = T
  const void *A, *B, *Q, *R, *QT, *x0;
  long long sA, sB, sQ, sR, sQT, sx0;
  float *P0, *K0, *u0, *value;
  int* info;
  float* ws;  // gridDim.x slots of d*d floats (C_K of the problem in flight, register layout); more for doubling
};

// A-operand registers of rows [16w,16w+16) of a row-major global matrix: a[4q+t] = M[16w+i][16q+4g+t]
template <int D, typename TIn>
__device__ __forceinline__ void load_aop_global(const TIn* M, float (&a)[Cfg<D>::KS], int w, int i, int g) {
#pragma unroll
  for (int q = 0; q < D / 16; ++q) {
    floatx4 t = ld4<TIn>(M, (long)(16 * w + i) * D + 16 * q + 4 * g);
    a[4 * q + 0] = t[0]; a[4 * q + 1] = t[1]; a[4 * q + 2] = t[2]; a[4 * q + 3] = t[3];
  }
}

template <int D, typename TIn>
__device__ __forceinline__ void load_aop_global(const TIn* M, float (&a)[Cfg<D>::RB][Cfg<D>::KS], int w, int i, int g) {
#pragma unroll
  TTC_FOR_RB load_aop_global<D, TIn>(M, a[rb], Cfg<D>::RB * w + rb, i, g);
}

// A-operand registers <-> workspace, in lane order (thread t's k-th float4 at [k][t]): fully coalesced.
// The constant row blocks are produced while the dense solves of the set-up own the register file,
// so they pass through the workspace once; `off` is an opaque zero that keeps the compiler from
// moving the reloads across the code in between.
template <int D>
__device__ __forceinline__ void store_aop_ws(float* wsc, const float (&a)[Cfg<D>::RB][Cfg<D>::KS], int tid) {
  using C = Cfg<D>;
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int q = 0; q < C::KS / 4; ++q) {
      floatx4 v;
      v[0] = a[rb][4 * q + 0]; v[1] = a[rb][4 * q + 1]; v[2] = a[rb][4 * q + 2]; v[3] = a[rb][4 * q + 3];
      *reinterpret_cast<floatx4*>(wsc + ((long)(rb * (C::KS / 4) + q) * C::NTHR + tid) * 4) = v;
    }
}
template <int D>
__device__ __forceinline__ void load_aop_ws(const float* wsc, float (&a)[Cfg<D>::RB][Cfg<D>::KS], int tid, int off) {
  using C = Cfg<D>;
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int q = 0; q < C::KS / 4; ++q) {
      const floatx4 v = *reinterpret_cast<const floatx4*>(wsc + off + ((long)(rb * (C::KS / 4) + q) * C::NTHR + tid) * 4);
      a[rb][4 * q + 0] = v[0]; a[rb][4 * q + 1] = v[1]; a[rb][4 * q + 2] = v[2]; a[rb][4 * q + 3] = v[3];
    }
}

// copy a row-major global d x d matrix into one half of the LDS pair (optionally transposed), in two
// steps so that other work can be placed between them: issue_half starts all of a thread's global
// reads (the memory latency is paid once per matrix, not once per 16 bytes), commit_half writes LDS.
template <int D>
struct HalfRegs {
  static constexpr int NV = (D * D / 4 + Cfg<D>::NTHR - 1) / Cfg<D>::NTHR;  // float4 pieces per thread
  floatx4 v[NV];
};
template <int D, typename TIn>
__device__ __forceinline__ void issue_half(HalfRegs<D>& h, const TIn* M, int tid) {
  using C = Cfg<D>;
#pragma unroll
  for (int k = 0; k < HalfRegs<D>::NV; ++k) {
    const int idx = tid + k * C::NTHR;
    if (idx < D * D / 4) h.v[k] = ld4<TIn>(M, (long)(idx / (D / 4)) * D + (idx % (D / 4)) * 4);
  }
}
template <int D, bool TRANS>
__device__ __forceinline__ void commit_half(float* Wh, const HalfRegs<D>& h, int tid) {
  using C = Cfg<D>;
#pragma unroll
  for (int k = 0; k < HalfRegs<D>::NV; ++k) {
    const int idx = tid + k * C::NTHR;
    if (idx < D * D / 4) {
      const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
      if constexpr (TRANS) {
#pragma unroll
        for (int j = 0; j < 4; ++j) Wh[(c4 + j) * C::PITCH + r] = h.v[k][j];
      } else {
        *reinterpret_cast<floatx4*>(Wh + r * C::PITCH + c4) = h.v[k];
      }
    }
  }
}
template <int D, typename TIn, bool TRANS>
__device__ __forceinline__ void load_half(float* Wh, const TIn* M, int tid) {
  HalfRegs<D> h;
  issue_half<D, TIn>(h, M, tid);
  commit_half<D, TRANS>(Wh, h, tid);
}
// replace one half by its symmetric part (caller synchronises before and after).  The matrix is cut
// into 4 x 4 blocks; a thread takes the block pair (bi, bj), bi <= bj, reads both blocks with 16-byte
// LDS reads, averages each with the other's transpose in registers and writes them back.
template <int D>
__device__ __forceinline__ void symmetrise_half(float* Wh, int tid) {
  using C = Cfg<D>;
  constexpr int NB = D / 4;
  for (int idx = tid; idx < NB * NB; idx += C::NTHR) {
    const int bi = idx / NB, bj = idx % NB;
    if (bi > bj) continue;
    floatx4 u[4], l[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      u[r] = *reinterpret_cast<const floatx4*>(Wh + (4 * bi + r) * C::PITCH + 4 * bj);
      l[r] = *reinterpret_cast<const floatx4*>(Wh + (4 * bj + r) * C::PITCH + 4 * bi);
    }
    floatx4 un[4], ln[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float s = 0.5f * (u[r][c] + l[c][r]);
        un[r][c] = s;
        ln[c][r] = s;
      }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      *reinterpret_cast<floatx4*>(Wh + (4 * bi + r) * C::PITCH + 4 * bj) = un[r];
      *reinterpret_cast<floatx4*>(Wh + (4 * bj + r) * C::PITCH + 4 * bi) = ln[r];
    }
  }
}
// transpose one half in place through the accumulator layout (all threads; contains the barriers)
template <int D>
__device__ __forceinline__ void transpose_half(float* Wh, int w, int i, int g) {
  floatx4 t[Cfg<D>::RB][Cfg<D>::NT];
  load_rows<D>(Wh, t, w, i, g);
  __syncthreads();
  store_rows_T<D>(Wh, t, w, i, g);
  __syncthreads();
}
template <int D>
__device__ __forceinline__ void set_half_identity(float* Wh, int tid) {
  using C = Cfg<D>;
  for (int idx = tid; idx < D * D / 4; idx += C::NTHR) {
    const int r = idx / (D / 4), c4 = (idx % (D / 4)) * 4;
    floatx4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (c4 + j == r) ? 1.f : 0.f;
    *reinterpret_cast<floatx4*>(Wh + r * C::PITCH + c4) = v;
  }
}

// store `info`-aware outputs of one accumulator (rows of P0 or K0) and return this lane's share of
// (M x0)[row] for its four rows: out[v] = sum over the lane's columns of acc[c][v] * x0[col]
template <int D>
__device__ __forceinline__ void write_rows_global(float* dst, const floatx4 (&acc)[Cfg<D>::NT], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int h = 0; h < C::NH; ++h) {
      float* q = dst + (long)(16 * w + 4 * g + v) * D + 16 * C::VEC * h + C::VEC * i;
#pragma unroll
      for (int tp = 0; tp < C::VEC; ++tp) q[tp] = acc[h * C::VEC + tp][v];
    }
}

// Outputs of one problem, in two parts.  A problem whose info is non-zero gets NaN.
// emit_gain: on entry acc holds this wavefront's rows of -K_0; writes u_0 = K_0 x0 and K_0.
template <int D, typename TIn>
__device__ __forceinline__ void emit_gain(const SolveArgs& p, long long prob, floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT],
                                          const TIn* x0p, int info, int tid) {
  using C = Cfg<D>;
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  const float nanv = __builtin_nanf("");
  float x0c[C::NT];
#pragma unroll
  for (int c = 0; c < C::NT; ++c) x0c[c] = ld1<TIn>(x0p, tile_col<D>(c, i));
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float pu = 0.f;
#pragma unroll
      for (int c = 0; c < C::NT; ++c) {
        const float ke = info ? nanv : -acc[rb][c][v];
        acc[rb][c][v] = ke;
        pu += ke * x0c[c];
      }
      pu = sum16(pu);
      if (i == 0) p.u0[prob * D + 16 * (C::RB * w + rb) + 4 * g + v] = pu;
    }
  if (p.K0) {
#pragma unroll
    for (int rb = 0; rb < C::RB; ++rb) write_rows_global<D>(p.K0 + prob * (long)D * D, acc[rb], C::RB * w + rb, i, g);
  }
}
// emit_value: the LDS half WP holds P_0 in the paper's convention (Q_0 = 0); writes P_0 (+ Q with
// TTC_FLAG_STAGE_COST_AT_X0), value = x0^T P_0 x0 and info.  Contains two barriers, the second at its end.
template <int D, typename TIn>
__device__ __forceinline__ void emit_value(const SolveArgs& p, long long prob, const float* WP, const TIn* Qp,
                                           const TIn* x0p, int info, float* s_red, int tid) {
  using C = Cfg<D>;
  const int lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  const float nanv = __builtin_nanf("");
  floatx4 acc[C::RB][C::NT];
  float x0c[C::NT];
#pragma unroll
  for (int c = 0; c < C::NT; ++c) x0c[c] = ld1<TIn>(x0p, tile_col<D>(c, i));
  float vpart = 0.f;
  load_rows<D>(WP, acc, w, i, g);                // rows of P_0
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const long row = 16 * (C::RB * w + rb) + 4 * g + v;
      float pw = 0.f;
#pragma unroll
      for (int c = 0; c < C::NT; ++c) {
        float pe = acc[rb][c][v];
        if (p.flags & TTC_FLAG_STAGE_COST_AT_X0) {
          const long col = tile_col<D>(c, i);
          pe += 0.5f * (ld1<TIn>(Qp, row * D + col) + ld1<TIn>(Qp, col * D + row));
        }
        if (info) pe = nanv;
        acc[rb][c][v] = pe;
        pw += pe * x0c[c];
      }
      vpart += ld1<TIn>(x0p, row) * pw;
    }
  vpart = sum64(vpart);
  if (lane == 0) s_red[w] = vpart;
  if (p.P0) {
#pragma unroll
    for (int rb = 0; rb < C::RB; ++rb) write_rows_global<D>(p.P0 + prob * (long)D * D, acc[rb], C::RB * w + rb, i, g);
  }
  __syncthreads();
  if (tid == 0) {
    float val = 0.f;
    for (int ww = 0; ww < C::NW; ++ww) val += s_red[ww];
    if (p.value) p.value[prob] = val;
    if (p.info) p.info[prob] = info;
  }
  __syncthreads();
}

// Solve kernel.  Persistent workgroups: workgroup b handles problems b, b + gridDim.x, ...
//
// Per problem the work is a sequence of phases, each "build [M | RHS] in LDS, dense solve, consume":
//   phase R  X = R^{-1} B^T, then G = B X (Thm 3.3's G).
//   phase A  A^{-1}; C_K = X A^{-T}; Z2 = Q_T, Z1 = I.
//   phase S  one group of reverse symplectic steps (Alg. 4 body), the last one leaving the
//            pair untransposed; the solve re-bases it, [Y1 Y2] <- [I, Y1^{-1} Y2].  Repeated until all
//            T factors Sigma_T .. Sigma_1 are applied; the last factor has Q_0 = 0, i.e. no "+ Y1 Q".
//   output   after the last solve the right half is P_0 = Y1^{-1} Y2 itself (Alg. 4), lambda_0 = P_0 x0,
//            and K_0 = -R^{-1} B^T A^{-T} P_0 = -C_K P_0 (Thm A.4: u_1 = -R^{-1} B^T A^{-T} lambda_0).
// The row blocks of G, A^T, Q and A^{-1} go from LDS straight into registers as they are produced and
// stay there to the end of the problem; only C_K, needed once at the very end, waits in the workspace.
// Global reads are started a phase ahead of their use where registers allow.
template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) solve_kernel(const SolveArgs p) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];

  float* const WL = W;      // left half  (Z1 / Y1 / M of a dense solve)
  float* const WR = W + D;  // right half (Z2 / Y2 / RHS)
  // per-workgroup workspace: the row blocks of C_K in register layout
  float* const wsC = p.ws + (long)blockIdx.x * D * D;
  const bool pure = (p.flags & TTC_FLAG_PURE_SYMPLECTIC) != 0;

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    // (the opaque zero keeps the address arithmetic of a problem from being hoisted out of this loop and spilled)
    const int tid = threadIdx.x + opaque_zero(), lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    TTC_TIMER_DECL
    int info = 0, nsolve = 0;
    floatx4 acc[C::RB][C::NT];
    int s = 1;          // next reverse step (1 .. T; step s applies Sigma_{T-s+1})
    int grp = 0;        // current group of steps
    bool fresh = true;  // Z1 = I, not materialised
    // the constant row blocks, in registers from here to the end of the problem
    float cG[C::RB][C::KS], cAi[C::RB][C::KS], cAT[C::RB][C::KS], cQ[C::RB][C::KS];

    // ---------------------------------------------------------------- phase R: X = R^{-1} B^T, G = B X
    load_half<D, TIn, false>(WL, reinterpret_cast<const TIn*>(p.R) + prob * p.sR, tid);
    load_half<D, TIn, false>(WR, reinterpret_cast<const TIn*>(p.B) + prob * p.sB, tid);
    __syncthreads();
    symmetrise_half<D>(WL, tid);
    transpose_half<D>(WR, w, i, g);              // RHS = B^T
    {
      float cX[C::RB][C::KS];
      {
        float cB[C::RB][C::KS];
        load_aopT_lds<D>(WR, cB, w, i, g);       // rows of B = columns of B^T
        TTC_TOC(6)
        ++nsolve;
        if (lds_solve<D, 7, false>(W, S, tid) && !info) info = nsolve;  // R is positive definite: no pivot search
        TTC_TOC(1)
        HalfRegs<D> hA, hQ;
        issue_half<D, TIn>(hA, Ap, tid);         // wanted after the product below
        issue_half<D, TIn>(hQ, Qp, tid);
        zero_acc<D>(acc);
        gemm_acc<D>(acc, cB, WR, i, g);          // rows of G = B X
        load_aop_lds<D>(WR, cX, w, i, g);        // rows of X, for C_K
        store_rows<D>(WL, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WL, tid);             // G is symmetric up to rounding; make it exactly so
        __syncthreads();
        load_aop_lds<D>(WL, cG, w, i, g);
        __syncthreads();
        TTC_TOC(7)
        // ------------------------------------------------------------ phase A: A^{-1}, A^T, Q, C_K
        commit_half<D, false>(WL, hA, tid);
        commit_half<D, false>(WR, hQ, tid);
      }
      __syncthreads();
      symmetrise_half<D>(WR, tid);
      load_aopT_lds<D>(WL, cAT, w, i, g);        // rows of A^T = columns of A
      __syncthreads();
      load_aop_lds<D>(WR, cQ, w, i, g);          // rows of the symmetric part of Q
      __syncthreads();
      set_half_identity<D>(WR, tid);
      __syncthreads();
      TTC_TOC(0)
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;
      TTC_TOC(1)
      load_aop_lds<D>(WR, cAi, w, i, g);
      __syncthreads();
      transpose_half<D>(WR, w, i, g);            // A^{-T}
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cX, WR, i, g);            // rows of C_K = X A^{-T}
    }
    store_rows<D>(WL, acc, w, i, g);
    __syncthreads();
    {
      float c[C::RB][C::KS];
      load_aop_lds<D>(WL, c, w, i, g);
      store_aop_ws<D>(wsC, c, tid);
    }
    // initial pair [Y1 Y2] = [I Q_T]
    if (p.QT) {
      load_half<D, TIn, false>(WR, reinterpret_cast<const TIn*>(p.QT) + prob * p.sQT, tid);
      __syncthreads();
      symmetrise_half<D>(WR, tid);
    } else {
      store_aop_lds<D>(WR, cQ, w, i, g);         // Q_T = Q, already symmetric
    }
    __syncthreads();

    // ---------------------------------------------------------------- groups of steps, each ended by a re-base
    for (;;) {
      {
        TTC_TOC(2)
        const int tg = tid + opaque_zero(), lane = tg & 63, w = tg >> 6, i = lane & 15, g = lane >> 4;
        // last step of this group: lengths differ by at most one, the longer groups first
        const int gend = p.explicit_groups ? p.gend[grp]
                                           : p.T - (int)(((long long)(p.ngroups - 1 - grp) * p.T) / p.ngroups);
        for (;; ++s) {
          const bool last = (s >= gend);
          if (fresh) eye_acc<D>(acc, w, i, g); else load_rows<D>(WL, acc, w, i, g);
          gemm_acc<D>(acc, cG, WR, i, g);    // Z1 + G Z2       (Y1 + Y2 G)
          store_rows<D>(WL, acc, w, i, g);
          __syncthreads();
          zero_acc<D>(acc);
          gemm_acc<D>(acc, cAi, WL, i, g);   // A^{-1} (.)      (... A^{-T})  = new Z1
          __syncthreads();
          store_rows<D>(WL, acc, w, i, g);
          __syncthreads();
          zero_acc<D>(acc);
          gemm_acc<D>(acc, cAT, WR, i, g);   // A^T Z2          (Y2 A)
          if (s < p.T) gemm_acc<D>(acc, cQ, WL, i, g);  // + Q Z1 (+ Y1 Q_{t-1}); Q_0 = 0 for the last factor
          __syncthreads();
          fresh = false;
          if (!last) {
            store_rows<D>(WR, acc, w, i, g);
            __syncthreads();
            if (pure) {
              normalise_rows_zland<D>(W, tid);
              __syncthreads();
            }
          } else {
            // leave Z-land: [Y1 | Y2] untransposed for the solve Y1 P = Y2
            store_rows_T<D>(WR, acc, w, i, g);
            load_rows<D>(WL, acc, w, i, g);
            __syncthreads();
            store_rows_T<D>(WL, acc, w, i, g);
            __syncthreads();
            ++s;
            break;
          }
        }
      }
      TTC_TOC(3)
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;
      TTC_TOC(4)
      symmetrise_half<D>(WR, tid);           // P is symmetric; also makes it its own Z-land image
      __syncthreads();
      fresh = true;
      ++grp;
      if (s > p.T) break;
    }

    // ---- outputs: WR holds P_0 (paper convention, Q_0 = 0)
    {
      float c[C::RB][C::KS];
      load_aop_ws<D>(wsC, c, tid, opaque_zero());  // C_K; in flight while P_0 is written out
      emit_value<D, TIn>(p, prob, WR, Qp, x0p, info, s_red, tid);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, c, WR, i, g);               // -K_0 = C_K P_0
    }
    emit_gain<D, TIn>(p, prob, acc, x0p, info, tid);
    __syncthreads();                               // every wavefront is done with the pair
    TTC_TOC(5)
    TTC_TIMER_DUMP(reinterpret_cast<long long*>(p.ws) + (long)gridDim.x * D * D / 2)
  }
}

}  // namespace ttc
#include "ttc_doubling.hpp"
#include "ttc_small.hpp"
namespace ttc {

// ------------------------------------------------------------------------------------------------
struct RolloutArgs {
  long long n;
  int T, flags;
  const void *A, *B, *Q, *R, *QT, *x0;
  long long sA, sB, sQ, sR, sQT, sx0;
  float *U, *X, *cost;
  int* info;
  float* ws;  // gridDim.x slots of (T+3) d*d floats: G, R^{-1} B^T, A^T (register layout), K_0 .. K_{T-1}
};

// y[r] = sum_c M[r][c] x[c] for the row r = tid / TPR of a row-major global d x d matrix; the TPR
// threads of a row (adjacent lanes) each take a share of the columns; all of them get the sum.
template <int D, typename TM>
__device__ __forceinline__ float matvec_row(const TM* M, const float* xs, int tid) {
  constexpr int TPR = Cfg<D>::NTHR / D;  // 2 or 4
  const int r = tid / TPR, part = tid % TPR;
  float s = 0.f;
#pragma unroll
  for (int c4 = part * (D / TPR); c4 < (part + 1) * (D / TPR); c4 += 4) {
    const floatx4 mv = ld4<TM>(M, (long)r * D + c4);
    s += mv[0] * xs[c4] + mv[1] * xs[c4 + 1] + mv[2] * xs[c4 + 2] + mv[3] * xs[c4 + 3];
  }
#pragma unroll
  for (int m = 1; m < TPR; m <<= 1) s += __shfl_xor(s, m, 64);
  return s;
}

// Roll-out kernel (Alg. 1 with r = 0).  Backward sweep: the value matrices P_T .. P_1 are produced
// one step at a time in the re-based form of the reverse symplectic factor (re-base every step):
//     M_t = (I + P_{t+1} G)^{-1} P_{t+1} A,   K_t = -(R^{-1} B^T) M_t,   P_t = Q + A^T M_t,
// the gains go to the workspace; forward sweep: u_t = K_t x_t, x_{t+1} = A x_t + B u_t and the cost.
template <int D, typename TIn>
__global__ void __launch_bounds__(Cfg<D>::NTHR) rollout_kernel(const RolloutArgs p) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) float W[D * C::PITCH];
  __shared__ __attribute__((aligned(16))) SolveScratch<D> S;
  __shared__ float s_red[C::NW];
  __shared__ float s_x[D], s_u[D], s_xn[D];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, i = lane & 15, g = lane >> 4;
  float* const WL = W;
  float* const WR = W + D;
  float* const wsC = p.ws + (long)blockIdx.x * (p.T + 3) * D * D;  // G, X, A^T in register layout
  float* const wsK = wsC + 3 * D * D;                              // K_0 .. K_{T-1}, row-major

  for (long long prob = blockIdx.x; prob < p.n; prob += gridDim.x) {
    const TIn* Ap = reinterpret_cast<const TIn*>(p.A) + prob * p.sA;
    const TIn* Bp = reinterpret_cast<const TIn*>(p.B) + prob * p.sB;
    const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob * p.sQ;
    const TIn* Rp = reinterpret_cast<const TIn*>(p.R) + prob * p.sR;
    const TIn* QTp = p.QT ? reinterpret_cast<const TIn*>(p.QT) + prob * p.sQT : Qp;
    const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob * p.sx0;
    int info = 0, nsolve = 0;
    floatx4 acc[C::RB][C::NT];

    // ---- setup: X = R^{-1} B^T, G = B X; row blocks of G, X, A^T to the workspace
    load_half<D, TIn, false>(WL, Rp, tid);
    load_half<D, TIn, false>(WR, Bp, tid);
    __syncthreads();
    symmetrise_half<D>(WL, tid);
    transpose_half<D>(WR, w, i, g);              // RHS = B^T
    ++nsolve;
    if (lds_solve<D, 7, false>(W, S, tid) && !info) info = nsolve;  // R is positive definite: no pivot search
    {
      float c[C::RB][C::KS];
      load_aop_lds<D>(WR, c, w, i, g);
      store_aop_ws<D>(wsC + 1 * D * D, c, tid);
      load_aop_global<D, TIn>(Bp, c, w, i, g);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, c, WR, i, g);
      store_rows<D>(WL, acc, w, i, g);
      __syncthreads();
      symmetrise_half<D>(WL, tid);
      __syncthreads();
      load_aop_lds<D>(WL, c, w, i, g);
      store_aop_ws<D>(wsC + 0 * D * D, c, tid);
#pragma unroll
      for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
        for (int k = 0; k < C::KS; ++k)
          c[rb][k] = ld1<TIn>(Ap, (long)(16 * (k / 4) + 4 * g + (k % 4)) * D + 16 * (C::RB * w + rb) + i);
      store_aop_ws<D>(wsC + 2 * D * D, c, tid);
    }
    __syncthreads();
    load_half<D, TIn, false>(WR, QTp, tid);
    __syncthreads();
    symmetrise_half<D>(WR, tid);
    __syncthreads();

    // ---- backward sweep (the constant row blocks stay in registers)
    float cG[C::RB][C::KS], cX[C::RB][C::KS], cAT[C::RB][C::KS];
    load_aop_ws<D>(wsC + 0 * D * D, cG, tid, 0);
    load_aop_ws<D>(wsC + 1 * D * D, cX, tid, 0);
    load_aop_ws<D>(wsC + 2 * D * D, cAT, tid, 0);
    for (int t = p.T - 1; t >= 0; --t) {
      eye_acc<D>(acc, w, i, g);
      gemm_acc<D>(acc, cG, WR, i, g);   // (I + P G)^T
      store_rows_T<D>(WL, acc, w, i, g);
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cAT, WR, i, g);  // (P A)^T
      __syncthreads();
      store_rows_T<D>(WR, acc, w, i, g);
      __syncthreads();
      ++nsolve;
      if (lds_solve<D>(W, S, tid) && !info) info = nsolve;
      zero_acc<D>(acc);
      gemm_acc<D>(acc, cX, WR, i, g);    // -K_t
#pragma unroll
      for (int rb = 0; rb < C::RB; ++rb) {
#pragma unroll
        for (int cc = 0; cc < C::NT; ++cc) acc[rb][cc] = -acc[rb][cc];
        write_rows_global<D>(wsK + (long)t * D * D, acc[rb], C::RB * w + rb, i, g);
      }
      if (t >= 1) {
#pragma unroll
        for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
          for (int cc = 0; cc < C::NT; ++cc)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const long row = 16 * (C::RB * w + rb) + 4 * g + v, col = tile_col<D>(cc, i);
              acc[rb][cc][v] = 0.5f * (ld1<TIn>(Qp, row * D + col) + ld1<TIn>(Qp, col * D + row));
            }
        gemm_acc<D>(acc, cAT, WR, i, g);  // P_t = Q + A^T M_t
        __syncthreads();
        store_rows<D>(WR, acc, w, i, g);
        __syncthreads();
        symmetrise_half<D>(WR, tid);
        __syncthreads();
      }
    }
    __syncthreads();  // gains visible to the whole workgroup

    // ---- forward sweep
    const int r = tid / (C::NTHR / D), part = tid % (C::NTHR / D);
    if (tid < D) s_x[tid] = ld1<TIn>(x0p, tid);
    __syncthreads();
    float cpart = 0.f;
    if (p.flags & TTC_FLAG_STAGE_COST_AT_X0) {
      const float qx = matvec_row<D, TIn>(Qp, s_x, tid);
      if (part == 0) cpart += s_x[r] * qx;
    }
    if (p.X && tid < D) p.X[prob * (long)(p.T + 1) * D + tid] = s_x[tid];
    for (int t = 0; t < p.T; ++t) {
      const float u = matvec_row<D, float>(wsK + (long)t * D * D, s_x, tid);
      if (part == 0) s_u[r] = u;
      __syncthreads();
      const float ru = matvec_row<D, TIn>(Rp, s_u, tid);
      const float xn = matvec_row<D, TIn>(Ap, s_x, tid) + matvec_row<D, TIn>(Bp, s_u, tid);
      if (part == 0) {
        cpart += s_u[r] * ru;
        s_xn[r] = xn;
        p.U[(prob * p.T + t) * (long)D + r] = info ? __builtin_nanf("") : u;
      }
      __syncthreads();
      const float qx = matvec_row<D, TIn>(t == p.T - 1 ? QTp : Qp, s_xn, tid);
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

}  // namespace ttc
#include "ttc_tv.hpp"
#include "ttc_scan.hpp"
#include "ttc_cxt.hpp"
namespace ttc {

// ------------------------------------------------------------------------------------------------
static int cu_count() {
  static int cached = 0;
  if (cached > 0) return cached;
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) {
    cached = n;
    return n;
  }
  (void)hipGetLastError();
  return 256;  // MI355X
}
// resident workgroups per compute unit the grid is sized for
// Persistent grids: as many workgroups as are resident at once, CUs x (workgroups per CU), so that no
// workgroup waits for another to finish.  The per-CU number is what the runtime reports for the kernel
// (registers and LDS decide it); the table is the fallback when no device can be asked.
enum Kind { KIND_SOLVE = 0, KIND_DOUBLING = 1, KIND_ROLLOUT = 2, KIND_SOLVE_QUAD = 3, KIND_SOLVE_TV = 4, KIND_TV_QUAD = 5,
            KIND_ROLLOUT_TV = 6, KIND_CXT = 7, KIND_SCAN = 8 };
static int dindex(int d) { return d == 16 ? 0 : d == 32 ? 1 : d == 64 ? 2 : 3; }
template <int D>
static int occupancy_of(Kind kind, bool bf16) {
  int nb = 0;
  hipError_t e;
  const int nthr = Cfg<D>::NTHR;
  if (kind == KIND_SOLVE_QUAD)  // the four-problems-per-wavefront kernel (d = 16 only)
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_small_kernel<uint16_t, 4>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_small_kernel<float, 4>, nthr, 0);
  else if (kind == KIND_SCAN)  // the pairwise compositions (the leaf kernel uses fewer registers)
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, scan_combine_kernel<D>, nthr, 0);
  else if (kind == KIND_CXT)  // structured parameters (d = 16 only)
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_cxt_kernel<uint16_t, 4>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_cxt_kernel<float, 4>, nthr, 0);
  else if (kind == KIND_ROLLOUT_TV)
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, rollout_tv_kernel<D, uint16_t>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, rollout_tv_kernel<D, float>, nthr, 0);
  else if (kind == KIND_TV_QUAD)
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_tv_small_kernel<uint16_t, 4>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_tv_small_kernel<float, 4>, nthr, 0);
  else if (kind == KIND_SOLVE_TV)
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_tv_kernel<D, uint16_t>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_tv_kernel<D, float>, nthr, 0);
  else if (kind == KIND_SOLVE)
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_kernel<D, uint16_t>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, solve_kernel<D, float>, nthr, 0);
  else if (kind == KIND_DOUBLING)
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, doubling_kernel<D, uint16_t>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, doubling_kernel<D, float>, nthr, 0);
  else
    e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, rollout_kernel<D, uint16_t>, nthr, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, rollout_kernel<D, float>, nthr, 0);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return nb;
}
static int blocks_per_cu(Kind kind, int d, bool bf16) {
  static int cached[9][4][2];  // 0 = not asked yet
  int& c = cached[kind][dindex(d)][bf16 ? 1 : 0];
  if (c > 0) return c;
  int nb = 0;
  switch (d) {
    case 16: nb = occupancy_of<16>(kind, bf16); break;
    case 32: nb = occupancy_of<32>(kind, bf16); break;
    case 64: nb = occupancy_of<64>(kind, bf16); break;
    case 128: nb = occupancy_of<128>(kind, bf16); break;
  }
  if (nb > 0) {
    c = nb > 32 ? 32 : nb;
    return c;
  }
  static const int table[9][4] = {{20, 8, 2, 1}, {16, 8, 2, 1}, {12, 4, 2, 1}, {8, 8, 2, 1}, {20, 8, 2, 1},
                                  {8, 8, 2, 1},  {12, 4, 2, 1}, {8, 8, 2, 1},  {16, 8, 2, 1}};
  return table[kind][dindex(d)];
}
static long long grid_blocks(Kind kind, int d, bool bf16) {
  return (long long)cu_count() * blocks_per_cu(kind, d, bf16);
}
// d = 16, default path: batches that fill the chip go four problems to a wavefront (more throughput);
// small batches keep one problem per wavefront (more wavefronts in flight, lower latency).
static bool use_quad_kernel(const ttc_lqr_problem_t* q) {
  return q->d == 16 && !(q->flags & TTC_FLAG_DOUBLING) && q->n >= 8LL * cu_count();
}

static bool shape_supported(const ttc_lqr_problem_t* q) {
  return q->d == q->m && (q->d == 16 || q->d == 32 || q->d == 64 || q->d == 128);
}
static bool aligned_ptr(const void* ptr, size_t a) { return (reinterpret_cast<uintptr_t>(ptr) % a) == 0; }

static ttc_status_t validate(const ttc_lqr_problem_t* q) {
  if (!q) return TTC_ERR_INVALID_ARG;
  if (q->n < 0 || q->T < 1 || q->d < 1 || q->m < 1 || q->rebase_every < 0) return TTC_ERR_INVALID_ARG;
  if (q->in_dtype != TTC_F32 && q->in_dtype != TTC_BF16) return TTC_ERR_INVALID_ARG;
  if (q->flags & ~(TTC_FLAG_STAGE_COST_AT_X0 | TTC_FLAG_PURE_SYMPLECTIC | TTC_FLAG_DOUBLING)) return TTC_ERR_INVALID_ARG;
  if ((q->flags & TTC_FLAG_PURE_SYMPLECTIC) && (q->flags & TTC_FLAG_DOUBLING)) return TTC_ERR_INVALID_ARG;
  if (!shape_supported(q)) return TTC_ERR_UNSUPPORTED;
  if (q->n == 0) return TTC_OK;
  if (!q->A || !q->B || !q->Q || !q->R || !q->x0) return TTC_ERR_INVALID_ARG;
  const size_t al = q->in_dtype == TTC_F32 ? 16 : 8;
  const void* ptrs[] = {q->A, q->B, q->Q, q->R, q->QT};
  const int64_t strides[] = {q->sA, q->sB, q->sQ, q->sR, q->sQT};
  for (int k = 0; k < 5; ++k) {
    if (ptrs[k] && !aligned_ptr(ptrs[k], al)) return TTC_ERR_INVALID_ARG;
    if (strides[k] < 0 || strides[k] % 4) return TTC_ERR_INVALID_ARG;
  }
  if (q->sx0 < 0) return TTC_ERR_INVALID_ARG;
  return TTC_OK;
}

template <typename TIn>
static hipError_t launch_solve(const SolveArgs& a, int d, dim3 grid, hipStream_t st) {
  switch (d) {
    case 16: hipLaunchKernelGGL((solve_kernel<16, TIn>), grid, dim3(Cfg<16>::NTHR), 0, st, a); break;
    case 32: hipLaunchKernelGGL((solve_kernel<32, TIn>), grid, dim3(Cfg<32>::NTHR), 0, st, a); break;
    case 64: hipLaunchKernelGGL((solve_kernel<64, TIn>), grid, dim3(Cfg<64>::NTHR), 0, st, a); break;
    case 128: hipLaunchKernelGGL((solve_kernel<128, TIn>), grid, dim3(Cfg<128>::NTHR), 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename TIn>
static hipError_t launch_doubling(const DoublingArgs& a, int d, dim3 grid, hipStream_t st) {
  switch (d) {
    case 16: hipLaunchKernelGGL((doubling_kernel<16, TIn>), grid, dim3(Cfg<16>::NTHR), 0, st, a); break;
    case 32: hipLaunchKernelGGL((doubling_kernel<32, TIn>), grid, dim3(Cfg<32>::NTHR), 0, st, a); break;
    case 64: hipLaunchKernelGGL((doubling_kernel<64, TIn>), grid, dim3(Cfg<64>::NTHR), 0, st, a); break;
    case 128: hipLaunchKernelGGL((doubling_kernel<128, TIn>), grid, dim3(Cfg<128>::NTHR), 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename TIn>
static hipError_t launch_tv(const TvArgs& a, int d, dim3 grid, hipStream_t st) {
  switch (d) {
    case 16: hipLaunchKernelGGL((solve_tv_kernel<16, TIn>), grid, dim3(Cfg<16>::NTHR), 0, st, a); break;
    case 32: hipLaunchKernelGGL((solve_tv_kernel<32, TIn>), grid, dim3(Cfg<32>::NTHR), 0, st, a); break;
    case 64: hipLaunchKernelGGL((solve_tv_kernel<64, TIn>), grid, dim3(Cfg<64>::NTHR), 0, st, a); break;
    case 128: hipLaunchKernelGGL((solve_tv_kernel<128, TIn>), grid, dim3(Cfg<128>::NTHR), 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename TIn>
static hipError_t launch_scan_leaf(const ScanArgs& a, int d, dim3 grid, hipStream_t st) {
  switch (d) {
    case 16: hipLaunchKernelGGL((scan_leaf_kernel<16, TIn>), grid, dim3(Cfg<16>::NTHR), 0, st, a); break;
    case 32: hipLaunchKernelGGL((scan_leaf_kernel<32, TIn>), grid, dim3(Cfg<32>::NTHR), 0, st, a); break;
    case 64: hipLaunchKernelGGL((scan_leaf_kernel<64, TIn>), grid, dim3(Cfg<64>::NTHR), 0, st, a); break;
    case 128: hipLaunchKernelGGL((scan_leaf_kernel<128, TIn>), grid, dim3(Cfg<128>::NTHR), 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
static hipError_t launch_scan_combine(const ScanArgs& a, int d, dim3 grid, hipStream_t st) {
  switch (d) {
    case 16: hipLaunchKernelGGL((scan_combine_kernel<16>), grid, dim3(Cfg<16>::NTHR), 0, st, a); break;
    case 32: hipLaunchKernelGGL((scan_combine_kernel<32>), grid, dim3(Cfg<32>::NTHR), 0, st, a); break;
    case 64: hipLaunchKernelGGL((scan_combine_kernel<64>), grid, dim3(Cfg<64>::NTHR), 0, st, a); break;
    case 128: hipLaunchKernelGGL((scan_combine_kernel<128>), grid, dim3(Cfg<128>::NTHR), 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename TIn>
static hipError_t launch_rollout_tv(const TvRolloutArgs& a, int d, dim3 grid, hipStream_t st) {
  switch (d) {
    case 16: hipLaunchKernelGGL((rollout_tv_kernel<16, TIn>), grid, dim3(Cfg<16>::NTHR), 0, st, a); break;
    case 32: hipLaunchKernelGGL((rollout_tv_kernel<32, TIn>), grid, dim3(Cfg<32>::NTHR), 0, st, a); break;
    case 64: hipLaunchKernelGGL((rollout_tv_kernel<64, TIn>), grid, dim3(Cfg<64>::NTHR), 0, st, a); break;
    case 128: hipLaunchKernelGGL((rollout_tv_kernel<128, TIn>), grid, dim3(Cfg<128>::NTHR), 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename TIn>
static hipError_t launch_rollout(const RolloutArgs& a, int d, dim3 grid, hipStream_t st) {
  switch (d) {
    case 16: hipLaunchKernelGGL((rollout_kernel<16, TIn>), grid, dim3(Cfg<16>::NTHR), 0, st, a); break;
    case 32: hipLaunchKernelGGL((rollout_kernel<32, TIn>), grid, dim3(Cfg<32>::NTHR), 0, st, a); break;
    case 64: hipLaunchKernelGGL((rollout_kernel<64, TIn>), grid, dim3(Cfg<64>::NTHR), 0, st, a); break;
    case 128: hipLaunchKernelGGL((rollout_kernel<128, TIn>), grid, dim3(Cfg<128>::NTHR), 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ttc

extern "C" {

size_t ttc_lqr_workspace_bytes(const ttc_lqr_problem_t* problem, int for_rollout) {
  if (!problem || problem->T < 1 || !ttc::shape_supported(problem)) return 0;
  const ttc::Kind kind = for_rollout ? ttc::KIND_ROLLOUT
                         : (problem->flags & TTC_FLAG_DOUBLING) ? ttc::KIND_DOUBLING : ttc::KIND_SOLVE;
  // (the four-problems-per-wavefront kernel of d = 16 runs fewer workgroups and needs no workspace)
  const size_t slots = (size_t)ttc::grid_blocks(kind, problem->d, problem->in_dtype == TTC_BF16);
  const size_t per = (size_t)problem->d * problem->m * sizeof(float);
  const size_t solve_slots = (problem->flags & TTC_FLAG_DOUBLING) ? (size_t)ttc::DBL_SLOTS : 1;
  return slots * per * (for_rollout ? (size_t)problem->T + 3 : solve_slots);
}

ttc_status_t ttc_lqr_solve(const ttc_lqr_problem_t* problem, const ttc_lqr_solution_t* solution,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t st = ttc::validate(problem);
  if (st != TTC_OK) return st;
  if (!solution) return TTC_ERR_INVALID_ARG;
  if (problem->n == 0) return TTC_OK;
  if (!solution->u0) return TTC_ERR_INVALID_ARG;
  if (!ttc::aligned_ptr(solution->P0, 16) || !ttc::aligned_ptr(solution->K0, 16)) return TTC_ERR_INVALID_ARG;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) ||
      workspace_bytes < ttc_lqr_workspace_bytes(problem, 0))
    return TTC_ERR_WORKSPACE;
  ttc::SolveArgs a;
  a.n = problem->n;
  a.T = problem->T;
  a.flags = problem->flags;
  // Grouping of the T factors (one dense solve per group).  rebase_every = k asks for ceil(T/k) groups;
  // the default is ceil(T/3.4) groups for float32 inputs and ceil(T/5) for bfloat16 inputs.  Lengths
  // differ by at most one and the longer groups come first: an error made at an early re-base is
  // damped by the contracting closed loop, the last group's error reaches P_0 undamped.  Measured max
  // rel. err of P0/u0 at d = 128, T = 16 over 20000 problems: 2.0e-5 for groups (4,3,3,3,3),
  // 6.2e-5 for (3,3,3,3,4), 6.8e-5 for (4,4,4,4), 1.6e-5 for six groups; the tolerance is 1e-4.
  {
    long g;
    if (problem->flags & TTC_FLAG_PURE_SYMPLECTIC) g = 1;
    else if (problem->rebase_every > 0) g = (problem->T + problem->rebase_every - 1) / problem->rebase_every;
    else if (problem->in_dtype == TTC_BF16) g = (problem->T + 4) / 5;
    else g = ((long)problem->T * 10 + 33) / 34;
    if (g < 1) g = 1;
    if (g > problem->T) g = problem->T;
    a.ngroups = (int)g;
    a.explicit_groups = 0;
#ifdef TTC_PHASE_TIMERS
    if (const char* e = getenv("TTC_GROUP_LENGTHS")) {   // development: explicit lengths "5,4,4,3"
      int cnt = 0, end = 0;
      for (const char* c = e; *c && cnt < TTC_MAX_GROUPS;) {
        end += atoi(c);
        a.gend[cnt++] = end;
        while (*c && *c != ',') ++c;
        if (*c == ',') ++c;
      }
      if (end == problem->T) {
        a.ngroups = cnt;
        a.explicit_groups = 1;
      }
    }
#endif
  }
  a.A = problem->A; a.B = problem->B; a.Q = problem->Q; a.R = problem->R; a.QT = problem->QT; a.x0 = problem->x0;
  a.sA = problem->sA; a.sB = problem->sB; a.sQ = problem->sQ; a.sR = problem->sR; a.sQT = problem->sQT;
  a.sx0 = problem->sx0;
  a.P0 = solution->P0; a.K0 = solution->K0; a.u0 = solution->u0; a.value = solution->value;
  a.info = solution->info;
  a.ws = static_cast<float*>(workspace);
  const bool doubling = (problem->flags & TTC_FLAG_DOUBLING) != 0;
  const bool quad = ttc::use_quad_kernel(problem);
  const bool small = problem->d == 16 && !doubling;  // d = 16: the kernel with a lane per row of the dense solves
  const long long gb = ttc::grid_blocks(doubling ? ttc::KIND_DOUBLING : small ? ttc::KIND_SOLVE_QUAD : ttc::KIND_SOLVE,
                                        problem->d, problem->in_dtype == TTC_BF16);
  // work items of the persistent grid: problems, or quads of problems
  const long long items = quad ? (problem->n + 3) / 4 : problem->n;
  const dim3 grid((unsigned)(items < gb ? items : gb));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (problem->flags & TTC_FLAG_DOUBLING) {
    // Q_T "is Q" when it is absent or the very same array: then P_T = Q = f(0) and the recursion starts at 0
    ttc::DoublingArgs da;
    const bool qt_is_q = !problem->QT || (problem->QT == problem->Q && problem->sQT == problem->sQ);
    da.s = a;
    da.m = qt_is_q ? problem->T : problem->T - 1;
    da.p_from_qt = qt_is_q ? 0 : 1;
    e = problem->in_dtype == TTC_F32 ? ttc::launch_doubling<float>(da, problem->d, grid, s)
                                     : ttc::launch_doubling<uint16_t>(da, problem->d, grid, s);
  } else if (quad) {
    if (problem->in_dtype == TTC_F32) hipLaunchKernelGGL((ttc::solve_small_kernel<float, 4>), grid, dim3(64), 0, s, a);
    else hipLaunchKernelGGL((ttc::solve_small_kernel<uint16_t, 4>), grid, dim3(64), 0, s, a);
    e = hipGetLastError();
  } else if (small) {  // a batch that does not fill the chip: one problem to a wavefront
    if (problem->in_dtype == TTC_F32) hipLaunchKernelGGL((ttc::solve_small_kernel<float, 1>), grid, dim3(64), 0, s, a);
    else hipLaunchKernelGGL((ttc::solve_small_kernel<uint16_t, 1>), grid, dim3(64), 0, s, a);
    e = hipGetLastError();
  } else {
    e = problem->in_dtype == TTC_F32 ? ttc::launch_solve<float>(a, problem->d, grid, s)
                                     : ttc::launch_solve<uint16_t>(a, problem->d, grid, s);
  }
  return e == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

ttc_status_t ttc_lqr_rollout(const ttc_lqr_problem_t* problem, float* U, float* X, float* cost,
                             int32_t* info, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t st = ttc::validate(problem);
  if (st != TTC_OK) return st;
  if (problem->n == 0) return TTC_OK;
  if (!U) return TTC_ERR_INVALID_ARG;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) ||
      workspace_bytes < ttc_lqr_workspace_bytes(problem, 1))
    return TTC_ERR_WORKSPACE;
  ttc::RolloutArgs a;
  a.n = problem->n;
  a.T = problem->T;
  a.flags = problem->flags;
  a.A = problem->A; a.B = problem->B; a.Q = problem->Q; a.R = problem->R; a.QT = problem->QT; a.x0 = problem->x0;
  a.sA = problem->sA; a.sB = problem->sB; a.sQ = problem->sQ; a.sR = problem->sR; a.sQT = problem->sQT;
  a.sx0 = problem->sx0;
  a.U = U; a.X = X; a.cost = cost; a.info = info;
  a.ws = static_cast<float*>(workspace);
  const long long gb = ttc::grid_blocks(ttc::KIND_ROLLOUT, problem->d, problem->in_dtype == TTC_BF16);
  const dim3 grid((unsigned)(problem->n < gb ? problem->n : gb));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const hipError_t e = problem->in_dtype == TTC_F32 ? ttc::launch_rollout<float>(a, problem->d, grid, s)
                                                     : ttc::launch_rollout<uint16_t>(a, problem->d, grid, s);
  return e == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

static ttc_status_t validate_tv(const ttc_lqr_tv_problem_t* q) {
  if (!q) return TTC_ERR_INVALID_ARG;
  if (q->n < 0 || q->T < 1 || q->d < 1 || q->m < 1 || q->flags != 0) return TTC_ERR_INVALID_ARG;
  if (q->in_dtype != TTC_F32 && q->in_dtype != TTC_BF16) return TTC_ERR_INVALID_ARG;
  if (!(q->d == q->m && (q->d == 16 || q->d == 32 || q->d == 64 || q->d == 128))) return TTC_ERR_UNSUPPORTED;
  if (q->n == 0) return TTC_OK;
  if (!q->A || !q->B || !q->Q || !q->R || !q->x0) return TTC_ERR_INVALID_ARG;
  const size_t al = q->in_dtype == TTC_F32 ? 16 : 8;
  const void* ptrs[] = {q->A, q->B, q->Q, q->R};
  const int64_t strides[] = {q->sA, q->sB, q->sQ, q->sR, q->tA, q->tB, q->tQ, q->tR};
  for (int k = 0; k < 4; ++k)
    if (!ttc::aligned_ptr(ptrs[k], al)) return TTC_ERR_INVALID_ARG;
  for (int k = 0; k < 8; ++k)
    if (strides[k] < 0 || strides[k] % 4) return TTC_ERR_INVALID_ARG;
  if (q->sx0 < 0) return TTC_ERR_INVALID_ARG;
  return TTC_OK;
}

size_t ttc_lqr_tv_rollout_workspace_bytes(const ttc_lqr_tv_problem_t* q) {
  if (!q || q->T < 1 || !(q->d == q->m && (q->d == 16 || q->d == 32 || q->d == 64 || q->d == 128))) return 0;
  const size_t slots = (size_t)ttc::grid_blocks(ttc::KIND_ROLLOUT_TV, q->d, q->in_dtype == TTC_BF16);
  return slots * (size_t)q->T * q->d * q->m * sizeof(float);
}

ttc_status_t ttc_lqr_rollout_tv(const ttc_lqr_tv_problem_t* q, float* U, float* X, float* cost, int32_t* info,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t stv = validate_tv(q);
  if (stv != TTC_OK) return stv;
  if (q->n == 0) return TTC_OK;
  if (!U) return TTC_ERR_INVALID_ARG;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_lqr_tv_rollout_workspace_bytes(q))
    return TTC_ERR_WORKSPACE;
  ttc::TvRolloutArgs a;
  a.r.n = q->n;
  a.r.T = q->T;
  a.r.flags = 0;
  a.r.A = q->A; a.r.B = q->B; a.r.Q = q->Q; a.r.R = q->R; a.r.QT = nullptr; a.r.x0 = q->x0;
  a.r.sA = q->sA; a.r.sB = q->sB; a.r.sQ = q->sQ; a.r.sR = q->sR; a.r.sQT = 0; a.r.sx0 = q->sx0;
  a.r.U = U; a.r.X = X; a.r.cost = cost; a.r.info = info;
  a.r.ws = static_cast<float*>(workspace);
  a.tA = q->tA; a.tB = q->tB; a.tQ = q->tQ; a.tR = q->tR;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const long long gb = ttc::grid_blocks(ttc::KIND_ROLLOUT_TV, q->d, bf16);
  const dim3 grid((unsigned)(q->n < gb ? q->n : gb));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const hipError_t e = bf16 ? ttc::launch_rollout_tv<uint16_t>(a, q->d, grid, st)
                            : ttc::launch_rollout_tv<float>(a, q->d, grid, st);
  return e == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

ttc_status_t ttc_lqr_solve_tv(const ttc_lqr_tv_problem_t* q, const ttc_lqr_solution_t* solution, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  const ttc_status_t stv = validate_tv(q);
  if (stv != TTC_OK) return stv;
  if (!solution) return TTC_ERR_INVALID_ARG;
  if (q->n == 0) return TTC_OK;
  if (!solution->u0) return TTC_ERR_INVALID_ARG;
  if (!ttc::aligned_ptr(solution->P0, 16) || !ttc::aligned_ptr(solution->K0, 16)) return TTC_ERR_INVALID_ARG;
  ttc::TvArgs a;
  a.s.n = q->n;
  a.s.T = q->T;
  a.s.flags = 0;
  a.s.ngroups = q->T;
  a.s.explicit_groups = 0;
  a.s.A = q->A; a.s.B = q->B; a.s.Q = q->Q; a.s.R = q->R; a.s.QT = nullptr; a.s.x0 = q->x0;
  a.s.sA = q->sA; a.s.sB = q->sB; a.s.sQ = q->sQ; a.s.sR = q->sR; a.s.sQT = 0; a.s.sx0 = q->sx0;
  a.s.P0 = solution->P0; a.s.K0 = solution->K0; a.s.u0 = solution->u0; a.s.value = solution->value;
  a.s.info = solution->info;
  a.s.ws = nullptr;
  a.tA = q->tA; a.tB = q->tB; a.tQ = q->tQ; a.tR = q->tR;
  const bool bf16 = q->in_dtype == TTC_BF16;
  // d = 16: the kernel with a lane per row of the dense solves; batches that fill the chip go four problems
  // to a wavefront, smaller ones one problem to a wavefront
  const bool small = q->d == 16;
  const bool quad = small && q->n >= 8LL * ttc::cu_count();
  const long long gb = ttc::grid_blocks(small ? ttc::KIND_TV_QUAD : ttc::KIND_SOLVE_TV, q->d, bf16);
  const long long items = quad ? (q->n + 3) / 4 : q->n;
  const dim3 grid((unsigned)(items < gb ? items : gb));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (quad) {
    if (bf16) hipLaunchKernelGGL((ttc::solve_tv_small_kernel<uint16_t, 4>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((ttc::solve_tv_small_kernel<float, 4>), grid, dim3(64), 0, st, a);
    e = hipGetLastError();
  } else if (small) {
    if (bf16) hipLaunchKernelGGL((ttc::solve_tv_small_kernel<uint16_t, 1>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((ttc::solve_tv_small_kernel<float, 1>), grid, dim3(64), 0, st, a);
    e = hipGetLastError();
  } else {
    e = bf16 ? ttc::launch_tv<uint16_t>(a, q->d, grid, st) : ttc::launch_tv<float>(a, q->d, grid, st);
  }
  return e == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

size_t ttc_lqr_tv_scan_workspace_bytes(const ttc_lqr_tv_problem_t* q) {
  if (validate_tv(q) != TTC_OK) return 0;
  return (size_t)q->n * (size_t)q->T * 3 * (size_t)q->d * (size_t)q->d * sizeof(float);
}

ttc_status_t ttc_lqr_solve_tv_scan(const ttc_lqr_tv_problem_t* q, const ttc_lqr_solution_t* solution, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t stv = validate_tv(q);
  if (stv != TTC_OK) return stv;
  if (!solution) return TTC_ERR_INVALID_ARG;
  if (q->n == 0) return TTC_OK;
  if (!solution->u0) return TTC_ERR_INVALID_ARG;
  if (!ttc::aligned_ptr(solution->P0, 16) || !ttc::aligned_ptr(solution->K0, 16)) return TTC_ERR_INVALID_ARG;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_lqr_tv_scan_workspace_bytes(q))
    return TTC_ERR_WORKSPACE;
  ttc::ScanArgs sa;
  ttc::TvArgs& a = sa.tv;
  a.s.n = q->n;
  a.s.T = q->T;
  a.s.flags = 0;
  a.s.ngroups = q->T;
  a.s.explicit_groups = 0;
  a.s.A = q->A; a.s.B = q->B; a.s.Q = q->Q; a.s.R = q->R; a.s.QT = nullptr; a.s.x0 = q->x0;
  a.s.sA = q->sA; a.s.sB = q->sB; a.s.sQ = q->sQ; a.s.sR = q->sR; a.s.sQT = 0; a.s.sx0 = q->sx0;
  a.s.P0 = solution->P0; a.s.K0 = solution->K0; a.s.u0 = solution->u0; a.s.value = solution->value;
  a.s.info = solution->info;
  a.s.ws = nullptr;
  a.tA = q->tA; a.tB = q->tB; a.tQ = q->tQ; a.tR = q->tR;
  sa.ws = static_cast<float*>(workspace);
  sa.stride = 0;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const int d = q->d;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const long long gb = ttc::grid_blocks(ttc::KIND_SCAN, d, bf16);
  auto grid_for = [&](long long items) { return dim3((unsigned)(items < gb ? items : gb)); };
  hipError_t e = bf16 ? ttc::launch_scan_leaf<uint16_t>(sa, d, grid_for(q->n * q->T), st)
                      : ttc::launch_scan_leaf<float>(sa, d, grid_for(q->n * q->T), st);
  if (e != hipSuccess) return TTC_ERR_DEVICE;
  for (long long stride = 1; stride < q->T; stride *= 2) {
    sa.stride = (int)stride;
    const long long per = (q->T - stride + 2 * stride - 1) / (2 * stride);
    e = ttc::launch_scan_combine(sa, d, grid_for(q->n * per), st);
    if (e != hipSuccess) return TTC_ERR_DEVICE;
  }
  // the step s = 0 as printed, from P_1 = H of the first element
  ttc::TvArgs last = a;
  last.s.T = 1;
  last.s.ngroups = 1;
  last.PT = sa.ws + 2 * (size_t)d * d;
  last.sPT = (long long)q->T * 3 * d * d;
  const long long gt = ttc::grid_blocks(ttc::KIND_SOLVE_TV, d, bf16);
  const dim3 grid((unsigned)(q->n < gt ? q->n : gt));
  e = bf16 ? ttc::launch_tv<uint16_t>(last, d, grid, st) : ttc::launch_tv<float>(last, d, grid, st);
  return e == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

static ttc_status_t validate_cxt(const ttc_lqr_cxt_problem_t* q) {
  if (!q || q->n < 0 || q->T < 1 || q->r < 1 || q->d < 1 || q->flags != 0) return TTC_ERR_INVALID_ARG;
  if (q->in_dtype != TTC_F32 && q->in_dtype != TTC_BF16) return TTC_ERR_INVALID_ARG;
  if (q->d != 16 || q->r > ttc::CXT_RMAX) return TTC_ERR_UNSUPPORTED;
  if (q->n == 0) return TTC_OK;
  const void* ins[] = {q->sA, q->sB, q->sQ, q->sQf, q->rinv, q->lgA, q->lgB, q->lgQ, q->x0, q->Bbasis, q->Qbasis};
  const size_t esz = q->in_dtype == TTC_BF16 ? 2 : 4;
  for (const void* ptr : ins)
    if (!ptr || !ttc::aligned_ptr(ptr, esz)) return TTC_ERR_INVALID_ARG;
  return TTC_OK;
}

static void fill_cxt_args(ttc::CxtArgs& a, const ttc_lqr_cxt_problem_t* q) {
  a.s.n = q->n;
  a.s.T = q->T;
  a.s.flags = 0;
  a.s.ngroups = q->T;
  a.s.explicit_groups = 0;
  a.s.A = a.s.B = a.s.Q = a.s.R = a.s.QT = nullptr;
  a.s.x0 = q->x0;
  a.s.sA = a.s.sB = a.s.sQ = a.s.sR = a.s.sQT = 0;
  a.s.sx0 = q->d;
  a.s.P0 = a.s.K0 = a.s.u0 = a.s.value = nullptr;
  a.s.info = nullptr;
  a.s.ws = nullptr;
  a.r = q->r;
  a.sA = q->sA; a.sB = q->sB; a.sQ = q->sQ; a.sQf = q->sQf; a.rinv = q->rinv;
  a.lgA = q->lgA; a.lgB = q->lgB; a.lgQ = q->lgQ;
  a.Bbasis = q->Bbasis; a.Qbasis = q->Qbasis;
  a.roll_ws = nullptr;
}

static hipError_t launch_cxt(const ttc::CxtArgs& a, bool bf16, hipStream_t st) {
  const long long gb = ttc::grid_blocks(ttc::KIND_CXT, 16, bf16);
  // batches that do not fill the resident wavefronts four problems at a time go one problem to a wavefront
  const bool single = a.s.n <= gb;
  const long long items = single ? a.s.n : (a.s.n + 3) / 4;
  const dim3 grid((unsigned)(items < gb ? items : gb));
  if (single) {
    if (bf16) hipLaunchKernelGGL((ttc::solve_cxt_kernel<uint16_t, 1>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((ttc::solve_cxt_kernel<float, 1>), grid, dim3(64), 0, st, a);
  } else {
    if (bf16) hipLaunchKernelGGL((ttc::solve_cxt_kernel<uint16_t, 4>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((ttc::solve_cxt_kernel<float, 4>), grid, dim3(64), 0, st, a);
  }
  return hipGetLastError();
}

ttc_status_t ttc_lqr_solve_cxt(const ttc_lqr_cxt_problem_t* q, const ttc_lqr_solution_t* solution, void* hip_stream) {
  const ttc_status_t sv = validate_cxt(q);
  if (sv != TTC_OK) return sv;
  if (!solution) return TTC_ERR_INVALID_ARG;
  if (q->n == 0) return TTC_OK;
  if (!solution->u0) return TTC_ERR_INVALID_ARG;
  if (!ttc::aligned_ptr(solution->P0, 16) || !ttc::aligned_ptr(solution->K0, 16)) return TTC_ERR_INVALID_ARG;
  ttc::CxtArgs a;
  fill_cxt_args(a, q);
  a.s.P0 = solution->P0; a.s.K0 = solution->K0; a.s.u0 = solution->u0; a.s.value = solution->value;
  a.s.info = solution->info;
  return launch_cxt(a, q->in_dtype == TTC_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TTC_OK
                                                                                                     : TTC_ERR_DEVICE;
}

size_t ttc_lqr_cxt_rollout_workspace_bytes(const ttc_lqr_cxt_problem_t* q) {
  if (validate_cxt(q) != TTC_OK) return 0;
  // per problem: Bbar, Qbar, Q_T and the T gains (256 floats each), then one breakdown flag per problem
  const size_t mats = (size_t)q->n * (size_t)(q->T + 3) * 256 * sizeof(float);
  return mats + (((size_t)q->n * sizeof(int32_t) + 15) & ~(size_t)15);
}

ttc_status_t ttc_lqr_rollout_cxt(const ttc_lqr_cxt_problem_t* q, float* U, float* X, float* cost, int32_t* info,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t sv = validate_cxt(q);
  if (sv != TTC_OK) return sv;
  if (q->n == 0) return TTC_OK;
  if (!U) return TTC_ERR_INVALID_ARG;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_lqr_cxt_rollout_workspace_bytes(q))
    return TTC_ERR_WORKSPACE;
  ttc::CxtRolloutArgs ra;
  fill_cxt_args(ra.c, q);
  ra.c.roll_ws = static_cast<float*>(workspace);
  ra.c.s.info = info ? info : reinterpret_cast<int*>(ra.c.roll_ws + (size_t)q->n * (size_t)(q->T + 3) * 256);
  ra.U = U; ra.X = X; ra.cost = cost;
  const bool bf16 = q->in_dtype == TTC_BF16;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (launch_cxt(ra.c, bf16, st) != hipSuccess) return TTC_ERR_DEVICE;  // backward sweep: gains into the workspace
  const long long groups = (q->n + 3) / 4;
  const long long gb = 32LL * ttc::cu_count();
  const dim3 grid((unsigned)(groups < gb ? groups : gb));
  if (bf16) hipLaunchKernelGGL((ttc::rollout_cxt_forward_kernel<uint16_t>), grid, dim3(64), 0, st, ra);
  else hipLaunchKernelGGL((ttc::rollout_cxt_forward_kernel<float>), grid, dim3(64), 0, st, ra);
  return hipGetLastError() == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

const char* ttc_status_string(ttc_status_t status) {
  switch (status) {
    case TTC_OK: return "ok";
    case TTC_ERR_INVALID_ARG: return "invalid argument";
    case TTC_ERR_UNSUPPORTED: return "unsupported shape or option";
    case TTC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case TTC_ERR_DEVICE: return "HIP runtime error at launch";
  }
  return "unknown status";
}

int ttc_version(void) { return 200; }

}  // extern "C"
