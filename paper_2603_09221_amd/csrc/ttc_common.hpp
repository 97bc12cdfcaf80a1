// Argument blocks and device helpers shared by every kernel family of the batched LQR solver
// (see include/ttc_lqr.h for the operations).  Each family is compiled in its own translation unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ttc_lqr.h"
#include "ttc_device.hpp"
#include "ttc_args.hpp"

namespace ttc {

// Development aid: with -DTTC_PHASE_TIMERS, workgroup 0 accumulates s_memtime ticks per phase and adds
// them to the eight counters of the argument block's debug buffer; otherwise no code.
#ifdef TTC_PHASE_TIMERS
#define TTC_TIMER_DECL long long tt_[8] = {0, 0, 0, 0, 0, 0, 0, 0}; long long tt0_ = __builtin_amdgcn_s_memtime();
#define TTC_TOC(k) { const long long now_ = __builtin_amdgcn_s_memtime(); tt_[k] += now_ - tt0_; tt0_ = now_; }
#define TTC_TIMER_DUMP(args) if (threadIdx.x == 0 && blockIdx.x == 0 && (args).dbg) { for (int k_ = 0; k_ < 8; ++k_) (args).dbg[k_] += tt_[k_]; }
#else
#define TTC_TIMER_DECL
#define TTC_TOC(k)
#define TTC_TIMER_DUMP(args)
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
  template <typename Args>
  __device__ __forceinline__ void dump(const Args& args) const {
    if (threadIdx.x == 0 && blockIdx.x == 0 && args.dbg)
      for (int k = 0; k < 8; ++k) args.dbg[k] += t[k];
  }
#else
  __device__ __forceinline__ void toc(int) {}
  template <typename Args>
  __device__ __forceinline__ void dump(const Args&) const {}
#endif
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
// (A matrix is a whole number of pieces per thread, so a thread reads all its pieces or none: one test around the
// reads instead of one per piece, inside which the compiler waits for every 16-byte read on its own.)
template <int D, typename TIn>
__device__ __forceinline__ void issue_half(HalfRegs<D>& h, const TIn* M, int tid) {
  using C = Cfg<D>;
  static_assert((D * D / 4) % C::NTHR == 0, "a matrix is a whole number of 16-byte pieces per thread");
  if (tid < C::NTHR) {
#pragma unroll
    for (int k = 0; k < HalfRegs<D>::NV; ++k) {
      const int idx = tid + k * C::NTHR;
      h.v[k] = ld4<TIn>(M, (long)(idx / (D / 4)) * D + (idx % (D / 4)) * 4);
    }
  }
}
template <int D, bool TRANS>
__device__ __forceinline__ void commit_half(float* Wh, const HalfRegs<D>& h, int tid) {
  using C = Cfg<D>;
  if (tid < C::NTHR) {
#pragma unroll
    for (int k = 0; k < HalfRegs<D>::NV; ++k) {
      const int idx = tid + k * C::NTHR;
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
// into 4 x 4 blocks; a thread takes a block pair (bi, bj), reads both blocks with 16-byte LDS reads, averages
// each with the other's transpose in registers and writes them back.  Consecutive lanes take consecutive
// pairs of one diagonal, (bi, bj) = ((j + s) mod NB, j) for j = 0, 1, ...: both blocks then move by four rows
// and four columns from lane to lane, 4 * PITCH + 4 = 20 (mod 64) words, which spreads sixteen lanes' 16-byte
// accesses over all banks (walking along a row of blocks instead, the lower blocks of a wavefront would share
// four banks).  Diagonals s = 0 .. NB/2 hold every unordered pair once (the last one only its first half).
template <int D>
__device__ __forceinline__ void symmetrise_half(float* Wh, int tid) {
  using C = Cfg<D>;
  constexpr int NB = D / 4;
  constexpr int NITEM = NB * (NB / 2) + NB / 2;  // diagonals 0 .. NB/2-1 in full, half of diagonal NB/2
  for (int idx = tid; idx < NITEM; idx += C::NTHR) {
    const int sd = idx / NB, bj = idx % NB, bi = (bj + sd) % NB;
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
        const float sy = 0.5f * (u[r][c] + l[c][r]);
        un[r][c] = sy;
        ln[c][r] = sy;
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

}  // namespace ttc
