// The d = 16 shape of the solver: four problems per wavefront.
//
// At d = 16 a problem fills a quarter of a wavefront, and the dense solves (one pivot after the other,
// each a reduction and a broadcast) are most of the instructions.  This kernel gives a workgroup of one
// wavefront four problems at a time: the products are formed problem by problem on the matrix cores
// exactly as in the larger shapes (Z-land pair in LDS, constant row blocks in registers), and the dense
// solves of the four problems run side by side, lane 16q + r owning row r of problem q's augmented
// [M | RHS] in registers.  The method is that of solve_kernel: reverse symplectic steps (Thm 3.3,
// App. C "Kernel Fusion") in groups, a pivoted solve re-basing the pair after each group (Alg. 4's
// P = Y1^{-1} Y2), the last factor with Q_0 = 0, K_0 = -R^{-1} B^T A^{-T} P_0 (Thm A.4).
#pragma once
#include "ttc_common.hpp"

namespace ttc {

// max of an unsigned key over each row of 16 lanes; every lane of the row gets it (DPP only)
__device__ __forceinline__ uint32_t row16_max_u32(uint32_t x) {
  auto mx = [](uint32_t a, uint32_t b) { return a > b ? a : b; };
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, false));  // row_half_mirror
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, false));  // row_mirror
  return x;
}

// Dense solves M X = RHS of the four 16 x 32 augmented arrays Wm[q] = [M | RHS] (row r at
// Wm[q] + r*PITCH), all at once: Gauss-Jordan with partial pivoting, a lane holding one row.  The pivot
// of a column is found by a 16-lane DPP max of a packed key (|value| with the row index in the low
// mantissa bits), the pivot row is broadcast with ds_bpermute, every other row of that problem is
// eliminated.  Rows never move; the row that was the pivot of column c ends up as row c of X, written
// to the right half.  PIVOT = false takes the diagonal (symmetric positive definite M); the pivot row is
// then known at compile time and is broadcast by DPP (row_newbcast) instead.
// Returns, per lane, whether its problem broke down (zero / non-finite / non-positive pivot).
template <bool PIVOT>
__device__ __forceinline__ int solve_rows16(float* Wq, int lane) {
  using C = Cfg<16>;
  const int r = lane & 15;
  float a[32];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const floatx4 t = *reinterpret_cast<const floatx4*>(Wq + r * C::PITCH + 4 * k);
    a[4 * k + 0] = t[0]; a[4 * k + 1] = t[1]; a[4 * k + 2] = t[2]; a[4 * k + 3] = t[3];
  }
  __syncthreads();  // every row is in registers; the right half may be overwritten below
  bool act = true;
  int myj = 0;
  float mypiv = 1.f;
  int bad = 0;
  static_for<0, 16>([&](auto J) {
    constexpr int j = decltype(J)::value;
    int pr;
    if constexpr (PIVOT) {
      uint32_t key = (__float_as_uint(a[j]) & 0x7FFFFF80u) | (uint32_t)(127 - r);
      key = act ? key : 0u;
      key = row16_max_u32(key);
      pr = 127 - (int)(key & 0x7Fu);
      pr = pr < 16 ? pr : 15;  // never leave the problem's lanes, whatever the data
    } else {
      pr = j;
    }
    float prow[32];
    if constexpr (PIVOT) {
      const int src = ((lane & 48) | pr) << 2;  // byte address of the pivot row's lane
      static_for<j, 32>([&](auto K) {
        constexpr int k = decltype(K)::value;
        prow[k] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, __builtin_bit_cast(int, a[k])));
      });
    } else {
      // the pivot row is lane j of every row of 16 lanes: a DPP broadcast within the row, no LDS crossbar
      static_for<j, 32>([&](auto K) {
        constexpr int k = decltype(K)::value;
        prow[k] = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, a[k]), 0x150 + j, 0xF, 0xF,
                                                                      true));  // row_newbcast:j
      });
    }
    const float pv = prow[j];
    const float apv = PIVOT ? fabsf(pv) : pv;
    if (!(apv > 0.f && apv < __builtin_inff())) bad = 1;
    const bool mine = (r == pr);
    const float nl = mine ? 0.f : -a[j] * __builtin_amdgcn_rcpf(pv);
    act = act && !mine;
    myj = mine ? j : myj;
    mypiv = mine ? pv : mypiv;
    static_for<j + 1, 32>([&](auto K) {
      constexpr int k = decltype(K)::value;
      a[k] = __builtin_fmaf(prow[k], nl, a[k]);  // nl = 0 for the pivot row itself
    });
  });
  const float s = __builtin_amdgcn_rcpf(mypiv);
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    floatx4 t;
    t[0] = a[16 + 4 * k + 0] * s; t[1] = a[16 + 4 * k + 1] * s; t[2] = a[16 + 4 * k + 2] * s; t[3] = a[16 + 4 * k + 3] * s;
    *reinterpret_cast<floatx4*>(Wq + myj * C::PITCH + 16 + 4 * k) = t;
  }
  __syncthreads();
  return bad;
}

// In-place inverses of the four symmetric positive definite 16 x 16 matrices in the left halves of
// Wm[q] (row r at Wq + r*PITCH), all at once, a lane holding one row: Gauss-Jordan without pivoting on
// [M | I], where the column of the right part that becomes non-trivial at step j takes the place of
// column j of M, which has just become a unit vector.  Rows are scaled by their pivots at the end.
// The pivot row is broadcast within each row of 16 lanes by DPP.  The caller synchronises before (M
// complete in LDS); the function ends with a barrier.  Returns, per lane, whether its problem broke
// down (a pivot that is not positive and finite).
__device__ __forceinline__ int invert_rows16(float* Wq, int lane) {
  using C = Cfg<16>;
  const int r = lane & 15;
  float a[16];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const floatx4 t = *reinterpret_cast<const floatx4*>(Wq + r * C::PITCH + 4 * k);
    a[4 * k + 0] = t[0]; a[4 * k + 1] = t[1]; a[4 * k + 2] = t[2]; a[4 * k + 3] = t[3];
  }
  float mypiv = 1.f;
  int bad = 0;
  static_for<0, 16>([&](auto J) {
    constexpr int j = decltype(J)::value;
    const float pv = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, a[j]), 0x150 + j, 0xF, 0xF,
                                                                         true));  // row_newbcast:j: the pivot
    if (!(pv > 0.f && pv < __builtin_inff())) bad = 1;
    const bool mine = (r == j);
    const float nl = mine ? 0.f : -a[j] * __builtin_amdgcn_rcpf(pv);  // 0 for the pivot row itself
    mypiv = mine ? pv : mypiv;
    // a[k] += nl * (a[k] of the pivot row, lane j of this row of 16 lanes), k != j: the broadcast rides on the
    // multiply-add as its DPP operand.  Written as one block so that the wait states a DPP read needs after a
    // vector write of the same register are in our hands: within the block every instruction touches its own
    // register, and the block starts and ends with the two idle states.
#define TTC_AK(n) a[(n) < j ? (n) : (n) + 1]  // the 15 registers other than a[j], in ascending order
    asm volatile(
        "s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %4, %4, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %5, %5, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %6, %6, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %7, %7, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %8, %8, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %9, %9, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %10, %10, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %11, %11, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %12, %12, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %13, %13, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %14, %14, %15 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(TTC_AK(0)), "+v"(TTC_AK(1)), "+v"(TTC_AK(2)), "+v"(TTC_AK(3)), "+v"(TTC_AK(4)), "+v"(TTC_AK(5)),
          "+v"(TTC_AK(6)), "+v"(TTC_AK(7)), "+v"(TTC_AK(8)), "+v"(TTC_AK(9)), "+v"(TTC_AK(10)), "+v"(TTC_AK(11)),
          "+v"(TTC_AK(12)), "+v"(TTC_AK(13)), "+v"(TTC_AK(14))
        : "v"(nl), "n"(j));
#undef TTC_AK
    a[j] = mine ? 1.f : nl;  // column j of the right part
  });
  const float s = __builtin_amdgcn_rcpf(mypiv);
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    floatx4 t;
    t[0] = a[4 * k + 0] * s; t[1] = a[4 * k + 1] * s; t[2] = a[4 * k + 2] * s; t[3] = a[4 * k + 3] * s;
    *reinterpret_cast<floatx4*>(Wq + r * C::PITCH + 4 * k) = t;
  }
  __syncthreads();
  return bad;
}

// acc[q] += C_q Z_q for the wavefront's PPW problems at once, Z_q = the half of Wm[q] starting at column `half`.
// At d = 16 a product is four dependent matrix-core instructions; taking the k-steps of the four
// problems in turn keeps the pipe busy, and all sixteen B-operand reads are in flight together.
template <int PPW = 4>
__device__ __forceinline__ void gemm_acc_quad(floatx4 (&acc)[PPW][1][1], const float (&a)[PPW][1][4],
                                              float (*Wm)[16 * Cfg<16>::PITCH], int half, int i, int g) {
  using C = Cfg<16>;
  float b[PPW][4];
#pragma unroll
  for (int q = 0; q < PPW; ++q)
#pragma unroll
    for (int t = 0; t < 4; ++t) b[q][t] = Wm[q][half + (4 * g + t) * C::PITCH + i];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int q = 0; q < PPW; ++q)
      acc[q][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[q][0][t], b[q][t], acc[q][0][0], 0, 0, 0);
}

// PPW = problems per wavefront: 4 for batches that fill the chip, 1 for small ones (the four rows of 16 lanes
// then all hold the same problem and compute, and write, the same values; every per-problem loop runs once).
template <typename TIn, int PPW>
__global__ void __launch_bounds__(64) solve_small_kernel(const SolveArgs p) {
  constexpr int D = 16;
  using C = Cfg<D>;
  static_assert(PPW == 1 || PPW == 4, "one problem or four per wavefront");
  __shared__ __attribute__((aligned(16))) float Wm[PPW][D * C::PITCH];
  __shared__ float s_red[C::NW];
  const bool pure = (p.flags & TTC_FLAG_PURE_SYMPLECTIC) != 0;
  const long long nquads = (p.n + PPW - 1) / PPW;

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
    float* const Wmine = Wm[g & (PPW - 1)];  // the problem whose rows this lane holds during the dense solves
    int info[PPW] = {};
    int nsolve = 0;
    auto note = [&](int bad) {   // fold a dense solve's per-lane breakdown flags into the per-problem info
      ++nsolve;
      const unsigned long long m = __ballot(bad != 0);
#pragma unroll
      for (int q = 0; q < PPW; ++q)
        if (!info[q] && ((m >> (16 * q)) & 0xFFFFull)) info[q] = nsolve;
    };
    PhaseTimers tm;  // phases: 0 set-up, 1 dense solves, 2 steps, 3 outputs
    floatx4 acc[PPW][C::RB][C::NT];
    float cG[PPW][C::RB][C::KS], cAi[PPW][C::RB][C::KS], cAT[PPW][C::RB][C::KS], cQ[PPW][C::RB][C::KS];
    float cCK[PPW][C::RB][C::KS];

    // ---- phase R: X = R^{-1} B^T, G = B X
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      load_half<D, TIn, false>(Wm[q], reinterpret_cast<const TIn*>(p.R) + prob[q] * p.sR, tid);
      load_half<D, TIn, true>(Wm[q] + D, reinterpret_cast<const TIn*>(p.B) + prob[q] * p.sB, tid);  // RHS = B^T
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
    __syncthreads();
    {
      float cB[PPW][C::RB][C::KS], cX[PPW][C::RB][C::KS];
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aopT_lds<D>(Wm[q] + D, cB[q], w, i, g);  // rows of B = columns of B^T
      tm.toc(0);
      note(solve_rows16<false>(Wmine, lane));  // R is positive definite: no pivot search
      tm.toc(1);
#pragma unroll
      for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
      gemm_acc_quad<PPW>(acc, cB, Wm, D, i, g);  // rows of G = B X
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_aop_lds<D>(Wm[q] + D, cX[q], w, i, g);
        store_rows<D>(Wm[q], acc[q], w, i, g);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q], tid);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q], cG[q], w, i, g);
      __syncthreads();
      // ---- phase A: A^{-1}, A^T, Q, C_K = X A^{-T}
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_half<D, TIn, false>(Wm[q], reinterpret_cast<const TIn*>(p.A) + prob[q] * p.sA, tid);
        load_half<D, TIn, false>(Wm[q] + D, reinterpret_cast<const TIn*>(p.Q) + prob[q] * p.sQ, tid);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        symmetrise_half<D>(Wm[q] + D, tid);
        load_aopT_lds<D>(Wm[q], cAT[q], w, i, g);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q] + D, cQ[q], w, i, g);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) set_half_identity<D>(Wm[q] + D, tid);
      __syncthreads();
      tm.toc(0);
      note(solve_rows16<true>(Wmine, lane));
      tm.toc(1);
#pragma unroll
      for (int q = 0; q < PPW; ++q) {
        load_aop_lds<D>(Wm[q] + D, cAi[q], w, i, g);
        load_rows<D>(Wm[q] + D, acc[q], w, i, g);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows_T<D>(Wm[q] + D, acc[q], w, i, g);  // A^{-T}
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
      gemm_acc_quad<PPW>(acc, cX, Wm, D, i, g);  // rows of C_K = X A^{-T}
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) load_aop_lds<D>(Wm[q], cCK[q], w, i, g);
    }
    // initial pair [Y1 Y2] = [I Q_T]
    if (p.QT) {
#pragma unroll
      for (int q = 0; q < PPW; ++q)
        load_half<D, TIn, false>(Wm[q] + D, reinterpret_cast<const TIn*>(p.QT) + prob[q] * p.sQT, tid);
      __syncthreads();
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
    } else {
#pragma unroll
      for (int q = 0; q < PPW; ++q) store_aop_lds<D>(Wm[q] + D, cQ[q], w, i, g);  // Q_T = Q, already symmetric
    }
    __syncthreads();

    tm.toc(0);
    // ---- groups of reverse symplectic steps, each ended by a re-base
    int s = 1;
    bool fresh = true;
    for (int grp = 0;; ++grp) {
      const int gend = p.T - (int)(((long long)(p.ngroups - 1 - grp) * p.T) / p.ngroups);
      for (;; ++s) {
        const bool last = (s >= gend);
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          if (fresh) eye_acc<D>(acc[q], w, i, g); else load_rows<D>(Wm[q], acc[q], w, i, g);
        }
        gemm_acc_quad<PPW>(acc, cG, Wm, D, i, g);   // Z1 + G Z2
#pragma unroll
        for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
        gemm_acc_quad<PPW>(acc, cAi, Wm, 0, i, g);  // A^{-1} (.) = new Z1
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q], acc[q], w, i, g);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PPW; ++q) zero_acc<D>(acc[q]);
        gemm_acc_quad<PPW>(acc, cAT, Wm, D, i, g);              // A^T Z2
        if (s < p.T) gemm_acc_quad<PPW>(acc, cQ, Wm, 0, i, g);  // + Q Z1; Q_0 = 0 for the last factor
        __syncthreads();
        fresh = false;
        if (!last) {
#pragma unroll
          for (int q = 0; q < PPW; ++q) store_rows<D>(Wm[q] + D, acc[q], w, i, g);
          __syncthreads();
          if (pure) {
#pragma unroll
            for (int q = 0; q < PPW; ++q) normalise_rows_zland<D>(Wm[q], tid);
            __syncthreads();
          }
        } else {
          // leave Z-land: [Y1 | Y2] untransposed for the solve Y1 P = Y2
          floatx4 z1[PPW][C::RB][C::NT];
#pragma unroll
          for (int q = 0; q < PPW; ++q) {
            store_rows_T<D>(Wm[q] + D, acc[q], w, i, g);
            load_rows<D>(Wm[q], z1[q], w, i, g);
          }
          __syncthreads();
#pragma unroll
          for (int q = 0; q < PPW; ++q) store_rows_T<D>(Wm[q], z1[q], w, i, g);
          __syncthreads();
          ++s;
          break;
        }
      }
      tm.toc(2);
      note(solve_rows16<true>(Wmine, lane));
      tm.toc(1);
#pragma unroll
      for (int q = 0; q < PPW; ++q) symmetrise_half<D>(Wm[q] + D, tid);
      __syncthreads();
      fresh = true;
      if (s > p.T) break;
    }

    tm.toc(2);
    // ---- outputs: the right halves hold P_0 (paper convention, Q_0 = 0)
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
      if (!valid[q]) continue;  // uniform over the wavefront
      const TIn* Qp = reinterpret_cast<const TIn*>(p.Q) + prob[q] * p.sQ;
      const TIn* x0p = reinterpret_cast<const TIn*>(p.x0) + prob[q] * p.sx0;
      zero_acc<D>(acc[q]);
      gemm_acc<D>(acc[q], cCK[q], Wm[q] + D, i, g);  // -K_0 = C_K P_0
      emit_gain<D, TIn>(p, prob[q], acc[q], x0p, info[q], tid);
      emit_value<D, TIn>(p, prob[q], Wm[q] + D, Qp, x0p, info[q], s_red, tid);
    }
    __syncthreads();
    tm.toc(3);
    tm.dump(p);
  }
}

}  // namespace ttc
