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

#ifndef TTC_PIVOT_THRESHOLD
#define TTC_PIVOT_THRESHOLD 0.25f  // a diagonal entry this close to the column's largest is taken as the pivot
#endif
// Dense solves M X = RHS of the four 16 x 32 augmented arrays Wm[q] = [M | RHS] (row r at
// Wm[q] + r*PITCH), all at once: Gauss-Jordan with partial pivoting, a lane holding one row.  The pivot
// of a column is found by a 16-lane DPP max of a packed key (|value| with the row index in the low
// mantissa bits), the pivot row is broadcast with ds_bpermute, every other row of that problem is
// eliminated.  Rows never move; the row that was the pivot of column c ends up as row c of X, written
// to the right half.  The search is threshold pivoting: row c itself is preferred when it is still free and its
// entry is at least TTC_PIVOT_THRESHOLD times the column's largest (element growth stays bounded by 1 + 1/threshold
// per step instead of 2); when that holds for all four problems of the wavefront, the pivot row is known at compile
// time and is broadcast by DPP (row_newbcast) instead of going through the LDS crossbar, which is what bounds this
// function otherwise.  PIVOT = false always takes the diagonal (symmetric positive definite M).
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
    bool diagonal = !PIVOT;  // the pivot row is lane j of every row of 16 lanes
    if constexpr (PIVOT) {
      uint32_t key = (__float_as_uint(a[j]) & 0x7FFFFF80u) | (uint32_t)(127 - r);
      key = act ? key : 0u;
      // Threshold pivoting: row j itself is taken when it is still free and its entry is within a factor of
      // TTC_PIVOT_THRESHOLD of the column's largest; when that holds for all of the wavefront's problems the
      // pivot row is known at compile time and travels by DPP instead of the LDS crossbar.
      const uint32_t own = (uint32_t)__builtin_amdgcn_mov_dpp((int)key, 0x150 + j, 0xF, 0xF, true);  // row j's key, 0 if used
      key = row16_max_u32(key);
      const float big = __uint_as_float(key & 0x7FFFFF80u), mine_abs = __uint_as_float(own & 0x7FFFFF80u);
      const bool fine = own != 0u && mine_abs >= TTC_PIVOT_THRESHOLD * big;
      diagonal = __ballot(!fine) == 0ull;
      pr = 127 - (int)(key & 0x7Fu);
      pr = pr < 16 ? pr : 15;  // never leave the problem's lanes, whatever the data
      pr = diagonal ? j : pr;
    } else {
      pr = j;
    }
    float prow[32];
    if (PIVOT && !diagonal) {
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
// down (a pivot that is not positive and finite).  NEGATE leaves -M^{-1} instead (the sign rides on the final scaling);
// ONE_WAVE: the workgroup is this wavefront alone, and the final barrier is replaced by an ordering of its LDS
// traffic that does not wait for its global stores.
template <bool NEGATE = false, bool ONE_WAVE = false>
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
  const float s = NEGATE ? -__builtin_amdgcn_rcpf(mypiv) : __builtin_amdgcn_rcpf(mypiv);
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    floatx4 t;
    t[0] = a[4 * k + 0] * s; t[1] = a[4 * k + 1] * s; t[2] = a[4 * k + 2] * s; t[3] = a[4 * k + 3] * s;
    *reinterpret_cast<floatx4*>(Wq + r * C::PITCH + 4 * k) = t;
  }
  if (ONE_WAVE) wave_lds_sync();
  else __syncthreads();
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

}  // namespace ttc
