// Device-side building blocks of the batched LQR solver (gfx950 / CDNA4, wave64).
//
// One workgroup solves one problem at a time.  Every d x d product is formed in 16-row blocks; a
// wavefront owns RB of them (two at d >= 32: 256 threads at d = 128, one wavefront per SIMD, so that
// each wavefront may use the whole 512-entry register file).  The d x 2d pair [Y1 Y2] of the reverse
// symplectic iteration (Thm 3.3) lives in LDS in transposed form Z = [Y1 Y2]^T ("Z-land": left
// half Z1 = Y1^T, right half Z2 = Y2^T), so that one factored step (App. C "Kernel Fusion")
//     Y1 <- (Y1 + Y2 G) A^{-T},   Y2 <- Y2 A + Y1 Q
// becomes left-multiplications by constant matrices,
//     Z1 <- A^{-1} (Z1 + G Z2),   Z2 <- A^T Z2 + Q Z1,
// whose row blocks stay in the owning wavefront's registers for the whole horizon (MFMA A operand)
// while the state is the shared MFMA B operand read from LDS.  Nothing is re-read from HBM inside
// the horizon loop.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// 16-row blocks per wavefront as a function of d (workgroup = d/16/RB wavefronts)
#ifndef TTC_ROW_BLOCKS
#define TTC_ROW_BLOCKS(D) ((D) >= 32 ? 2 : 1)
#endif
// column tiles a wavefront updates in one batch of the dense solve (registers: 4*NRT*NTC accumulators)
#ifndef TTC_SOLVE_NTC
#define TTC_SOLVE_NTC 4
#endif
#ifndef TTC_SCHED_BARRIER
#define TTC_SCHED_BARRIER() __builtin_amdgcn_sched_barrier(0)
#endif

namespace ttc {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// compile-time loop: f(std::integral_constant<int, I>) for I = B..E-1.  Used where register arrays
// must only ever be indexed by constants (a plain "#pragma unroll" is a request, not a guarantee).
template <int I>
struct IntC { static constexpr int value = I; };
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(IntC<B>{});
    static_for<B + 1, E>(f);
  }
}

// A zero the compiler cannot see through.  Added to a thread index, it makes the address arithmetic
// derived from it start at that point of the program: otherwise the compiler computes every LDS and
// global address of the whole kernel once, ahead of the loop over problems, and spills most of them.
__device__ __forceinline__ int opaque_zero() {
  int z = 0;
  asm volatile("" : "+v"(z));
  return z;
}

__device__ __forceinline__ int opaque_int(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

template <int D>
struct Cfg {
  static constexpr int RB = TTC_ROW_BLOCKS(D);  // 16-row blocks owned by one wavefront
  static constexpr int NRT = D / 16;            // 16-row blocks (= 16-column tiles) of a d x d matrix
  static constexpr int NW = NRT / RB;           // wavefronts per workgroup
  static constexpr int NTHR = 64 * NW;          // threads per workgroup (256 at d = 128: one wave per SIMD)
  static constexpr int KS = D / 4;              // k-steps of v_mfma_f32_16x16x4_f32 per product
  static constexpr int NT = D / 16;             // 16-column tiles per row block
  static constexpr int VEC = NT >= 4 ? 4 : NT;  // consecutive floats per B-operand LDS read
  static constexpr int NH = NT / VEC;           // B-operand reads per k-step
  static constexpr int PITCH = 2 * D + 4;       // floats per LDS row of the d x 2d pair (+4: bank skew)
};

// ----------------------------------------------------------------------------------------------
// input element access: float32 or bfloat16 (stored as uint16_t), widened to float32
template <typename TIn>
__device__ __forceinline__ float ld1(const TIn* p, long i);
template <>
__device__ __forceinline__ float ld1<float>(const float* p, long i) { return p[i]; }
template <>
__device__ __forceinline__ float ld1<uint16_t>(const uint16_t* p, long i) {
  return __uint_as_float(((uint32_t)p[i]) << 16);
}
// Orders the wavefront's own LDS traffic without waiting for its global loads: a workgroup here is one wavefront,
// whose LDS instructions execute in issue order, so what one lane wrote is what another lane reads after this point
// once the compiler keeps the order.  A workgroup barrier would also drain every load in flight, which kernels that
// keep loads or stores in flight across their LDS exchanges rely on not happening.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename TIn>
__device__ __forceinline__ floatx4 ld4(const TIn* p, long i);  // i % 4 == 0, p + i vector-aligned
template <>
__device__ __forceinline__ floatx4 ld4<float>(const float* p, long i) {
  return *reinterpret_cast<const floatx4*>(p + i);
}
template <>
__device__ __forceinline__ floatx4 ld4<uint16_t>(const uint16_t* p, long i) {
  uint2 u = *reinterpret_cast<const uint2*>(p + i);
  floatx4 r;
  r[0] = __uint_as_float(u.x << 16);
  r[1] = __uint_as_float(u.x & 0xffff0000u);
  r[2] = __uint_as_float(u.y << 16);
  r[3] = __uint_as_float(u.y & 0xffff0000u);
  return r;
}

// ----------------------------------------------------------------------------------------------
// LDS access of VEC consecutive floats
template <int VEC>
__device__ __forceinline__ void lds_ldv(const float* p, float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    floatx4 t = *reinterpret_cast<const floatx4*>(p);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
  } else if constexpr (VEC == 2) {
    floatx2 t = *reinterpret_cast<const floatx2*>(p);
    v[0] = t[0]; v[1] = t[1];
  } else {
    v[0] = p[0];
  }
}
template <int VEC>
__device__ __forceinline__ void lds_stv(float* p, const float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    floatx4 t; t[0] = v[0]; t[1] = v[1]; t[2] = v[2]; t[3] = v[3];
    *reinterpret_cast<floatx4*>(p) = t;
  } else if constexpr (VEC == 2) {
    floatx2 t; t[0] = v[0]; t[1] = v[1];
    *reinterpret_cast<floatx2*>(p) = t;
  } else {
    p[0] = v[0];
  }
}

// ----------------------------------------------------------------------------------------------
// wavefront reductions
// max over the 64 lanes of an unsigned key, returned as a wave-uniform value (DPP only)
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  auto mx = [](uint32_t a, uint32_t b) { return a > b ? a : b; };
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, false));  // row_half_mirror
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, false));  // row_mirror
  // every lane of a row now holds its row's max; fold the four rows: row_bcast15 into rows 1 and 3,
  // row_bcast31 into rows 2 and 3, so that lane 63 ends up with the max of all 64 lanes
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xA, 0xF, false));
  x = mx(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xC, 0xF, false));
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
// max over the 64 lanes of a non-negative float (NaN counts as larger than every number), wave-uniform
__device__ __forceinline__ float wave_max_nonneg(float x) {
  return __uint_as_float(wave_max_u32(__float_as_uint(x)));
}
// sum over the 16 lanes that share lane/16 (xor butterflies 1,2,4,8)
__device__ __forceinline__ float sum16(float x) {
  x += __shfl_xor(x, 1, 64);
  x += __shfl_xor(x, 2, 64);
  x += __shfl_xor(x, 4, 64);
  x += __shfl_xor(x, 8, 64);
  return x;
}
__device__ __forceinline__ float sum64(float x) {
  x = sum16(x);
  x += __shfl_xor(x, 16, 64);
  x += __shfl_xor(x, 32, 64);
  return x;
}

// ----------------------------------------------------------------------------------------------
// Row-block product on the matrix cores: acc(16 x D) += C[16w:16w+16, :] * Z(D x D) for each row block w of the wavefront.
//
// v_mfma_f32_16x16x4_f32 operand layout (lane = 16 g + i): A operand = A[i][g], B operand =
// B[g][i], accumulator register v = D[4 g + v][i].
//   * a[4q+t] holds C[16w+i][16q+4g+t]: the contraction index is visited in the permuted order
//     k(q,t,g) = 16q + 4g + t so that a lane's four values for fixed q are contiguous in memory.
//   * the matching B operand is row k(q,t,g) of Z; one LDS read of VEC consecutive floats at
//     column 16*VEC*h + VEC*i feeds VEC tiles, i.e. tile c = h*VEC + tp covers the strided column
//     set { 16*VEC*h + VEC*i + tp : i = 0..15 }.
//   * acc[c][v] is therefore element (row 16w+4g+v, column 16*VEC*h + VEC*i + tp) of the product.
template <int D>
__device__ __forceinline__ void gemm_acc(floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT],
                                         const float (&a)[Cfg<D>::RB][Cfg<D>::KS],
                                         const float* __restrict__ Zb, int i, int g) {
  using C = Cfg<D>;
  // software pipeline of depth one: the B operand of k-step ks+1 is read from LDS while the RB*NT
  // matrix-core instructions of k-step ks run (every B value feeds all RB row blocks); scheduling
  // barriers keep the compiler from hoisting more reads than that.
  // An LDS instruction carries a 16-bit byte offset.  Rows further than that from the lane's base get
  // a second base register (an opaque offset, so that the compiler does not fold it back into one
  // base plus 32-bit constants, which costs an address register per read).
  constexpr int SEG = 65000 / (C::PITCH * 4) - 1;      // rows reachable from one base
  constexpr int NSEG = (16 * (D / 16 - 1) + 3) / SEG + 1;
  const float* base = Zb + 4 * g * C::PITCH + C::VEC * i;
  const float* segbase[NSEG];
  segbase[0] = base;
#pragma unroll
  for (int sg = 1; sg < NSEG; ++sg) segbase[sg] = base + opaque_int(sg * SEG * C::PITCH);
  float b[2][C::NH][C::VEC];
#pragma unroll
  for (int h = 0; h < C::NH; ++h) lds_ldv<C::VEC>(base + 16 * C::VEC * h, b[0][h]);
  static_for<0, C::KS>([&](auto KS_) {
    constexpr int ks = decltype(KS_)::value;  // = 4q + t, contraction rows 16q + 4g + t
    constexpr int cur = ks & 1, nxt = cur ^ 1;
    if constexpr (ks + 1 < C::KS) {
      constexpr int r1 = 16 * ((ks + 1) / 4) + (ks + 1) % 4;
#pragma unroll
      for (int h = 0; h < C::NH; ++h)
        lds_ldv<C::VEC>(segbase[r1 / SEG] + (r1 % SEG) * C::PITCH + 16 * C::VEC * h, b[nxt][h]);
      TTC_SCHED_BARRIER();  // reads first: a full k-step of matrix-core work hides their latency
    }
#pragma unroll
    for (int h = 0; h < C::NH; ++h)
#pragma unroll
      for (int tp = 0; tp < C::VEC; ++tp)
#pragma unroll
        for (int rb = 0; rb < C::RB; ++rb)
          acc[rb][h * C::VEC + tp] =
              __builtin_amdgcn_mfma_f32_16x16x4f32(a[rb][ks], b[cur][h][tp], acc[rb][h * C::VEC + tp], 0, 0, 0);
    TTC_SCHED_BARRIER();
  });
}

template <int D>
__device__ __forceinline__ int tile_col(int c, int i) {  // column of tile c, lane-in-row i
  using C = Cfg<D>;
  return 16 * C::VEC * (c / C::VEC) + C::VEC * i + (c % C::VEC);
}

template <int D>
__device__ __forceinline__ void zero_acc(floatx4 (&acc)[Cfg<D>::NT]) {
#pragma unroll
  for (int c = 0; c < Cfg<D>::NT; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
}
// rows [16w,16w+16) of the identity in accumulator layout
template <int D>
__device__ __forceinline__ void eye_acc(floatx4 (&acc)[Cfg<D>::NT], int w, int i, int g) {
#pragma unroll
  for (int c = 0; c < Cfg<D>::NT; ++c)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[c][v] = (16 * w + 4 * g + v == tile_col<D>(c, i)) ? 1.f : 0.f;
}
// accumulator rows <-> LDS, untransposed: element (r, col) at Zb[r*PITCH + col]
template <int D>
__device__ __forceinline__ void store_rows(float* Zb, const floatx4 (&acc)[Cfg<D>::NT], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int h = 0; h < C::NH; ++h) {
      float t[C::VEC];
#pragma unroll
      for (int tp = 0; tp < C::VEC; ++tp) t[tp] = acc[h * C::VEC + tp][v];
      lds_stv<C::VEC>(Zb + (16 * w + 4 * g + v) * C::PITCH + 16 * C::VEC * h + C::VEC * i, t);
    }
}
template <int D>
__device__ __forceinline__ void load_rows(const float* Zb, floatx4 (&acc)[Cfg<D>::NT], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int h = 0; h < C::NH; ++h) {
      float t[C::VEC];
      lds_ldv<C::VEC>(Zb + (16 * w + 4 * g + v) * C::PITCH + 16 * C::VEC * h + C::VEC * i, t);
#pragma unroll
      for (int tp = 0; tp < C::VEC; ++tp) acc[h * C::VEC + tp][v] = t[tp];
    }
}
// accumulator rows -> LDS transposed: element (r, col) at Yb[col*PITCH + r]; a lane's four rows
// 16w+4g..+3 are contiguous there
template <int D>
__device__ __forceinline__ void store_rows_T(float* Yb, const floatx4 (&acc)[Cfg<D>::NT], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int c = 0; c < C::NT; ++c)
    *reinterpret_cast<floatx4*>(Yb + tile_col<D>(c, i) * C::PITCH + 16 * w + 4 * g) = acc[c];
}
// A-operand registers of rows [16w,16w+16) of a matrix held in LDS: a[4q+t] = M[16w+i][16q+4g+t]
template <int D>
__device__ __forceinline__ void load_aop_lds(const float* Mb, float (&a)[Cfg<D>::KS], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int q = 0; q < D / 16; ++q) {
    floatx4 t = *reinterpret_cast<const floatx4*>(Mb + (16 * w + i) * C::PITCH + 16 * q + 4 * g);
    a[4 * q + 0] = t[0]; a[4 * q + 1] = t[1]; a[4 * q + 2] = t[2]; a[4 * q + 3] = t[3];
  }
}

// The same helpers for all RB row blocks of wavefront w (row block index RB*w + rb)
#define TTC_FOR_RB for (int rb = 0; rb < Cfg<D>::RB; ++rb)
template <int D>
__device__ __forceinline__ void zero_acc(floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT]) {
#pragma unroll
  TTC_FOR_RB zero_acc<D>(acc[rb]);
}
template <int D>
__device__ __forceinline__ void eye_acc(floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT], int w, int i, int g) {
#pragma unroll
  TTC_FOR_RB eye_acc<D>(acc[rb], Cfg<D>::RB * w + rb, i, g);
}
template <int D>
__device__ __forceinline__ void store_rows(float* Zb, const floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT], int w, int i, int g) {
#pragma unroll
  TTC_FOR_RB store_rows<D>(Zb, acc[rb], Cfg<D>::RB * w + rb, i, g);
}
template <int D>
__device__ __forceinline__ void load_rows(const float* Zb, floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT], int w, int i, int g) {
#pragma unroll
  TTC_FOR_RB load_rows<D>(Zb, acc[rb], Cfg<D>::RB * w + rb, i, g);
}
template <int D>
__device__ __forceinline__ void store_rows_T(float* Yb, const floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT], int w, int i, int g) {
#pragma unroll
  TTC_FOR_RB store_rows_T<D>(Yb, acc[rb], Cfg<D>::RB * w + rb, i, g);
}
template <int D>
__device__ __forceinline__ void load_aop_lds(const float* Mb, float (&a)[Cfg<D>::RB][Cfg<D>::KS], int w, int i, int g) {
#pragma unroll
  TTC_FOR_RB load_aop_lds<D>(Mb, a[rb], Cfg<D>::RB * w + rb, i, g);
}

// max |.| over the wavefront's accumulator rows (wave-uniform; NaN counts as larger than every number)
template <int D>
__device__ __forceinline__ float wave_absmax(const floatx4 (&acc)[Cfg<D>::RB][Cfg<D>::NT]) {
  uint32_t m = 0;  // |x| as bits: for non-negative floats the unsigned order is the numeric one, NaN on top
#pragma unroll
  for (int rb = 0; rb < Cfg<D>::RB; ++rb)
#pragma unroll
    for (int c = 0; c < Cfg<D>::NT; ++c)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const uint32_t b = __float_as_uint(acc[rb][c][v]) & 0x7FFFFFFFu;
        m = b > m ? b : m;
      }
  return __uint_as_float(wave_max_u32(m));
}

// A-operand registers of the wavefront's rows of M^T, M held in LDS: a[4q+t] = M[16q+4g+t][row]
template <int D>
__device__ __forceinline__ void load_aopT_lds(const float* Mb, float (&a)[Cfg<D>::RB][Cfg<D>::KS], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int k = 0; k < C::KS; ++k)
      a[rb][k] = Mb[(16 * (k / 4) + 4 * g + (k % 4)) * C::PITCH + 16 * (C::RB * w + rb) + i];
}

// the inverse of load_aop_lds: A-operand registers of the wavefront's rows -> row-major matrix in LDS
template <int D>
__device__ __forceinline__ void store_aop_lds(float* Mb, const float (&a)[Cfg<D>::RB][Cfg<D>::KS], int w, int i, int g) {
  using C = Cfg<D>;
#pragma unroll
  for (int rb = 0; rb < C::RB; ++rb)
#pragma unroll
    for (int q = 0; q < D / 16; ++q) {
      floatx4 t;
      t[0] = a[rb][4 * q + 0]; t[1] = a[rb][4 * q + 1]; t[2] = a[rb][4 * q + 2]; t[3] = a[rb][4 * q + 3];
      *reinterpret_cast<floatx4*>(Mb + (16 * (C::RB * w + rb) + i) * C::PITCH + 16 * q + 4 * g) = t;
    }
}

// ----------------------------------------------------------------------------------------------
// Dense solve M X = RHS inside LDS: blocked Gauss-Jordan elimination with partial (row) pivoting on
// the augmented d x 2d array W = [M | RHS] (row r at W + r*PITCH; M = columns [0,d), RHS = [d,2d)),
// 16 columns per panel.  Rows are never moved: the pivot row of column c is remembered in S.piv[c]
// (implicit pivoting) and the solution, X[c][:] = RHS[S.piv[c]][:] / pivot_c, is put in order by the last panel's
// update as it writes its rows.
//
// Per panel P = [16p, 16p+16):
//   (a) wavefront 0 holds the d x 16 panel in registers (a lane owns rows lane, lane+64) and runs
//       unblocked Gauss-Jordan on it: pivot = max |.| over rows never used as a pivot (one DPP max
//       of a packed key), pivot row broadcast with v_readlane, every other row -- pivoted earlier or
//       not -- gets its multiplier and is updated.  It leaves in W[:, P] the multiplier matrix Lm
//       (for the j-th pivot row of the panel: its multipliers against the earlier pivot rows of the
//       panel, zero in column j, the later "Jordan" multipliers after it) and in S.L11 a copy of
//       the unit-lower multipliers among the 16 pivot rows.
//   (b) U12 = Lf^{-1} P for the 16 pivot rows P of the remaining columns, Lf the unit-lower factor among
//       the pivot rows (S.L11): wavefront 0 inverts Lf right after factoring the panel (S.Linv), and every
//       wavefront forms U12 tile by tile on the matrix cores; negated, it stays in registers as an operand of (c).
//   (c) W[:, rest] -= Lm * U12 on the matrix cores, all d rows, in 16 x 16 tiles (a pivot row holds
//       P_j = U12_j + sum_{k<j} L_jk U12_k, so the same update serves it); the product is
//       formed transposed (MFMA M index = column, N index = row) so that a lane's four accumulator
//       values, and its four operand values of either side, are 16 contiguous bytes of LDS.
// Schedule.  A single wavefront issues about one instruction every five cycles whatever its kind, and a
// column of (a) is a chain of some 300 cycles (six DPP steps, broadcasts, a reciprocal), so (a) is the
// critical path: the next panel's columns are updated first, by all wavefronts together (each its own
// row tiles), then wavefront 0 factors panel p+1 while the others share the remaining column tiles of
// panel p, each software-pipelined over its tiles: three workgroup barriers per panel.
// Returns nonzero (uniformly) if a pivot was zero or not finite.  All threads must call it; W must be
// visible on entry (caller synchronised); the result is visible to every thread on return.
template <int D>
struct SolveScratch {
  float L11[16 * 16];      // unit-lower factor among the panel's pivot rows (the factoring wavefront's own)
  float Linv[2][16 * 16];  // its inverse; double-buffered: panel p+1 is factored while p's is still read
  float rinv[D];  // 1 / pivot, by pivot row
  int piv[D];     // pivot row of column c
  int ipiv[D];    // column whose pivot row r is
  int flag;
};

// signed max over the 64 lanes of keys that are either non-negative or to be ignored (negative), wave-uniform
__device__ __forceinline__ int wave_max_nonneg_i32(int x) {
  auto mx = [](int a, int b) { return a > b ? a : b; };
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false));  // row_half_mirror
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, false));  // row_mirror
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false));  // row_bcast15 into rows 1 and 3
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false));  // row_bcast31 into rows 2 and 3
  return __builtin_amdgcn_readlane(x, 63);
}

// (a) Gauss-Jordan on the d x 16 panel at column cb by one wavefront, rows in registers (a lane owns rows lane
// and lane + 64).  A lone wavefront is bound by the number of instructions it issues, so a column costs as few
// as possible: the pivot search is one signed DPP max of the key (|value| bits above 7 | atag), atag = 127 - row
// while the row has not been a pivot and the sign bit afterwards (such a key loses against every live row);
// the pivot row is broadcast with v_readlane from the half of the rows it lies in (a uniform branch: the code
// of a column exists once per half, and only the pivot's half pays for the masks that exempt the pivot row).
template <int D, bool PIVOT>
__device__ __forceinline__ void solve_panel(float* W, SolveScratch<D>& S, int cb, int lane,
                                             int (&atag)[(D + 63) / 64], int& bad) {
  using C = Cfg<D>;
  constexpr int NRL = (D + 63) / 64;
  float a[NRL][16];
  int myj[NRL];
#pragma unroll
  for (int rr = 0; rr < NRL; ++rr) {
    const int r = lane + 64 * rr;
    myj[rr] = 16;  // 16 = not a pivot row of this panel
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      floatx4 t = floatx4{0.f, 0.f, 0.f, 0.f};
      if (r < D) t = *reinterpret_cast<const floatx4*>(W + r * C::PITCH + cb + 4 * q);
      a[rr][4 * q + 0] = t[0]; a[rr][4 * q + 1] = t[1]; a[rr][4 * q + 2] = t[2]; a[rr][4 * q + 3] = t[3];
    }
  }
  int lane_piv = 0;     // lane j: pivot row of column cb + j
  float lane_pv = 1.f;  // lane j: its pivot value
  // pivot row of column cb + j: the live row with the largest |value| (ties and zeros: the lowest row)
  auto search = [&](auto JC) {
    constexpr int j = decltype(JC)::value;
    if constexpr (PIVOT) {
      int key = (int)(__float_as_uint(a[0][j]) & 0x7FFFFF80u) | atag[0];
      if constexpr (NRL > 1) {
        const int k1 = (int)(__float_as_uint(a[1][j]) & 0x7FFFFF80u) | atag[1];
        key = k1 > key ? k1 : key;
      }
      key = wave_max_nonneg_i32(key);
      const int pr = 127 - (key & 0x7F);
      return pr < D ? pr : D - 1;  // never leave the array, whatever the data
    } else {
      return cb + j;
    }
  };
  int pr = search(IntC<0>{});
  static_for<0, 16>([&](auto J) {
    constexpr int j = decltype(J)::value;
    const int pl = pr & 63;
    // one column step with the pivot row in half PH of the rows; it ends with the search of the next column,
    // which only needs that column updated and can therefore run beside the other columns' updates
    auto step = [&](auto PHC) {
      constexpr int PH = decltype(PHC)::value;
      float prow[16];
      static_for<j, 16>([&](auto JJ) {
        constexpr int jj = decltype(JJ)::value;
        prow[jj] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a[PH][jj]), pl));
      });
      const float inv = __builtin_amdgcn_rcpf(prow[j]);
      asm("v_writelane_b32 %0, %1, %2" : "+v"(lane_piv) : "s"(pr), "n"(j));
      asm("v_writelane_b32 %0, %1, %2" : "+v"(lane_pv) : "s"(prow[j]), "n"(j));
      const bool hot = (lane == pl);  // in half PH, this lane's row is the pivot row
      float l[NRL];
#pragma unroll
      for (int rr = 0; rr < NRL; ++rr) {
        if (rr == PH) {
          l[rr] = (hot ? 0.f : a[rr][j]) * inv;  // the pivot row itself is not updated
          atag[rr] = hot ? (int)0x80000000 : atag[rr];
          myj[rr] = hot ? j : myj[rr];
        } else {
          l[rr] = a[rr][j] * inv;
        }
        a[rr][j] = l[rr];
        if constexpr (j + 1 < 16) a[rr][j + 1] = __builtin_fmaf(-l[rr], prow[j + 1], a[rr][j + 1]);
      }
      int next = 0;
      if constexpr (j + 1 < 16) next = search(IntC<j + 1>{});
#pragma unroll
      for (int rr = 0; rr < NRL; ++rr) {
        static_for<j + 2, 16>([&](auto JJ) {
          constexpr int jj = decltype(JJ)::value;
          a[rr][jj] = __builtin_fmaf(-l[rr], prow[jj], a[rr][jj]);
        });
        // the column's updates end here, inside their branch: otherwise the compiler moves them behind the point
        // where the two branches meet and copies the broadcast row into vector registers to get them there
#pragma unroll
        for (int jj = j; jj < 16; ++jj) asm volatile("" : "+v"(a[rr][jj]));
      }
      return next;
    };
    if constexpr (NRL > 1) {
      if (pr >= 64) pr = step(IntC<NRL - 1>{});
      else pr = step(IntC<0>{});
    } else {
      pr = step(IntC<0>{});
    }
  });
  if (lane < 16) {
    const float apv = PIVOT ? fabsf(lane_pv) : lane_pv;
    S.piv[cb + lane] = lane_piv;
    S.ipiv[lane_piv] = cb + lane;
    S.rinv[lane_piv] = __builtin_amdgcn_rcpf(lane_pv);
    if (!(apv > 0.f && apv < __builtin_inff())) bad = 1;
  }
  bad = __any(bad) ? 1 : 0;
  float* L11 = S.L11;
#pragma unroll
  for (int rr = 0; rr < NRL; ++rr) {
    const int r = lane + 64 * rr;
    if (r < D) {
      const int j0 = myj[rr];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        floatx4 t;
        t[0] = a[rr][4 * q + 0]; t[1] = a[rr][4 * q + 1]; t[2] = a[rr][4 * q + 2]; t[3] = a[rr][4 * q + 3];
        // row j0 of the unit-lower factor: only its entries left of the diagonal are read back
        if (j0 < 16) *reinterpret_cast<floatx4*>(L11 + j0 * 16 + 4 * q) = t;
        *reinterpret_cast<floatx4*>(W + r * C::PITCH + cb + 4 * q) = t;
      }
    }
  }
}

// Inverse of the panel's unit-lower factor Lf (rows of multipliers in S.L11), by the wavefront that factored the
// panel, into S.Linv, from where every wavefront reads its matrix-core A operand of U12 = Lf^{-1} P (the lane
// (i, g) takes Linv[i][4g .. 4g+3]).  Lane i of every row of 16 lanes holds row i of Lf
// (its own registers, read from LDS without broadcasts) and builds row i of the inverse by forward substitution
// over the pivots k: Linv[i][:] -= Lf[i][k] Linv[k][:], with row k of the inverse taken from lane k by a DPP row
// broadcast (the four rows of lanes do the same work).
template <int D>
__device__ __forceinline__ void panel_linv(SolveScratch<D>& S, int cb, int lane) {
  const float* L11 = S.L11;  // written by this wavefront just now (LDS serves a wavefront's operations in order)
  const int i = lane & 15, g = lane >> 4;
  float l[16], x[16];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const floatx4 t = *reinterpret_cast<const floatx4*>(L11 + i * 16 + 4 * q);
#pragma unroll
    for (int e = 0; e < 4; ++e) l[4 * q + e] = (4 * q + e < i) ? -t[e] : 0.f;  // strictly lower part only, negated
  }
#pragma unroll
  for (int c = 0; c < 16; ++c) x[c] = (c == i) ? 1.f : 0.f;
  // x[c] += l[k] * (x[c] of lane k), c = 0..k, for k = 0..14: the broadcast rides on the multiply-add as its DPP
  // operand.  One block per k, so that the wait states a DPP read needs after a vector write of the same
  // register are in our hands: within a block every instruction touches its own register, and each block
  // starts and ends with the two idle states.
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %1 row_newbcast:0 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0])
      : "v"(l[0]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %2 row_newbcast:1 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %2 row_newbcast:1 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1])
      : "v"(l[1]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %3 row_newbcast:2 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %3 row_newbcast:2 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %3 row_newbcast:2 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2])
      : "v"(l[2]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %4 row_newbcast:3 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %4 row_newbcast:3 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %4 row_newbcast:3 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %4 row_newbcast:3 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3])
      : "v"(l[3]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %5 row_newbcast:4 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %5 row_newbcast:4 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %5 row_newbcast:4 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %5 row_newbcast:4 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %5 row_newbcast:4 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4])
      : "v"(l[4]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %6 row_newbcast:5 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %6 row_newbcast:5 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %6 row_newbcast:5 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %6 row_newbcast:5 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %6 row_newbcast:5 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %6 row_newbcast:5 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5])
      : "v"(l[5]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %7 row_newbcast:6 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %7 row_newbcast:6 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %7 row_newbcast:6 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %7 row_newbcast:6 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %7 row_newbcast:6 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %7 row_newbcast:6 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %7 row_newbcast:6 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6])
      : "v"(l[6]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %8 row_newbcast:7 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
      : "v"(l[7]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %8, %8, %9 row_newbcast:8 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+v"(x[8])
      : "v"(l[8]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %8, %8, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %9, %9, %10 row_newbcast:9 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+v"(x[8]), "+v"(x[9])
      : "v"(l[9]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %8, %8, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %9, %9, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %10, %10, %11 row_newbcast:10 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+v"(x[8]), "+v"(x[9]), "+v"(x[10])
      : "v"(l[10]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %8, %8, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %9, %9, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %10, %10, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %11, %11, %12 row_newbcast:11 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11])
      : "v"(l[11]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %8, %8, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %9, %9, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %10, %10, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %11, %11, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %12, %12, %13 row_newbcast:12 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12])
      : "v"(l[12]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %8, %8, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %9, %9, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %10, %10, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %11, %11, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %12, %12, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %13, %13, %14 row_newbcast:13 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13])
      : "v"(l[13]));
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %0, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %1, %1, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %2, %2, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %3, %3, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %4, %4, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %5, %5, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %6, %6, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %7, %7, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %8, %8, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %9, %9, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %10, %10, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %11, %11, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %12, %12, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %13, %13, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "v_fmac_f32_dpp %14, %14, %15 row_newbcast:14 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13]), "+v"(x[14])
      : "v"(l[14]));
  // the first row of lanes writes the inverse, row i by lane i (picking a lane's own quarter of its row out of
  // x[] would be an indexed access to a register array, which the compiler serves from scratch memory)
  if (g == 0) {
    float* dst = S.Linv[(cb >> 4) & 1] + i * 16;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<floatx4*>(dst + 4 * q) = floatx4{x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]};
  }
}

// (b) + (c) for the column tiles [lo, hi) of the rest of panel cb (tile t = columns [cb+16+16t, +16)), all row
// tiles, by one wavefront, software-pipelined: while the matrix cores update tile t, the rows of tile t+1 and
// its pivot rows are read and tile t-1 has been written.
// FINAL (the last panel, whose remaining columns are exactly the right-hand sides): the updated rows are the
// solution up to order and scale, row r being pivot^{-1} times row ipiv[r] of X; they are written there directly.
// Within a column tile every row has been read before the first is written, and no other wavefront touches
// the tile, so the permutation needs no second buffer.
template <int D, bool FINAL = false>
__device__ __forceinline__ void solve_update(float* W, SolveScratch<D>& S, int cb, int lane, int lo, int hi, floatx4 la) {
  using C = Cfg<D>;
  if (lo >= hi) return;
  const int i = lane & 15, g = lane >> 4;
  float* const rowp = W + i * C::PITCH + cb;  // row i of a row tile, at the panel's first column
  float* dst[C::NRT];                         // where row i of each row tile goes, at the panel's first column
  float scl[C::NRT];
#pragma unroll
  for (int rt = 0; rt < C::NRT; ++rt) {
    dst[rt] = rowp + 16 * rt * C::PITCH;
    scl[rt] = 1.f;
    if constexpr (FINAL) {
      dst[rt] = W + S.ipiv[16 * rt + i] * C::PITCH + cb;
      scl[rt] = S.rinv[16 * rt + i];
    }
  }
  floatx4 bl[C::NRT];                         // Lm[row i of the row tile][4g .. 4g+3]: the same for every column tile
#pragma unroll
  for (int rt = 0; rt < C::NRT; ++rt) bl[rt] = *reinterpret_cast<const floatx4*>(rowp + 16 * rt * C::PITCH + 4 * g);
  int pv[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) pv[t] = S.piv[cb + 4 * g + t] * C::PITCH + cb + 16 + i;
  floatx4 acc[2][C::NRT];
  float pb[2][4];
  auto issue = [&](int buf, int ct) {
#pragma unroll
    for (int t = 0; t < 4; ++t) pb[buf][t] = W[pv[t] + 16 * ct];
#pragma unroll
    for (int rt = 0; rt < C::NRT; ++rt)
      acc[buf][rt] = *reinterpret_cast<const floatx4*>(rowp + 16 * rt * C::PITCH + 16 + 16 * ct + 4 * g);
  };
  auto u12 = [&](int buf) {
    floatx4 av = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) av = __builtin_amdgcn_mfma_f32_16x16x4f32(la[t], pb[buf][t], av, 0, 0, 0);
    return -av;
  };
  issue(0, lo);
  floatx4 av = u12(0);
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the loop starts with nothing in flight
  for (int ct = lo; ct < hi; ct += 2) {
    // even step: tile ct in buffer 0, prefetch ct+1 into buffer 1
    const bool more1 = ct + 1 < hi;
    // The tile's reads have arrived: waited for here, by hand, because the compiler, which cannot count the
    // LDS operations in flight around the loop, would otherwise wait for all of them after the next tile's reads
    // have been issued, that is for the very reads the matrix-core work below is meant to hide.  LDS operations
    // complete in order, and the only ones issued after the tile's reads are the NRT writes of the tile before
    // it, which need not be waited for.
    __builtin_amdgcn_s_waitcnt(0xC07F | (C::NRT << 8));  // lgkmcnt(NRT)
    if (more1) issue(1, ct + 1);
    TTC_SCHED_BARRIER();
#pragma unroll
    for (int rt = 0; rt < C::NRT; ++rt)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc[0][rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[kk], bl[rt][kk], acc[0][rt], 0, 0, 0);
    floatx4 av1 = floatx4{0.f, 0.f, 0.f, 0.f};
    if (more1) av1 = u12(1);  // a chain of dependent matrix-core instructions runs at the full rate
    TTC_SCHED_BARRIER();
#pragma unroll
    for (int rt = 0; rt < C::NRT; ++rt)
      *reinterpret_cast<floatx4*>(dst[rt] + 16 + 16 * ct + 4 * g) = FINAL ? acc[0][rt] * scl[rt] : acc[0][rt];
    if (!more1) break;
    const bool more2 = ct + 2 < hi;
    __builtin_amdgcn_s_waitcnt(0xC07F | (C::NRT << 8));  // lgkmcnt(NRT), as above
    if (more2) issue(0, ct + 2);
    TTC_SCHED_BARRIER();
#pragma unroll
    for (int rt = 0; rt < C::NRT; ++rt)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc[1][rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av1[kk], bl[rt][kk], acc[1][rt], 0, 0, 0);
    if (more2) av = u12(0);
    TTC_SCHED_BARRIER();
#pragma unroll
    for (int rt = 0; rt < C::NRT; ++rt)
      *reinterpret_cast<floatx4*>(dst[rt] + 16 + 16 * (ct + 1) + 4 * g) = FINAL ? acc[1][rt] * scl[rt] : acc[1][rt];
  }
}

// The next panel's columns (column tile 0 of the rest of panel cb), which the next panel's factorisation waits
// for, shared by all wavefronts: every wavefront forms the tile's U12 (b), then, after a barrier (the pivot rows
// read by (b) are rows that (c) rewrites), updates its own RT0 row tiles (c).
template <int D>
__device__ __forceinline__ void solve_update_first(float* W, SolveScratch<D>& S, int cb, int lane, int w, floatx4 la) {
  using C = Cfg<D>;
  constexpr int RT0 = C::NRT / C::NW;  // row tiles per wavefront
  const int i = lane & 15, g = lane >> 4;
  float* const rowp = W + i * C::PITCH + cb;
  floatx4 bl[RT0], acc[RT0];
  float pb[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) pb[t] = W[S.piv[cb + 4 * g + t] * C::PITCH + cb + 16 + i];
#pragma unroll
  for (int r = 0; r < RT0; ++r) {
    const int rt = RT0 * w + r;
    bl[r] = *reinterpret_cast<const floatx4*>(rowp + 16 * rt * C::PITCH + 4 * g);
    acc[r] = *reinterpret_cast<const floatx4*>(rowp + 16 * rt * C::PITCH + 16 + 4 * g);
  }
  floatx4 av = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 4; ++t) av = __builtin_amdgcn_mfma_f32_16x16x4f32(la[t], pb[t], av, 0, 0, 0);
  av = -av;
#pragma unroll
  for (int r = 0; r < RT0; ++r)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) acc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[kk], bl[r][kk], acc[r], 0, 0, 0);
  __syncthreads();  // every wavefront has read the tile's pivot rows
#pragma unroll
  for (int r = 0; r < RT0; ++r)
    *reinterpret_cast<floatx4*>(rowp + 16 * (RT0 * w + r) * C::PITCH + 16 + 4 * g) = acc[r];
}

// PARTS is kept for the callers' template argument lists (always 7).
template <int D, int PARTS = 7, bool PIVOT = true>
__device__ __forceinline__ int lds_solve(float* W, SolveScratch<D>& S, int tid) {
  using C = Cfg<D>;
  constexpr int NP = D / 16;
  constexpr int NRL = (D + 63) / 64;
  tid += opaque_zero();
  const int lane = tid & 63, w = tid >> 6;
  int atag[NRL];
#pragma unroll
  for (int rr = 0; rr < NRL; ++rr) atag[rr] = (lane + 64 * rr) < D ? 127 - (lane + 64 * rr) : (int)0x80000000;
  int bad = 0;
  if (w == 0) {
    solve_panel<D, PIVOT>(W, S, 0, lane, atag, bad);
    panel_linv<D>(S, 0, lane);
  }
  for (int p = 0; p < NP; ++p) {
    __syncthreads();  // panel p is in place; every update of panel p-1 is done
    const int cb = 16 * p;
    const int nct = (2 * D - cb - 16) / 16;  // column tiles to the right of the panel
    const bool more = (p + 1 < NP);
    const floatx4 la = *reinterpret_cast<const floatx4*>(S.Linv[p & 1] + (lane & 15) * 16 + 4 * (lane >> 4));
    if (more && C::NW > 1) {
      solve_update_first<D>(W, S, cb, lane, w, la);
      __syncthreads();  // the next panel's columns are up to date
      if (w == 0) {
        solve_panel<D, PIVOT>(W, S, cb + 16, lane, atag, bad);
        panel_linv<D>(S, cb + 16, lane);
      } else {
        // a contiguous share of the other column tiles each; which wavefront gets the larger share rotates
        const int ntile = nct - 1, u = (w - 1 + p) % (C::NW - 1);
        solve_update<D>(W, S, cb, lane, 1 + (u * ntile) / (C::NW - 1), 1 + ((u + 1) * ntile) / (C::NW - 1), la);
      }
    } else if (more) {  // one wavefront: everything in turn
      solve_update<D>(W, S, cb, lane, 0, nct, la);
      solve_panel<D, PIVOT>(W, S, cb + 16, lane, atag, bad);
      panel_linv<D>(S, cb + 16, lane);
    } else {
      solve_update<D, true>(W, S, cb, lane, (w * nct) / C::NW, ((w + 1) * nct) / C::NW, la);
    }
  }
  if (tid == 0) S.flag = bad;
  __syncthreads();
  const int flag = S.flag;
  __syncthreads();
  return flag;
}


// Row normalisation of [Y1 Y2] (App. C "Numerical Stability") in Z-land: column c of Z is row c of
// the pair.  The scale is the power of two just below max(||Y1_c||_1, ||Y2_c||_1), so the scaling
// is exact and Y1^{-1} Y2 is unchanged bit for bit (barring under/overflow).
template <int D>
__device__ void normalise_rows_zland(float* W, int tid) {
  using C = Cfg<D>;
  constexpr int TPC = C::NTHR / D;           // threads per column (a power of two, 2 or 4)
  const int c = tid / TPC, part = tid % TPC;
  float s1 = 0.f, s2 = 0.f;
  for (int r = part; r < D; r += TPC) {
    s1 += fabsf(W[r * C::PITCH + c]);
    s2 += fabsf(W[r * C::PITCH + D + c]);
  }
#pragma unroll
  for (int m = 1; m < TPC; m <<= 1) {
    s1 += __shfl_xor(s1, m, 64);
    s2 += __shfl_xor(s2, m, 64);
  }
  const float mx = fmaxf(s1, s2);
  float scale = 1.0f;
  if (mx > 0.f && mx < __builtin_inff()) {
    int e;
    frexpf(mx, &e);              // mx = f * 2^e, f in [0.5, 1)
    scale = ldexpf(1.0f, -e);    // exact power of two
  }
  for (int r = part; r < D; r += TPC) {
    W[r * C::PITCH + c] *= scale;
    W[r * C::PITCH + D + c] *= scale;
  }
}

}  // namespace ttc
