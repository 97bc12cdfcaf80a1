// Kernels of the whole Test-Time Control block around the structured solver (Sec. 4, "Hybrid with Memory Layers",
// "Multi-Head Structure", "Contextualization", "Parameterization"):
//     h_0   = W_in LN(x_in) + b_in                     ln_stats_kernel + gemm_ln_kernel
//     the per-head contextualisation maps s_X(h_0)      cxt_maps_kernel (+ qbasis_kernel: Q^(i) = Qc Qc^T / sqrt(d))
//     o     = u_1^* of every head's problem             solve_cxt_kernel (ttc_cxt.hpp), fed from the arrays above
//     x_out = x_in + W_out LN(o) + b_out                ln_stats_kernel + gemm_ln_kernel with the residual
// The two projections are dense contractions and run on the matrix cores in float32 (v_mfma_f32_16x16x4_f32), the
// layer normalisation applied to the operand on its way from global memory into LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ttc_args.hpp"

namespace ttc {

typedef float blk_floatx4 __attribute__((ext_vector_type(4)));

// mean and reciprocal standard deviation of every row (float32 or bfloat16), one wavefront per row, two passes over
// the row (the second one reads what the first has just brought into the caches): no cancellation whatever the mean
typedef unsigned short blk_u16x4 __attribute__((ext_vector_type(4)));
typedef unsigned short blk_u16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 blk_bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_to_f32(unsigned short v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ unsigned short f32_to_bf16(float x) {  // round to nearest, ties to even (the hardware conversion)
  return __builtin_bit_cast(unsigned short, static_cast<__bf16>(x));
}
// four consecutive elements of a float32 or bfloat16 row, widened
template <typename T>
__device__ __forceinline__ blk_floatx4 blk_ld4(const T* p, long long i);
template <>
__device__ __forceinline__ blk_floatx4 blk_ld4<float>(const float* p, long long i) {
  return *reinterpret_cast<const blk_floatx4*>(p + i);
}
template <>
__device__ __forceinline__ blk_floatx4 blk_ld4<unsigned short>(const unsigned short* p, long long i) {
  const blk_u16x4 v = *reinterpret_cast<const blk_u16x4*>(p + i);
  return blk_floatx4{bf16_to_f32(v[0]), bf16_to_f32(v[1]), bf16_to_f32(v[2]), bf16_to_f32(v[3])};
}

template <typename TX>
__global__ void __launch_bounds__(256) ln_stats_kernel(const LnStatsArgs p) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= p.M) return;
  const TX* x = reinterpret_cast<const TX*>(p.X) + row * p.L;
  float s = 0.f;
  for (int k = 4 * lane; k < p.L; k += 256) {
    const blk_floatx4 v = blk_ld4<TX>(x, k);
    s += (v[0] + v[1]) + (v[2] + v[3]);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) s += __shfl_xor(s, o, 64);
  const float mean = s / (float)p.L;
  float q = 0.f;
  for (int k = 4 * lane; k < p.L; k += 256) {
    const blk_floatx4 v = blk_ld4<TX>(x, k);
    const float a = v[0] - mean, b = v[1] - mean, c = v[2] - mean, d = v[3] - mean;
    q += (a * a + b * b) + (c * c + d * d);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) q += __shfl_xor(q, o, 64);
  if (lane == 0) {
    p.stats[2 * row] = mean;
    p.stats[2 * row + 1] = 1.f / sqrtf(q / (float)p.L + p.eps);
  }
}

// Y = LN(X) W^T + bias (+ Res).  A workgroup of four wavefronts owns a tile of 128 rows of X by 128 rows of W and
// walks K in slices of 32: the two slices go through registers (where the rows of X are normalised) into LDS, double
// buffered, one barrier per slice.  A wavefront forms 64 x 64 of the tile as 4 x 4 matrix-core tiles with W on the
// row side, so that a lane ends up with four consecutive outputs of one row of Y.  The lanes of a k-group read four
// consecutive k (one 16-byte LDS read feeds four instructions); both operands use the same order of the
// contraction index, which is all that matters.  Row pitch 36 floats: the sixteen lanes of a k-group hit all banks.
constexpr int GEMM_BM = 128, GEMM_BN = 128, GEMM_BK = 32, GEMM_PITCH = GEMM_BK + 4;

__global__ void __launch_bounds__(256) gemm_ln_kernel(const GemmLnArgs p) {
  __shared__ __attribute__((aligned(16))) float lds[2 * (GEMM_BM + GEMM_BN) * GEMM_PITCH];
  auto Ws = [&](int buf) { return lds + buf * (GEMM_BM + GEMM_BN) * GEMM_PITCH; };  // the slice of W, then that of X
  auto Xs = [&](int buf) { return lds + buf * (GEMM_BM + GEMM_BN) * GEMM_PITCH + GEMM_BN * GEMM_PITCH; };
  const long long nMt = (p.M + GEMM_BM - 1) / GEMM_BM;
  const int nNt = (p.N + GEMM_BN - 1) / GEMM_BN;
  const long long total = nMt * nNt;
  // workgroups are dealt to the eight dies round-robin; give each die a contiguous run of tiles, so that the tiles
  // that share rows of X (consecutive ones) meet in one die's L2
  const long long per = (total + 7) / 8;
  const long long tile = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((long long)(blockIdx.x >> 3) >= per || tile >= total) return;
  const long long m0 = (tile / nNt) * GEMM_BM;
  const int n0 = (int)(tile % nNt) * GEMM_BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i = lane & 15, g = lane >> 4;
  const int wo = wave & 1, wn = wave >> 1;  // the wavefront's 64 outputs and 64 rows within the tile
  const int lr = tid >> 3, lc = 4 * (tid & 7);  // this thread's rows lr + 32 j and columns lc .. lc + 3 of a slice

  float mean[4], rstd[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const long long row = m0 + lr + 32 * j;
    mean[j] = row < p.M ? p.stats[2 * row] : 0.f;
    rstd[j] = row < p.M ? p.stats[2 * row + 1] : 0.f;
  }
  // a slice on its way: fetch() only issues the global reads, stash() normalises the rows of X and writes both slices
  // to LDS; the matrix-core work on the slice before sits between the two, so the reads' latency is covered
  blk_floatx4 rw[4], rx[4], gn, of;
  bool live[4];
  auto fetch = [&](int k0) {
    const int k = k0 + lc;
    gn = blk_floatx4{0.f, 0.f, 0.f, 0.f};
    of = blk_floatx4{0.f, 0.f, 0.f, 0.f};
    if (k < p.K) {
      gn = *reinterpret_cast<const blk_floatx4*>(p.gain + k);
      of = *reinterpret_cast<const blk_floatx4*>(p.offset + k);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int o = n0 + lr + 32 * j;
      const long long row = m0 + lr + 32 * j;
      rw[j] = blk_floatx4{0.f, 0.f, 0.f, 0.f};
      rx[j] = blk_floatx4{0.f, 0.f, 0.f, 0.f};
      live[j] = k < p.K && row < p.M;
      if (k < p.K && o < p.N) rw[j] = *reinterpret_cast<const blk_floatx4*>(p.W + (long long)o * p.K + k);
      if (live[j]) rx[j] = *reinterpret_cast<const blk_floatx4*>(p.X + row * p.K + k);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      blk_floatx4 v = {0.f, 0.f, 0.f, 0.f};
      if (live[j]) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (rx[j][e] - mean[j]) * rstd[j] * gn[e] + of[e];
      }
      *reinterpret_cast<blk_floatx4*>(Ws(buf) + (lr + 32 * j) * GEMM_PITCH + lc) = rw[j];
      *reinterpret_cast<blk_floatx4*>(Xs(buf) + (lr + 32 * j) * GEMM_PITCH + lc) = v;
    }
  };

  blk_floatx4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = blk_floatx4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int buf) {
    const float* wsb = Ws(buf) + (64 * wo + i) * GEMM_PITCH + 4 * g;
    const float* xsb = Xs(buf) + (64 * wn + i) * GEMM_PITCH + 4 * g;
#pragma unroll
    for (int h = 0; h < GEMM_BK / 16; ++h) {
      blk_floatx4 a[4], b[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        a[t] = *reinterpret_cast<const blk_floatx4*>(wsb + 16 * t * GEMM_PITCH + 16 * h);
        b[t] = *reinterpret_cast<const blk_floatx4*>(xsb + 16 * t * GEMM_PITCH + 16 * h);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int ob = 0; ob < 4; ++ob)
#pragma unroll
          for (int nb = 0; nb < 4; ++nb)
            acc[ob][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ob][e], b[nb][e], acc[ob][nb], 0, 0, 0);
    }
  };
  const int nk = (p.K + GEMM_BK - 1) / GEMM_BK;
  fetch(0);
  stash(0);
  __syncthreads();
  for (int kt = 0; kt + 1 < nk; ++kt) {
    fetch((kt + 1) * GEMM_BK);
    compute(kt & 1);
    stash((kt & 1) ^ 1);
    __syncthreads();
  }
  // the last slice has nothing to fetch: the residual is read under its matrix-core work instead
  blk_floatx4 res[4][4];
#pragma unroll
  for (int ob = 0; ob < 4; ++ob)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int o = n0 + 64 * wo + 16 * ob + 4 * g;
      const long long row = m0 + 64 * wn + 16 * nb + i;
      res[ob][nb] = blk_floatx4{0.f, 0.f, 0.f, 0.f};
      if (p.Res && o < p.N && row < p.M) res[ob][nb] = *reinterpret_cast<const blk_floatx4*>(p.Res + row * p.N + o);
    }
  compute((nk - 1) & 1);

  // acc[ob][nb][v] = Y[m0 + 64 wn + 16 nb + i][n0 + 64 wo + 16 ob + 4 g + v]
#pragma unroll
  for (int ob = 0; ob < 4; ++ob) {
    const int o = n0 + 64 * wo + 16 * ob + 4 * g;
    if (o >= p.N) continue;
    blk_floatx4 bs = {0.f, 0.f, 0.f, 0.f};
    if (p.bias) bs = *reinterpret_cast<const blk_floatx4*>(p.bias + o);
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const long long row = m0 + 64 * wn + 16 * nb + i;
      if (row >= p.M) continue;
      blk_floatx4 y = acc[ob][nb] + bs;
      y += res[ob][nb];
      *reinterpret_cast<blk_floatx4*>(p.Y + row * p.N + o) = y;
    }
  }
}

// The same projection with bfloat16 operands on the matrix cores (v_mfma_f32_16x16x32_bf16, float32 accumulation),
// for blocks whose token features and projection weights are stored in bfloat16: X float32 or bfloat16 (normalised in
// float32, then rounded to bfloat16), W bfloat16, the result float32 or bfloat16, the residual bfloat16.  Same tiling as
// gemm_ln_kernel with slices of 64: a lane reads eight consecutive k of a row (16 bytes) per instruction, rows 72
// bfloat16 apart in LDS (the sixteen lanes of a k-group hit all banks).
constexpr int GEMMB_BK = 64, GEMMB_PITCH = GEMMB_BK + 8;

template <typename TX, bool OUT_BF16>
__global__ void __launch_bounds__(256) gemm_ln_bf16_kernel(const GemmLnBf16Args p) {
  __shared__ __attribute__((aligned(16))) unsigned short lds[2 * (GEMM_BM + GEMM_BN) * GEMMB_PITCH];
  auto Ws = [&](int buf) { return lds + buf * (GEMM_BM + GEMM_BN) * GEMMB_PITCH; };
  auto Xs = [&](int buf) { return lds + buf * (GEMM_BM + GEMM_BN) * GEMMB_PITCH + GEMM_BN * GEMMB_PITCH; };
  const TX* const X = reinterpret_cast<const TX*>(p.X);
  const long long nMt = (p.M + GEMM_BM - 1) / GEMM_BM;
  const int nNt = (p.N + GEMM_BN - 1) / GEMM_BN;
  const long long total = nMt * nNt;
  const long long per = (total + 7) / 8;  // a contiguous run of tiles per die, as in gemm_ln_kernel
  const long long tile = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((long long)(blockIdx.x >> 3) >= per || tile >= total) return;
  const long long m0 = (tile / nNt) * GEMM_BM;
  const int n0 = (int)(tile % nNt) * GEMM_BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i = lane & 15, g = lane >> 4;
  const int wo = wave & 1, wn = wave >> 1;
  const int lr = tid >> 3, lc = 8 * (tid & 7);  // this thread's rows lr + 32 j and columns lc .. lc + 7 of a slice

  float mean[4], rstd[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const long long row = m0 + lr + 32 * j;
    mean[j] = row < p.M ? p.stats[2 * row] : 0.f;
    rstd[j] = row < p.M ? p.stats[2 * row + 1] : 0.f;
  }
  blk_u16x8 rw[4];
  blk_floatx4 rx[4][2], gn[2], of[2];
  bool live[4];
  auto fetch = [&](int k0) {
    const int k = k0 + lc;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      gn[h] = of[h] = blk_floatx4{0.f, 0.f, 0.f, 0.f};
      if (k < p.K) {
        gn[h] = *reinterpret_cast<const blk_floatx4*>(p.gain + k + 4 * h);
        of[h] = *reinterpret_cast<const blk_floatx4*>(p.offset + k + 4 * h);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int o = n0 + lr + 32 * j;
      const long long row = m0 + lr + 32 * j;
      rw[j] = blk_u16x8{0, 0, 0, 0, 0, 0, 0, 0};
      rx[j][0] = rx[j][1] = blk_floatx4{0.f, 0.f, 0.f, 0.f};
      live[j] = k < p.K && row < p.M;
      if (k < p.K && o < p.N) rw[j] = *reinterpret_cast<const blk_u16x8*>(p.W + (long long)o * p.K + k);
      if (live[j]) {
        rx[j][0] = blk_ld4<TX>(X, row * p.K + k);
        rx[j][1] = blk_ld4<TX>(X, row * p.K + k + 4);
      }
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      blk_u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (live[j]) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e) v[4 * h + e] = f32_to_bf16((rx[j][h][e] - mean[j]) * rstd[j] * gn[h][e] + of[h][e]);
      }
      *reinterpret_cast<blk_u16x8*>(Ws(buf) + (lr + 32 * j) * GEMMB_PITCH + lc) = rw[j];
      *reinterpret_cast<blk_u16x8*>(Xs(buf) + (lr + 32 * j) * GEMMB_PITCH + lc) = v;
    }
  };
  blk_floatx4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = blk_floatx4{0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int buf) {
    const unsigned short* wsb = Ws(buf) + (64 * wo + i) * GEMMB_PITCH + 8 * g;
    const unsigned short* xsb = Xs(buf) + (64 * wn + i) * GEMMB_PITCH + 8 * g;
#pragma unroll
    for (int h = 0; h < GEMMB_BK / 32; ++h) {
      blk_bf16x8 a[4], b[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        a[t] = *reinterpret_cast<const blk_bf16x8*>(wsb + 16 * t * GEMMB_PITCH + 32 * h);
        b[t] = *reinterpret_cast<const blk_bf16x8*>(xsb + 16 * t * GEMMB_PITCH + 32 * h);
      }
#pragma unroll
      for (int ob = 0; ob < 4; ++ob)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
          acc[ob][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ob], b[nb], acc[ob][nb], 0, 0, 0);
    }
  };
  const int nk = (p.K + GEMMB_BK - 1) / GEMMB_BK;
  fetch(0);
  stash(0);
  __syncthreads();
  for (int kt = 0; kt + 1 < nk; ++kt) {
    fetch((kt + 1) * GEMMB_BK);
    compute(kt & 1);
    stash((kt & 1) ^ 1);
    __syncthreads();
  }
  blk_floatx4 res[4][4];  // the residual, read under the last slice's matrix-core work
#pragma unroll
  for (int ob = 0; ob < 4; ++ob)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int o = n0 + 64 * wo + 16 * ob + 4 * g;
      const long long row = m0 + 64 * wn + 16 * nb + i;
      res[ob][nb] = blk_floatx4{0.f, 0.f, 0.f, 0.f};
      if (p.Res && o < p.N && row < p.M) res[ob][nb] = blk_ld4<unsigned short>(p.Res, row * p.N + o);
    }
  compute((nk - 1) & 1);
  // acc[ob][nb][v] = Y[m0 + 64 wn + 16 nb + i][n0 + 64 wo + 16 ob + 4 g + v]
#pragma unroll
  for (int ob = 0; ob < 4; ++ob) {
    const int o = n0 + 64 * wo + 16 * ob + 4 * g;
    if (o >= p.N) continue;
    blk_floatx4 bs = {0.f, 0.f, 0.f, 0.f};
    if (p.bias) bs = *reinterpret_cast<const blk_floatx4*>(p.bias + o);
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const long long row = m0 + 64 * wn + 16 * nb + i;
      if (row >= p.M) continue;
      const blk_floatx4 y = acc[ob][nb] + bs + res[ob][nb];
      if constexpr (OUT_BF16) {
        const blk_u16x4 v = {f32_to_bf16(y[0]), f32_to_bf16(y[1]), f32_to_bf16(y[2]), f32_to_bf16(y[3])};
        *reinterpret_cast<blk_u16x4*>(reinterpret_cast<unsigned short*>(p.Y) + row * p.N + o) = v;
      } else {
        *reinterpret_cast<blk_floatx4*>(reinterpret_cast<float*>(p.Y) + row * p.N + o) = y;
      }
    }
  }
}

__device__ __forceinline__ float softplus_f32(float z) {
  // log(1 + e^z); for large z the sum rounds to e^z and the result to z
  return z > 30.f ? z : log1pf(expf(z));
}

// The contextualisation maps of every (token, head): thread j of a workgroup owns output j of the 80 + 3r numbers of
// a problem (its row of the weights in registers) and walks the workgroup's tokens of one head; the head's initial
// state is read by all threads from the same 64 bytes.
__global__ void __launch_bounds__(320) cxt_maps_kernel(const CxtMapsArgs p) {
  const int r = p.r, nhead = 80 + r, nout = 80 + 3 * r;
  const int h = blockIdx.x % p.H;
  const long long t0 = (long long)(blockIdx.x / p.H) * p.tokens_per_block;
  const int j = threadIdx.x;
  if (j >= nout) return;
  const float* wrow;
  float bias;
  if (j < nhead) {
    wrow = p.W_head + ((long long)h * nhead + j) * 16;
    bias = p.b_head[(long long)h * nhead + j];
  } else {
    wrow = p.W_shared + (long long)(j - nhead) * 16;
    bias = p.b_shared[j - nhead];
  }
  float w[16];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const blk_floatx4 v = *reinterpret_cast<const blk_floatx4*>(wrow + 4 * q);
    w[4 * q] = v[0]; w[4 * q + 1] = v[1]; w[4 * q + 2] = v[2]; w[4 * q + 3] = v[3];
  }
  // where output j goes: array, its row length, the column
  float* dst;
  int len, col;
  bool act = true;
  if (j < 16) { dst = p.sA; len = 16; col = j; act = false; }
  else if (j < 32) { dst = p.rinv; len = 16; col = j - 16; }
  else if (j < 48) { dst = p.lgA; len = 16; col = j - 32; }
  else if (j < 64) { dst = p.lgB; len = 16; col = j - 48; }
  else if (j < 80) { dst = p.lgQ; len = 16; col = j - 64; }
  else if (j < nhead) { dst = p.sQf; len = r; col = j - 80; }
  else if (j < nhead + r) { dst = p.sB; len = r; col = j - nhead; act = false; }
  else { dst = p.sQ; len = r; col = j - nhead - r; }
  long long t1 = t0 + p.tokens_per_block;
  t1 = t1 < p.M ? t1 : p.M;
  for (long long t = t0; t < t1; ++t) {
    const long long prob = t * p.H + h;
    const float* x = p.H0 + prob * 16;
    float s0 = bias, s1 = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const blk_floatx4 v = *reinterpret_cast<const blk_floatx4*>(x + 4 * q);
      s0 = __builtin_fmaf(w[4 * q], v[0], s0);
      s1 = __builtin_fmaf(w[4 * q + 1], v[1], s1);
      s0 = __builtin_fmaf(w[4 * q + 2], v[2], s0);
      s1 = __builtin_fmaf(w[4 * q + 3], v[3], s1);
    }
    const float z = s0 + s1;
    dst[prob * len + col] = act ? softplus_f32(z) : z;
  }
}

// The same maps for r = 16 and a multiple of four heads, with coalesced stores: wavefront a of a workgroup of eight
// owns array a (sA, rinv, lgA, lgB, lgQ, sQf, sB, sQ), its lanes four consecutive heads times sixteen columns, so that a
// store writes 256 consecutive bytes; the workgroup walks its tokens for one group of four heads.
__global__ void __launch_bounds__(512) cxt_maps16_kernel(const CxtMapsArgs p) {
  const int groups = p.H / 4;
  const int hg = blockIdx.x % groups;
  const long long t0 = (long long)(blockIdx.x / groups) * p.tokens_per_block;
  const int a = threadIdx.x >> 6, lane = threadIdx.x & 63, q = lane >> 4, col = lane & 15;
  const int h = 4 * hg + q;
  const float* wrow;
  float bias;
  if (a < 6) {
    const int j = a < 5 ? 16 * a + col : 80 + col;
    wrow = p.W_head + ((long long)h * 96 + j) * 16;
    bias = p.b_head[(long long)h * 96 + j];
  } else {
    const int j = 16 * (a - 6) + col;
    wrow = p.W_shared + (long long)j * 16;
    bias = p.b_shared[j];
  }
  float w[16];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const blk_floatx4 v = *reinterpret_cast<const blk_floatx4*>(wrow + 4 * k);
    w[4 * k] = v[0]; w[4 * k + 1] = v[1]; w[4 * k + 2] = v[2]; w[4 * k + 3] = v[3];
  }
  float* const arrays[8] = {p.sA, p.rinv, p.lgA, p.lgB, p.lgQ, p.sQf, p.sB, p.sQ};
  float* dst = arrays[0];
#pragma unroll
  for (int k = 1; k < 8; ++k) dst = a == k ? arrays[k] : dst;
  const bool act = !(a == 0 || a == 6);
  long long t1 = t0 + p.tokens_per_block;
  t1 = t1 < p.M ? t1 : p.M;
  // four tokens at a time, so that their reads are in flight together
  for (long long t = t0; t < t1; t += 4) {
    blk_floatx4 v[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long tt = t + u < t1 ? t + u : t1 - 1;
      const float* x = p.H0 + (tt * p.H + h) * 16;
#pragma unroll
      for (int k = 0; k < 4; ++k) v[u][k] = *reinterpret_cast<const blk_floatx4*>(x + 4 * k);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (t + u >= t1) break;
      float s0 = bias, s1 = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        s0 = __builtin_fmaf(w[4 * k], v[u][k][0], s0);
        s1 = __builtin_fmaf(w[4 * k + 1], v[u][k][1], s1);
        s0 = __builtin_fmaf(w[4 * k + 2], v[u][k][2], s0);
        s1 = __builtin_fmaf(w[4 * k + 3], v[u][k][3], s1);
      }
      const float z = s0 + s1;
      dst[((t + u) * p.H + h) * 16 + col] = act ? softplus_f32(z) : z;
    }
  }
}

// Q^(i) = Qc^(i) Qc^(i)^T / sqrt(16), one workgroup of 256 threads per basis matrix
__global__ void __launch_bounds__(256) qbasis_kernel(const float* Qc, float* Qb) {
  const float* M = Qc + (long long)blockIdx.x * 256;
  const int a = threadIdx.x >> 4, b = threadIdx.x & 15;
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 16; ++k) s = __builtin_fmaf(M[16 * a + k], M[16 * b + k], s);
  Qb[(long long)blockIdx.x * 256 + threadIdx.x] = 0.25f * s;
}

}  // namespace ttc
