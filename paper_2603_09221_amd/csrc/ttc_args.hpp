// Kernel argument blocks (plain structs passed by value at launch), shared by the host entry points and
// the kernel translation units.
#pragma once
#include <stdint.h>

namespace ttc {

struct SolveArgs {
  long long n;
  int T, flags, ngroups;  // the T factors are applied in ngroups groups, one dense solve each
  float growth_limit;     // growth guard of the symplectic kernels: max |Y1| a group may reach; 0 = no guard
  const void *A, *B, *Q, *R, *QT, *x0;
  long long sA, sB, sQ, sR, sQT, sx0;
  float *P0, *K0, *u0, *value;
  int* info;
  float* ws;  // gridDim.x slots of d*d floats (C_K of the problem in flight, register layout); more for doubling
#ifdef TTC_PHASE_TIMERS
  long long* dbg = nullptr;  // development builds only: 8 cycle counters, accumulated by workgroup 0
#endif
};

struct RolloutArgs {
  long long n;
  int T, flags;
  const void *A, *B, *Q, *R, *QT, *x0;
  long long sA, sB, sQ, sR, sQT, sx0;
  float *U, *X, *cost;
  int* info;
  float* ws;  // gridDim.x slots of (T+3) d*d floats: G, R^{-1} B^T, A^T (register layout), K_0 .. K_{T-1}
};

struct DoublingArgs {
  SolveArgs s;  // problem, outputs, workspace (ngroups unused)
  int m;        // number of one-step maps composed before the last step (T, or T-1 when Q_T is given)
  int p_from_qt;  // 1: the backward recursion starts at Q_T; 0: it starts at 0 (Q_T is Q = f(0))
};

// workspace slots of a workgroup, d*d floats each
enum { DBL_A = 0, DBL_G = 1, DBL_H = 2, DBL_G0 = 3, DBL_P = 4, DBL_X = 5, DBL_SLOTS = 6 };

struct TvArgs {
  SolveArgs s;                 // n, T, A, B, Q, R, x0 and their problem strides, outputs (QT, ws, groups unused)
  long long tA, tB, tQ, tR;    // elements between consecutive steps
  const float* PT = nullptr;   // if set: the terminal value matrix, fp32, instead of Q[T-1] (solve_tv_kernel only)
  long long sPT = 0;           // elements between consecutive problems of PT
};

struct TvRolloutArgs {
  RolloutArgs r;               // n, T, A, B, Q, R, x0 and their problem strides, U, X, cost, info, ws (QT unused)
  long long tA, tB, tQ, tR;    // elements between consecutive steps
};

struct ScanArgs {
  TvArgs tv;   // the problems (inputs only)
  float* ws;   // n*T elements of 3 d^2 floats
  int stride;  // combine rounds: the stride st
};

struct BackwardArgs {
  RolloutArgs r;              // n, T, A, B, Q, R, QT (time-invariant problems only), x0, strides, info, ws; U, X, cost unused
  long long tA, tB, tQ, tR;   // elements between consecutive steps (0: the same matrix in every step)
  const float* g;             // (n, m) dl/du_0
  long long sg;
  float *gA, *gB, *gQ, *gR;   // (n, T, d, d), or (n, d, d) when sum_steps
  float* gQT;                 // (n, d, d) or NULL: the terminal cost's gradient when it is its own matrix (sum_steps)
  float* gx0;                 // (n, d)
  int sum_steps;              // 1: time-invariant parameters, gradients summed over the steps
};

constexpr int CXT_RMAX = 64;  // most basis matrices per group

struct CxtArgs {
  SolveArgs s;  // n, T, x0 (stride 16), outputs; flags = 0; the matrix inputs are unused
  int r;
  const void *sA, *sB, *sQ, *sQf, *rinv, *lgA, *lgB, *lgQ;  // (n,16) vectors, (n,r) coefficients
  const void *Bbasis, *Qbasis;                              // (r,16,16), shared by all problems
  // roll-out and backward pass: per problem roll_slots matrices of 256 floats: Bbar, Qbar, Q_T, K_0 .. K_{T-1} and, for
  // the backward pass (dual_g set, roll_slots = T + 4), in the first 16 floats of the last one the first control of the
  // dual problem, ut_0 = -S_0^{-1} g refined once with S_0; NULL for a plain solve
  float* roll_ws = nullptr;
  int roll_slots = 0;             // 0 stands for T + 3
  const float* dual_g = nullptr;  // (n,16) dl/du_0, or NULL
};

struct CxtRolloutArgs {
  CxtArgs c;  // the problems; c.roll_ws filled by solve_cxt_kernel, c.s.info written by it
  float *U, *X, *cost;
};

// ---- backward pass of the structured problems (ttc_cxt_backward.hpp)
constexpr int CXT_BASIS_SLAB = 32;  // the smallest slab of the basis sums
struct CxtBackwardArgs {
  CxtArgs c;             // the problems (inputs only, the whole batch; c.s.n = all problems)
  long long first;       // the chunk: problems first .. first + count - 1
  long long count;
  int basis_slab;        // problems per workgroup of the basis sums (>= CXT_BASIS_SLAB: atomic additions stay rare)
  int traj_in_lds;       // the trajectories of a wavefront's four problems stay in LDS: short horizons
  int basis_in_lds;      // the workgroup keeps a copy of the basis matrices in LDS: r <= 16
  float* roll;           // (count, T + 4, 256): what solve_cxt_kernel leaves for the backward pass (c.roll_ws layout)
  float* traj;           // (count, 4, T + 1, 16): the primal and dual states and controls
  float* keep;           // (count, 3, 256): dl/dBbar, dl/dQbar, dl/dQ_T
  const float* g;        // (n, 16) dl/du_0
  const int* info;       // (n) as written by the solve kernel
  float *gsA, *gsB, *gsQ, *gsQf, *grinv, *glgA, *glgB, *glgQ, *gx0;  // the caller's arrays, (n, 16) or (n, r)
  float *gBbasis, *gQbasis;                                          // the caller's arrays, (r, 256), accumulated
};

// ---- the block around the structured solver (ttc_block.hpp)
struct LnStatsArgs {
  const void* X;   // (M, L) row-major, float32 or bfloat16
  float* stats;    // (M, 2): mean, 1 / sqrt(biased variance + eps)
  long long M;
  int L;           // multiple of 4
  float eps;
};

struct GemmLnArgs {
  const float* X;       // (M, K) row-major, rows normalised on load with stats, gain, offset
  const float* stats;   // (M, 2)
  const float* gain;    // (K)
  const float* offset;  // (K)
  const float* W;       // (N, K) row-major
  const float* bias;    // (N) or NULL
  const float* Res;     // (M, N) or NULL: added to the result (may be Y itself)
  float* Y;             // (M, N)
  long long M;
  int N, K;             // multiples of 4
};

// the bfloat16 variant of the projections (the block's TTC_BLOCK_FLAG_BF16): X float32 or bfloat16, W bfloat16,
// Res bfloat16 or NULL, Y float32 or bfloat16 (bfloat16 values are stored as uint16_t)
struct GemmLnBf16Args {
  const void* X;        // (M, K): element type by the kernel's template argument
  const float* stats;   // (M, 2)
  const float* gain;    // (K) float32
  const float* offset;  // (K) float32
  const uint16_t* W;    // (N, K) bfloat16
  const float* bias;    // (N) float32 or NULL
  const uint16_t* Res;  // (M, N) bfloat16 or NULL (may be Y itself)
  void* Y;              // (M, N): element type by the kernel's template argument
  long long M;
  int N, K;             // multiples of 8
};

struct CxtMapsArgs {
  const float* H0;        // (M, H, 16)
  const float* W_head;    // (H, 80 + r, 16): rows sA, rinv, lgA, lgB, lgQ (16 each), sQf (r)
  const float* b_head;    // (H, 80 + r)
  const float* W_shared;  // (2r, 16): rows sB (r), sQ (r)
  const float* b_shared;  // (2r)
  float *sA, *rinv, *lgA, *lgB, *lgQ;  // (M*H, 16)
  float *sQf, *sB, *sQ;                // (M*H, r)
  long long M;
  int H, r;
  int tokens_per_block;
};

}  // namespace ttc
