// C-ABI entry points of the batched finite-horizon LQR solver (see include/ttc_lqr.h): argument checks,
// grid sizing and kernel selection.  The kernels live in the k_*.hip translation units.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/ttc_lqr.h"
#include "ttc_launch.hpp"

// Scratch of ttc_lqr_solve_noalloc: a fixed array in device memory, one copy per GPU the library is loaded
// on, held until the process ends.  Host code never uses the array's name as an address: it asks the runtime
// for the device address once per device (scratch_for_current_device) and passes that pointer on.
#define TTC_NOALLOC_SCRATCH_BYTES (24u << 20)
static __device__ __align__(256) unsigned char scratch[TTC_NOALLOC_SCRATCH_BYTES];

namespace ttc {

// Per-device facts, asked once per device (thread-safe): the compute-unit count and, per kernel instance,
// the resident workgroups per compute unit.
constexpr int MAX_DEVICES = 64;
static int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return dev < 0 || dev >= MAX_DEVICES ? 0 : dev;
}
static int cu_count() {
  static std::once_flag once[MAX_DEVICES];
  static int count[MAX_DEVICES];
  const int dev = current_device();
  std::call_once(once[dev], [dev] {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
      (void)hipGetLastError();
      n = 256;  // MI355X
    }
    count[dev] = n;
  });
  return count[dev];
}
// Device address of this GPU's copy of the scratch array (nullptr if the runtime refuses): asked once per
// device, with that device current, and kept.
static void* scratch_for_current_device() {
  static std::once_flag once[MAX_DEVICES];
  static void* ptr[MAX_DEVICES];
  const int dev = current_device();
  std::call_once(once[dev], [dev] {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      q = nullptr;
    }
    ptr[dev] = q;
  });
  return ptr[dev];
}
// Persistent grids: as many workgroups as are resident at once, CUs x (workgroups per CU), so that no
// workgroup waits for another to finish.  The per-CU number is what the runtime reports for the kernel
// (registers and LDS decide it); the table is the fallback when no device can be asked.
enum Kind { KIND_SOLVE = 0, KIND_DOUBLING = 1, KIND_ROLLOUT = 2, KIND_SOLVE_QUAD = 3, KIND_SOLVE_TV = 4, KIND_TV_QUAD = 5,
            KIND_ROLLOUT_TV = 6, KIND_CXT = 7, KIND_SCAN = 8, KIND_BACKWARD = 9, KIND_COUNT = 10 };
static int dindex(int d) { return d == 16 ? 0 : d == 32 ? 1 : d == 64 ? 2 : 3; }
template <int D>
static int occupancy_of(Kind kind, bool bf16) {
  switch (kind) {
    case KIND_SOLVE:
      if constexpr (D >= 32) return occupancy_solve<D>(bf16);
      else return 0;  // d = 16 has its own kernel
    case KIND_DOUBLING: return occupancy_doubling<D>(bf16);
    case KIND_ROLLOUT: return occupancy_rollout<D>(bf16);
    case KIND_SOLVE_TV: return occupancy_tv<D>(bf16);
    case KIND_ROLLOUT_TV: return occupancy_rollout_tv<D>(bf16);
    case KIND_SCAN: return occupancy_scan<D>();
    case KIND_BACKWARD: return occupancy_backward<D>(bf16);
    case KIND_SOLVE_QUAD: return occupancy_small(bf16);  // the d = 16 kernels
    case KIND_TV_QUAD: return occupancy_tv_small(bf16);
    case KIND_CXT: return occupancy_cxt(bf16);
    default: return 0;
  }
}
static int blocks_per_cu(Kind kind, int d, bool bf16) {
  struct Entry {
    std::once_flag once;
    int value;
  };
  static Entry cache[MAX_DEVICES][KIND_COUNT][4][2];
  Entry& c = cache[current_device()][kind][dindex(d)][bf16 ? 1 : 0];
  std::call_once(c.once, [&] {
    int nb = 0;
    switch (d) {
      case 16: nb = occupancy_of<16>(kind, bf16); break;
      case 32: nb = occupancy_of<32>(kind, bf16); break;
      case 64: nb = occupancy_of<64>(kind, bf16); break;
      case 128: nb = occupancy_of<128>(kind, bf16); break;
    }
    if (nb <= 0) {
      static const int table[KIND_COUNT][4] = {{20, 8, 2, 1}, {16, 8, 2, 1}, {12, 4, 2, 1}, {8, 8, 2, 1}, {20, 8, 2, 1},
                                               {8, 8, 2, 1},  {12, 4, 2, 1}, {8, 8, 2, 1},  {16, 8, 2, 1},
                                               {12, 4, 2, 1}};
      nb = table[kind][dindex(d)];
    }
    c.value = nb > 32 ? 32 : nb;
  });
  return c.value;
}
static long long grid_blocks(Kind kind, int d, bool bf16) {
  return (long long)cu_count() * blocks_per_cu(kind, d, bf16);
}
// Growth guard of the symplectic kernels: the largest max |Y1| a group of factors may reach before the problem is
// handed to the Riccati recursion.  Float32: measured on the benchmark generators and on inputs with R, Q scaled
// by 1e-2..1e2 and rho(A) in 0.5..1.2, every problem whose error exceeded 5e-5 had passed 260 and the worst error
// below 256 was 3.7e-5; default groups on the benchmark inputs reach 40..200.  Bfloat16 inputs carry a 2e-2
// tolerance: groups of five factors reach about 1e3.
constexpr float GROWTH_LIMIT_F32 = 256.f;
constexpr float GROWTH_LIMIT_BF16 = 16384.f;

// d = 16: large batches go four problems to a wavefront (more throughput per instruction issued), small ones
// one problem to a wavefront (more wavefronts in flight, lower latency).  Crossover measured on MI355X, in
// problems per compute unit: 12 for the symplectic kernel (T = 8), 24 for the Riccati kernel (T = 64).
constexpr long long QUAD_MIN_PER_CU_SOLVE = 12;
constexpr long long QUAD_MIN_PER_CU_TV = 24;
static bool use_quad_kernel(const ttc_lqr_problem_t* q) {
  return q->d == 16 && !(q->flags & TTC_FLAG_DOUBLING) && q->n >= QUAD_MIN_PER_CU_SOLVE * cu_count();
}
static bool use_quad_kernel_tv(const ttc_lqr_tv_problem_t* q) {
  return q->d == 16 && q->n >= QUAD_MIN_PER_CU_TV * cu_count();
}

static bool shape_supported_dm(int d, int m) { return d == m && (d == 16 || d == 32 || d == 64 || d == 128); }
static bool shape_supported(const ttc_lqr_problem_t* q) { return shape_supported_dm(q->d, q->m); }
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

// kernel launches by state size
#define TTC_BY_D(d, CALL)                               \
  switch (d) {                                          \
    case 16: { constexpr int D = 16; return CALL; }     \
    case 32: { constexpr int D = 32; return CALL; }     \
    case 64: { constexpr int D = 64; return CALL; }     \
    case 128: { constexpr int D = 128; return CALL; }   \
    default: return hipErrorInvalidValue;               \
  }
static hipError_t run_solve(const SolveArgs& a, int d, bool bf16, dim3 grid, hipStream_t st) {
  switch (d) {  // d = 16 runs solve_small_kernel instead
    case 32: return launch_solve<32>(a, bf16, grid, st);
    case 64: return launch_solve<64>(a, bf16, grid, st);
    case 128: return launch_solve<128>(a, bf16, grid, st);
    default: return hipErrorInvalidValue;
  }
}
static hipError_t run_doubling(const DoublingArgs& a, int d, bool bf16, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_doubling<D>(a, bf16, grid, st))
}
static hipError_t run_rollout(const RolloutArgs& a, int d, bool bf16, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_rollout<D>(a, bf16, grid, st))
}
static hipError_t run_tv(const TvArgs& a, int d, bool bf16, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_tv<D>(a, bf16, grid, st))
}
static hipError_t run_rollout_tv(const TvRolloutArgs& a, int d, bool bf16, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_rollout_tv<D>(a, bf16, grid, st))
}
static hipError_t run_scan_leaf(const ScanArgs& a, int d, bool bf16, int ipw, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_scan_leaf<D>(a, bf16, ipw, grid, st))
}
static hipError_t run_scan_combine(const ScanArgs& a, int d, int ipw, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_scan_combine<D>(a, ipw, grid, st))
}
static hipError_t run_scan_apply(const ScanArgs& a, int d, int ipw, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_scan_apply<D>(a, ipw, grid, st))
}
static hipError_t run_scan_gather(const ScanArgs& a, float* P, int d, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_scan_gather<D>(a, P, grid, st))
}
static hipError_t run_backward(const BackwardArgs& a, int d, bool bf16, dim3 grid, hipStream_t st) {
  TTC_BY_D(d, launch_backward<D>(a, bf16, grid, st))
}
#undef TTC_BY_D

}  // namespace ttc

#ifdef TTC_PHASE_TIMERS
// Development builds only: device buffer of eight cycle counters that workgroup 0 of ttc_lqr_solve adds to.
static long long* g_phase_timers = nullptr;
extern "C" void ttc_debug_set_phase_timers(long long* device_counters) { g_phase_timers = device_counters; }
#endif

extern "C" {

size_t ttc_lqr_workspace_bytes(const ttc_lqr_problem_t* problem, int for_rollout) {
  if (!problem || problem->T < 1 || !ttc::shape_supported(problem)) return 0;
  // (the default-path kernel of d = 16 needs no workspace; its grid size stands in)
  const ttc::Kind kind = for_rollout ? ttc::KIND_ROLLOUT
                         : (problem->flags & TTC_FLAG_DOUBLING) ? ttc::KIND_DOUBLING
                         : problem->d == 16 ? ttc::KIND_SOLVE_QUAD : ttc::KIND_SOLVE;
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
  // Grouping of the T factors (one dense solve per group); group lengths differ by at most one and the longer
  // groups come first.  rebase_every = k asks for ceil(T/k) groups.  The default for float32 inputs is groups of
  // three factors with at most one group of four, which then comes first, where the pair starts from the terminal
  // cost and grows least (an error made at an early re-base is also damped by the contracting closed loop, the
  // last group's error reaches P_0 undamped); for bfloat16 inputs, whose tolerance is that of their rounding,
  // groups of five.  Whatever the grouping, the kernels watch max |Y1| (the growth guard): a problem whose pair
  // grows beyond the limit inside a group is solved by the recursion of Prop. 3.1 in its printed form instead,
  // so that the accuracy does not rest on the inputs being like those the grouping was measured on.
  {
    const long T = problem->T;
    long g;
    if (problem->flags & TTC_FLAG_PURE_SYMPLECTIC) g = 1;
    else if (problem->rebase_every > 0) g = (T + problem->rebase_every - 1) / problem->rebase_every;
    else if (problem->in_dtype == TTC_BF16) g = (T + 4) / 5;
    else {
      const long by3 = (T + 1) / 3, by34 = (T * 10 + 33) / 34;  // ceil((T-1)/3), ceil(T/3.4)
      g = by3 > by34 ? by3 : by34;
    }
    if (g < 1) g = 1;
    if (g > T) g = T;
    a.ngroups = (int)g;
    a.growth_limit = (problem->flags & TTC_FLAG_PURE_SYMPLECTIC) ? 0.f
                     : problem->in_dtype == TTC_BF16 ? ttc::GROWTH_LIMIT_BF16 : ttc::GROWTH_LIMIT_F32;
  }
  a.A = problem->A; a.B = problem->B; a.Q = problem->Q; a.R = problem->R; a.QT = problem->QT; a.x0 = problem->x0;
  a.sA = problem->sA; a.sB = problem->sB; a.sQ = problem->sQ; a.sR = problem->sR; a.sQT = problem->sQT;
  a.sx0 = problem->sx0;
  a.P0 = solution->P0; a.K0 = solution->K0; a.u0 = solution->u0; a.value = solution->value;
  a.info = solution->info;
  a.ws = static_cast<float*>(workspace);
#ifdef TTC_PHASE_TIMERS
  a.dbg = g_phase_timers;
#endif
  const bool doubling = (problem->flags & TTC_FLAG_DOUBLING) != 0;
  const bool bf16 = problem->in_dtype == TTC_BF16;
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
    e = ttc::run_doubling(da, problem->d, bf16, grid, s);
  } else if (quad) {
    e = ttc::launch_small(a, bf16, 4, grid, s);
  } else if (small) {  // a batch that does not fill the chip: one problem to a wavefront
    e = ttc::launch_small(a, bf16, 1, grid, s);
  } else {
    e = ttc::run_solve(a, problem->d, bf16, grid, s);
  }
  return e == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

ttc_status_t ttc_lqr_solve_noalloc(const ttc_lqr_problem_t* problem, const ttc_lqr_solution_t* solution,
                                   void* hip_stream) {
  const ttc_status_t st = ttc::validate(problem);
  if (st != TTC_OK) return st;
  if (problem->flags & TTC_FLAG_DOUBLING) return TTC_ERR_UNSUPPORTED;  // its six slots per workgroup do not fit
  const size_t need = ttc_lqr_workspace_bytes(problem, 0);
  if (need > (size_t)TTC_NOALLOC_SCRATCH_BYTES) return TTC_ERR_WORKSPACE;
  void* const ws = ttc::scratch_for_current_device();
  if (!ws) return TTC_ERR_DEVICE;
  return ttc_lqr_solve(problem, solution, ws, (size_t)TTC_NOALLOC_SCRATCH_BYTES, hip_stream);
}

size_t ttc_lqr_noalloc_scratch_bytes(void) { return (size_t)TTC_NOALLOC_SCRATCH_BYTES; }

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
  const hipError_t e = ttc::run_rollout(a, problem->d, problem->in_dtype == TTC_BF16, grid, s);
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
  const hipError_t e = ttc::run_rollout_tv(a, q->d, bf16, grid, st);
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
  a.s.growth_limit = 0.f;
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
  const bool quad = ttc::use_quad_kernel_tv(q);
  const long long gb = ttc::grid_blocks(small ? ttc::KIND_TV_QUAD : ttc::KIND_SOLVE_TV, q->d, bf16);
  const long long items = quad ? (q->n + 3) / 4 : q->n;
  const dim3 grid((unsigned)(items < gb ? items : gb));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (quad) {
    e = ttc::launch_tv_small(a, bf16, 4, grid, st);
  } else if (small) {
    e = ttc::launch_tv_small(a, bf16, 1, grid, st);
  } else {
    e = ttc::run_tv(a, q->d, bf16, grid, st);
  }
  return e == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

size_t ttc_lqr_tv_scan_workspace_bytes(const ttc_lqr_tv_problem_t* q) {
  if (!q || q->n < 0 || q->T < 1 || !ttc::shape_supported_dm(q->d, q->m)) return 0;
  return (size_t)q->n * (size_t)q->T * 3 * (size_t)q->d * (size_t)q->d * sizeof(float);
}

// Launch shapes of the tree kernels: a round with `items` independent items runs one item per workgroup, except at
// d = 16 when there are at least fourteen items per compute unit: from there on the kernels that take four items per
// wavefront are faster (measured on 256 compute units: 16.8 against 17.7 us at 4096 items, 41 against 50 us at 16384;
// with 2048 items the one-item kernels finish the round sooner, 13 against 15.5).
struct ScanPlan {
  long long gb;   // resident workgroups of the one-item kernels
  long long gb4;  // of the four-item kernels (d = 16)
  long long cus;  // compute units
  bool quads;
  int ipw(long long items) const { return quads && items >= 14 * cus ? 4 : 1; }
  dim3 grid(long long items) const {
    if (ipw(items) == 4) {
      const long long groups = (items + 3) / 4;
      return dim3((unsigned)(groups < gb4 ? groups : gb4));
    }
    return dim3((unsigned)(items < gb ? items : gb));
  }
};
static ScanPlan scan_plan(int d, bool bf16) {
  ScanPlan p;
  p.gb = ttc::grid_blocks(ttc::KIND_SCAN, d, bf16);
  p.gb4 = 12LL * ttc::cu_count();  // three wavefronts per SIMD (registers)
  p.cus = ttc::cu_count();
  p.quads = d == 16;
  return p;
}

// The elements of every step and the rounds of pairwise compositions (the up-sweep), common to
// ttc_lqr_solve_tv_scan and ttc_lqr_tv_scan_values; fills sa for the launches that follow.
static hipError_t scan_up_sweep(const ttc_lqr_tv_problem_t* q, ttc::ScanArgs& sa, void* workspace, hipStream_t st) {
  ttc::TvArgs& a = sa.tv;
  a.s.n = q->n;
  a.s.T = q->T;
  a.s.flags = 0;
  a.s.ngroups = q->T;
  a.s.growth_limit = 0.f;
  a.s.A = q->A; a.s.B = q->B; a.s.Q = q->Q; a.s.R = q->R; a.s.QT = nullptr; a.s.x0 = q->x0;
  a.s.sA = q->sA; a.s.sB = q->sB; a.s.sQ = q->sQ; a.s.sR = q->sR; a.s.sQT = 0; a.s.sx0 = q->sx0;
  a.s.P0 = nullptr; a.s.K0 = nullptr; a.s.u0 = nullptr; a.s.value = nullptr; a.s.info = nullptr;
  a.s.ws = nullptr;
  a.tA = q->tA; a.tB = q->tB; a.tQ = q->tQ; a.tR = q->tR;
  sa.ws = static_cast<float*>(workspace);
  sa.stride = 0;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const int d = q->d;
  const ScanPlan plan = scan_plan(d, bf16);
  hipError_t e = ttc::run_scan_leaf(sa, d, bf16, plan.ipw(q->n * q->T), plan.grid(q->n * q->T), st);
  if (e != hipSuccess) return e;
  for (long long stride = 1; stride < q->T;) {
    sa.stride = (int)stride;
    const long long per = (q->T - stride + 2 * stride - 1) / (2 * stride);
    e = ttc::run_scan_combine(sa, d, plan.ipw(q->n * per), plan.grid(q->n * per), st);
    if (e != hipSuccess) return e;
    stride *= 2;
  }
  return hipSuccess;
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
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (scan_up_sweep(q, sa, workspace, st) != hipSuccess) return TTC_ERR_DEVICE;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const int d = q->d;
  // the step s = 0 as printed, from P_1 = H of the first element
  ttc::TvArgs last = sa.tv;
  last.s.P0 = solution->P0; last.s.K0 = solution->K0; last.s.u0 = solution->u0; last.s.value = solution->value;
  last.s.info = solution->info;
  last.s.T = 1;
  last.s.ngroups = 1;
  last.PT = sa.ws + 2 * (size_t)d * d;
  last.sPT = (long long)q->T * 3 * d * d;
  const long long gt = ttc::grid_blocks(ttc::KIND_SOLVE_TV, d, bf16);
  const dim3 grid((unsigned)(q->n < gt ? q->n : gt));
  return ttc::run_tv(last, d, bf16, grid, st) == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

size_t ttc_lqr_tv_scan_values_workspace_bytes(const ttc_lqr_tv_problem_t* q) {
  if (!q || q->n < 0 || q->T < 1 || !ttc::shape_supported_dm(q->d, q->m)) return 0;
  // the elements, then one control vector per (problem, step) that the gains' launch writes and nobody reads
  return ttc_lqr_tv_scan_workspace_bytes(q) + (size_t)q->n * (size_t)q->T * (size_t)q->m * sizeof(float);
}

ttc_status_t ttc_lqr_tv_scan_values(const ttc_lqr_tv_problem_t* q, float* P, float* K, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t stv = validate_tv(q);
  if (stv != TTC_OK) return stv;
  if (!P && !K) return TTC_ERR_INVALID_ARG;
  if (!ttc::aligned_ptr(P, 16) || !ttc::aligned_ptr(K, 16)) return TTC_ERR_INVALID_ARG;
  // the gains are computed as n*T one-step problems, which needs the steps of a problem to follow each other at the
  // problems' own spacing
  if (K && q->T > 1 && (q->sA != q->T * q->tA || q->sB != q->T * q->tB || q->sR != q->T * q->tR)) return TTC_ERR_UNSUPPORTED;
  if (q->n == 0) return TTC_OK;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_lqr_tv_scan_values_workspace_bytes(q))
    return TTC_ERR_WORKSPACE;
  ttc::ScanArgs sa;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (scan_up_sweep(q, sa, workspace, st) != hipSuccess) return TTC_ERR_DEVICE;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const int d = q->d;
  const ScanPlan plan = scan_plan(d, bf16);
  const long long gb = plan.gb;
  auto grid_for = [&](long long items) { return dim3((unsigned)(items < gb ? items : gb)); };
  long long top = 1;
  while (top * 2 < q->T) top *= 2;
  for (long long stride = top; stride >= 1; stride /= 2) {  // the down-sweep
    sa.stride = (int)stride;
    if (stride >= q->T) continue;  // T = 1: a single, constant element
    const long long per = (q->T - stride + 2 * stride - 1) / (2 * stride);
    if (ttc::run_scan_apply(sa, d, plan.ipw(q->n * per), plan.grid(q->n * per), st) != hipSuccess) return TTC_ERR_DEVICE;
  }
  if (P && ttc::run_scan_gather(sa, P, d, grid_for(q->n * q->T), st) != hipSuccess) return TTC_ERR_DEVICE;
  if (K) {
    // step s of problem p, from P_{s+1} = the H slot of element s: K_s = -S_s^{-1} B_s^T P_{s+1} A_s (Eq. "decode")
    ttc::TvArgs g = sa.tv;
    g.s.n = q->n * q->T;
    g.s.T = 1;
    g.s.ngroups = 1;
    g.s.sA = q->tA; g.s.sB = q->tB; g.s.sQ = q->tQ; g.s.sR = q->tR;
    if (q->T == 1) { g.s.sA = q->sA; g.s.sB = q->sB; g.s.sQ = q->sQ; g.s.sR = q->sR; }
    g.s.sx0 = 0;
    g.s.K0 = K;
    g.s.u0 = reinterpret_cast<float*>(static_cast<char*>(workspace) + ttc_lqr_tv_scan_workspace_bytes(q));
    g.PT = sa.ws + 2 * (size_t)d * d;
    g.sPT = 3LL * d * d;
    const long long gt = ttc::grid_blocks(ttc::KIND_SOLVE_TV, d, bf16);
    const dim3 grid((unsigned)(g.s.n < gt ? g.s.n : gt));
    if (ttc::run_tv(g, d, bf16, grid, st) != hipSuccess) return TTC_ERR_DEVICE;
  }
  return TTC_OK;
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
  a.s.growth_limit = 0.f;
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

static hipError_t run_cxt(const ttc::CxtArgs& a, bool bf16, hipStream_t st) {
  const long long gb = ttc::grid_blocks(ttc::KIND_CXT, 16, bf16);
  // batches that do not fill the resident wavefronts four problems at a time go one problem to a wavefront
  const bool single = a.s.n <= gb;
  const long long items = single ? a.s.n : (a.s.n + 3) / 4;
  const dim3 grid((unsigned)(items < gb ? items : gb));
  return ttc::launch_cxt(a, bf16, single ? 1 : 4, grid, st);
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
  return run_cxt(a, q->in_dtype == TTC_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

// ---- the whole block around the structured solver ------------------------------------------------------------
namespace {
struct BlockLayout {  // offsets into the workspace, in floats, each a multiple of 64
  size_t stats_in, h0, sA, rinv, lgA, lgB, lgQ, sQf, sB, sQ, qbasis, o, stats_out, info, total;
};
size_t round64(size_t x) { return (x + 63) / 64 * 64; }
BlockLayout block_layout(long long M, int H, int r) {
  BlockLayout L;
  const size_t P = (size_t)M * H;
  size_t at = 0;
  auto take = [&](size_t nfloats) { const size_t here = at; at += round64(nfloats); return here; };
  L.stats_in = take(2 * (size_t)M);
  L.h0 = take(P * 16);
  L.sA = take(P * 16); L.rinv = take(P * 16); L.lgA = take(P * 16); L.lgB = take(P * 16); L.lgQ = take(P * 16);
  L.sQf = take(P * r); L.sB = take(P * r); L.sQ = take(P * r);
  L.qbasis = take((size_t)r * 256);
  L.o = take(P * 16);
  L.stats_out = take(2 * (size_t)M);
  L.info = take(P);
  L.total = at;
  return L;
}
ttc_status_t validate_block(const ttc_block_t* b) {
  if (!b || b->n_tokens < 0 || b->C < 1 || b->H < 1 || b->d < 1 || b->r < 1 || b->T < 1 ||
      (b->flags & ~TTC_BLOCK_FLAG_BF16) != 0)
    return TTC_ERR_INVALID_ARG;
  if (!(b->eps > 0.f)) return TTC_ERR_INVALID_ARG;
  if (b->d != 16 || b->r > ttc::CXT_RMAX || b->r % 4 != 0 || b->C % 4 != 0) return TTC_ERR_UNSUPPORTED;
  if ((b->flags & TTC_BLOCK_FLAG_BF16) && b->C % 8 != 0) return TTC_ERR_UNSUPPORTED;
  if ((long long)b->n_tokens * b->H > (1LL << 40)) return TTC_ERR_INVALID_ARG;
  return TTC_OK;
}
}  // namespace

size_t ttc_block_workspace_bytes(const ttc_block_t* b) {
  if (validate_block(b) != TTC_OK) return 0;
  return block_layout(b->n_tokens, b->H, b->r).total * sizeof(float);
}

ttc_status_t ttc_block_forward(const ttc_block_t* b, const void* x_in, void* x_out, float* h0, float* o, int32_t* info,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t sv = validate_block(b);
  if (sv != TTC_OK) return sv;
  if (b->n_tokens == 0) return TTC_OK;
  const void* ptrs[] = {b->ln_in_gain, b->ln_in_offset, b->W_in, b->b_in, b->W_head, b->b_head, b->W_shared, b->b_shared,
                        b->Bbasis, b->Qc, b->ln_out_gain, b->ln_out_offset, b->W_out, b->b_out, x_in, x_out};
  for (const void* ptr : ptrs)
    if (!ptr || !ttc::aligned_ptr(ptr, 16)) return TTC_ERR_INVALID_ARG;
  if (!ttc::aligned_ptr(h0, 16) || !ttc::aligned_ptr(o, 16)) return TTC_ERR_INVALID_ARG;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_block_workspace_bytes(b))
    return TTC_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const long long M = b->n_tokens;
  const int H = b->H, r = b->r, HD = 16 * b->H;
  const BlockLayout L = block_layout(M, H, r);
  float* ws = static_cast<float*>(workspace);
  float* const h0p = h0 ? h0 : ws + L.h0;
  float* const op = o ? o : ws + L.o;

  // h_0 = W_in LN(x_in) + b_in
  const bool bf16 = (b->flags & TTC_BLOCK_FLAG_BF16) != 0;
  ttc::LnStatsArgs s1{x_in, ws + L.stats_in, M, b->C, b->eps};
  if (ttc::launch_ln_stats(s1, bf16, st) != hipSuccess) return TTC_ERR_DEVICE;
  if (bf16) {
    ttc::GemmLnBf16Args g1{x_in, ws + L.stats_in, b->ln_in_gain, b->ln_in_offset, static_cast<const uint16_t*>(b->W_in),
                           b->b_in, nullptr, h0p, M, HD, b->C};
    if (ttc::launch_gemm_ln_bf16(g1, true, false, st) != hipSuccess) return TTC_ERR_DEVICE;
  } else {
    ttc::GemmLnArgs g1{static_cast<const float*>(x_in), ws + L.stats_in, b->ln_in_gain, b->ln_in_offset,
                       static_cast<const float*>(b->W_in), b->b_in, nullptr, h0p, M, HD, b->C};
    if (ttc::launch_gemm_ln(g1, st) != hipSuccess) return TTC_ERR_DEVICE;
  }
  // the contextualisation maps and the Q basis
  ttc::CxtMapsArgs c;
  c.H0 = h0p;
  c.W_head = b->W_head; c.b_head = b->b_head; c.W_shared = b->W_shared; c.b_shared = b->b_shared;
  c.sA = ws + L.sA; c.rinv = ws + L.rinv; c.lgA = ws + L.lgA; c.lgB = ws + L.lgB; c.lgQ = ws + L.lgQ;
  c.sQf = ws + L.sQf; c.sB = ws + L.sB; c.sQ = ws + L.sQ;
  c.M = M; c.H = H; c.r = r;
  // workgroups per token chunk: one per head, or one per four heads in the coalesced variant (r = 16, H % 4 = 0)
  const int per_chunk = (r == 16 && H % 4 == 0) ? H / 4 : H;
  long long chunks = (8LL * ttc::cu_count() + per_chunk - 1) / per_chunk;  // about eight workgroups per compute unit
  chunks = chunks < 1 ? 1 : chunks > M ? M : chunks;
  c.tokens_per_block = (int)((M + chunks - 1) / chunks);
  chunks = (M + c.tokens_per_block - 1) / c.tokens_per_block;
  if (ttc::launch_cxt_maps(c, (int)(chunks * per_chunk), st) != hipSuccess) return TTC_ERR_DEVICE;
  if (ttc::launch_qbasis(b->Qc, ws + L.qbasis, r, st) != hipSuccess) return TTC_ERR_DEVICE;
  // o = the heads' first optimal controls
  ttc_lqr_cxt_problem_t q;
  q.n = M * H; q.d = 16; q.r = r; q.T = b->T; q.in_dtype = TTC_F32; q.flags = 0;
  q.sA = c.sA; q.sB = c.sB; q.sQ = c.sQ; q.sQf = c.sQf; q.rinv = c.rinv; q.lgA = c.lgA; q.lgB = c.lgB; q.lgQ = c.lgQ;
  q.x0 = h0p; q.Bbasis = b->Bbasis; q.Qbasis = ws + L.qbasis;
  ttc::CxtArgs a;
  fill_cxt_args(a, &q);
  a.s.u0 = op;
  a.s.info = info ? info : reinterpret_cast<int32_t*>(ws + L.info);
  if (run_cxt(a, false, st) != hipSuccess) return TTC_ERR_DEVICE;
  // x_out = x_in + W_out LN(o) + b_out
  ttc::LnStatsArgs s2{op, ws + L.stats_out, M, HD, b->eps};
  if (ttc::launch_ln_stats(s2, false, st) != hipSuccess) return TTC_ERR_DEVICE;
  if (bf16) {
    ttc::GemmLnBf16Args g2{op, ws + L.stats_out, b->ln_out_gain, b->ln_out_offset, static_cast<const uint16_t*>(b->W_out),
                           b->b_out, static_cast<const uint16_t*>(x_in), x_out, M, b->C, HD};
    if (ttc::launch_gemm_ln_bf16(g2, false, true, st) != hipSuccess) return TTC_ERR_DEVICE;
  } else {
    ttc::GemmLnArgs g2{op, ws + L.stats_out, b->ln_out_gain, b->ln_out_offset, static_cast<const float*>(b->W_out),
                       b->b_out, static_cast<const float*>(x_in), static_cast<float*>(x_out), M, b->C, HD};
    if (ttc::launch_gemm_ln(g2, st) != hipSuccess) return TTC_ERR_DEVICE;
  }
  return TTC_OK;
}

size_t ttc_lqr_cxt_rollout_workspace_bytes(const ttc_lqr_cxt_problem_t* q) {
  if (!q || q->n < 0 || q->T < 1 || q->d != 16) return 0;
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
  if (run_cxt(ra.c, bf16, st) != hipSuccess) return TTC_ERR_DEVICE;  // backward sweep: gains into the workspace
  const long long groups = (q->n + 3) / 4;
  const long long gb = 32LL * ttc::cu_count();
  const dim3 grid((unsigned)(groups < gb ? groups : gb));
  return ttc::launch_rollout_cxt_forward(ra, bf16, grid, st) == hipSuccess ? TTC_OK : TTC_ERR_DEVICE;
}

// ---- backward pass -------------------------------------------------------------------------------------------
static size_t backward_ws_bytes(int d, int T, bool bf16) {
  const size_t slots = (size_t)ttc::grid_blocks(ttc::KIND_BACKWARD, d, bf16);
  return slots * ((size_t)(T - 1) * d * d + 6 * (size_t)(T + 1) * d) * sizeof(float);
}

size_t ttc_lqr_backward_workspace_bytes(const ttc_lqr_problem_t* q) {
  if (!q || q->T < 1 || !ttc::shape_supported(q)) return 0;
  return backward_ws_bytes(q->d, q->T, q->in_dtype == TTC_BF16);
}

size_t ttc_lqr_backward_tv_workspace_bytes(const ttc_lqr_tv_problem_t* q) {
  if (!q || q->T < 1 || !ttc::shape_supported_dm(q->d, q->m)) return 0;
  return backward_ws_bytes(q->d, q->T, q->in_dtype == TTC_BF16);
}

static ttc_status_t check_grads(const float* grad_u0, const ttc_lqr_grads_t* gr) {
  if (!grad_u0 || !gr || !gr->gA || !gr->gB || !gr->gQ || !gr->gR || !gr->gx0) return TTC_ERR_INVALID_ARG;
  const void* ptrs[] = {gr->gA, gr->gB, gr->gQ, gr->gR, gr->gQT};
  for (const void* ptr : ptrs)
    if (!ttc::aligned_ptr(ptr, 16)) return TTC_ERR_INVALID_ARG;
  return TTC_OK;
}

ttc_status_t ttc_lqr_backward(const ttc_lqr_problem_t* q, const float* grad_u0, const ttc_lqr_grads_t* gr,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t st = ttc::validate(q);
  if (st != TTC_OK) return st;
  if (q->flags != 0) return TTC_ERR_INVALID_ARG;
  if (q->n == 0) return TTC_OK;
  const ttc_status_t sg = check_grads(grad_u0, gr);
  if (sg != TTC_OK) return sg;
  if ((q->QT != nullptr) != (gr->gQT != nullptr)) return TTC_ERR_INVALID_ARG;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_lqr_backward_workspace_bytes(q))
    return TTC_ERR_WORKSPACE;
  ttc::BackwardArgs a;
  a.r.n = q->n; a.r.T = q->T; a.r.flags = 0;
  a.r.A = q->A; a.r.B = q->B; a.r.Q = q->Q; a.r.R = q->R; a.r.QT = q->QT; a.r.x0 = q->x0;
  a.r.sA = q->sA; a.r.sB = q->sB; a.r.sQ = q->sQ; a.r.sR = q->sR; a.r.sQT = q->sQT; a.r.sx0 = q->sx0;
  a.r.U = a.r.X = a.r.cost = nullptr;
  a.r.info = gr->info;
  a.r.ws = static_cast<float*>(workspace);
  a.tA = a.tB = a.tQ = a.tR = 0;
  a.g = grad_u0; a.sg = q->m;
  a.gA = gr->gA; a.gB = gr->gB; a.gQ = gr->gQ; a.gR = gr->gR; a.gQT = gr->gQT; a.gx0 = gr->gx0;
  a.sum_steps = 1;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const long long gb = ttc::grid_blocks(ttc::KIND_BACKWARD, q->d, bf16);
  const dim3 grid((unsigned)(q->n < gb ? q->n : gb));
  return ttc::run_backward(a, q->d, bf16, grid, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TTC_OK
                                                                                                     : TTC_ERR_DEVICE;
}

ttc_status_t ttc_lqr_backward_tv(const ttc_lqr_tv_problem_t* q, const float* grad_u0, const ttc_lqr_grads_t* gr,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t st = validate_tv(q);
  if (st != TTC_OK) return st;
  if (q->n == 0) return TTC_OK;
  const ttc_status_t sg = check_grads(grad_u0, gr);
  if (sg != TTC_OK) return sg;
  if (gr->gQT) return TTC_ERR_INVALID_ARG;  // the terminal cost is Q of the last step here
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_lqr_backward_tv_workspace_bytes(q))
    return TTC_ERR_WORKSPACE;
  ttc::BackwardArgs a;
  a.r.n = q->n; a.r.T = q->T; a.r.flags = 0;
  a.r.A = q->A; a.r.B = q->B; a.r.Q = q->Q; a.r.R = q->R; a.r.QT = nullptr; a.r.x0 = q->x0;
  a.r.sA = q->sA; a.r.sB = q->sB; a.r.sQ = q->sQ; a.r.sR = q->sR; a.r.sQT = 0; a.r.sx0 = q->sx0;
  a.r.U = a.r.X = a.r.cost = nullptr;
  a.r.info = gr->info;
  a.r.ws = static_cast<float*>(workspace);
  a.tA = q->tA; a.tB = q->tB; a.tQ = q->tQ; a.tR = q->tR;
  a.g = grad_u0; a.sg = q->m;
  a.gA = gr->gA; a.gB = gr->gB; a.gQ = gr->gQ; a.gR = gr->gR; a.gQT = nullptr; a.gx0 = gr->gx0;
  a.sum_steps = 0;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const long long gb = ttc::grid_blocks(ttc::KIND_BACKWARD, q->d, bf16);
  const dim3 grid((unsigned)(q->n < gb ? q->n : gb));
  return ttc::run_backward(a, q->d, bf16, grid, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? TTC_OK
                                                                                                     : TTC_ERR_DEVICE;
}

// ---- backward pass of the structured problems ------------------------------------------------------------------
namespace {
// floats of workspace per problem of a chunk: T + 4 matrices left by the solve kernel, four trajectories of T + 1
// vectors, three matrices kept for the bases' sums, one int
size_t cxt_bwd_floats_per_problem(int T) { return (size_t)(T + 4) * 256 + 4 * (size_t)(T + 1) * 16 + 768 + 1; }
// problems per chunk: about 1 GiB of workspace
long long cxt_bwd_chunk(long long n, int T) {
  long long ch = (long long)((1ull << 28) / cxt_bwd_floats_per_problem(T));
  ch = ch < 256 ? 256 : ch;
  return n < ch ? n : ch;
}
}  // namespace

size_t ttc_lqr_backward_cxt_workspace_bytes(const ttc_lqr_cxt_problem_t* q) {
  if (!q || q->n < 0 || q->T < 1 || q->d != 16) return 0;
  const size_t chunk = (size_t)cxt_bwd_chunk(q->n, q->T);
  return round64(chunk * cxt_bwd_floats_per_problem(q->T)) * sizeof(float);
}

ttc_status_t ttc_lqr_backward_cxt(const ttc_lqr_cxt_problem_t* q, const float* grad_u0, const ttc_lqr_cxt_grads_t* gr,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  const ttc_status_t sv = validate_cxt(q);
  if (sv != TTC_OK) return sv;
  if (!gr || !gr->gBbasis || !gr->gQbasis) return TTC_ERR_INVALID_ARG;
  float* const outs[] = {gr->gsA, gr->gsB, gr->gsQ, gr->gsQf, gr->grinv, gr->glgA, gr->glgB, gr->glgQ, gr->gx0,
                         gr->gBbasis, gr->gQbasis};
  for (const float* ptr : outs)
    if ((q->n > 0 && !ptr) || !ttc::aligned_ptr(ptr, 4)) return TTC_ERR_INVALID_ARG;  // an empty batch has no per-problem arrays
  if (q->n > 0 && !grad_u0) return TTC_ERR_INVALID_ARG;
  // the kernels read the bases' rows with 16-byte (float32) or 8-byte (bfloat16) loads
  if (q->n > 0 && (!ttc::aligned_ptr(q->Bbasis, 16) || !ttc::aligned_ptr(q->Qbasis, 16))) return TTC_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // the sums over the problems start from zero (a fill kernel: also safe under stream capture)
  if (ttc::launch_zero_floats(gr->gBbasis, (long long)q->r * 256, st) != hipSuccess) return TTC_ERR_DEVICE;
  if (ttc::launch_zero_floats(gr->gQbasis, (long long)q->r * 256, st) != hipSuccess) return TTC_ERR_DEVICE;
  if (q->n == 0) return TTC_OK;
  if (!workspace || !ttc::aligned_ptr(workspace, 16) || workspace_bytes < ttc_lqr_backward_cxt_workspace_bytes(q))
    return TTC_ERR_WORKSPACE;
  const int T = q->T;
  const bool bf16 = q->in_dtype == TTC_BF16;
  const size_t esz = bf16 ? 2 : 4;
  const long long chunk = cxt_bwd_chunk(q->n, T);
  float* ws = static_cast<float*>(workspace);
  ttc::CxtBackwardArgs a;
  fill_cxt_args(a.c, q);
  a.roll = ws;
  a.traj = a.roll + (size_t)chunk * (T + 4) * 256;
  a.keep = a.traj + (size_t)chunk * 4 * (T + 1) * 16;
  int* const info_ws = reinterpret_cast<int*>(a.keep + (size_t)chunk * 768);  // the chunk's info when the caller wants none
  a.g = grad_u0;
  a.gsA = gr->gsA; a.gsB = gr->gsB; a.gsQ = gr->gsQ; a.gsQf = gr->gsQf; a.grinv = gr->grinv;
  a.glgA = gr->glgA; a.glgB = gr->glgB; a.glgQ = gr->glgQ; a.gx0 = gr->gx0;
  a.gBbasis = gr->gBbasis; a.gQbasis = gr->gQbasis;
  const long long vgrid = 4LL * ttc::cu_count();  // workgroups of the vector kernel: four wavefronts, four problems at a time each
  a.traj_in_lds = T <= 8;         // the kernel's LDS holds T + 1 <= 9 points of four trajectories per problem
  a.basis_in_lds = q->r <= 16;    // and two groups of up to sixteen basis matrices
  auto shifted = [&](const void* base, long long elems) {
    return static_cast<const void*>(static_cast<const char*>(base) + (size_t)elems * esz);
  };
  for (long long first = 0; first < q->n; first += chunk) {
    a.first = first;
    a.count = q->n - first < chunk ? q->n - first : chunk;
    // the backward recursion on the chunk's problems (their inputs start at `first`), keeping what the sweep below needs
    ttc::CxtArgs sc = a.c;
    sc.s.n = a.count;
    sc.s.x0 = shifted(q->x0, first * 16);
    sc.sA = shifted(q->sA, first * 16); sc.rinv = shifted(q->rinv, first * 16);
    sc.lgA = shifted(q->lgA, first * 16); sc.lgB = shifted(q->lgB, first * 16); sc.lgQ = shifted(q->lgQ, first * 16);
    sc.sB = shifted(q->sB, first * q->r); sc.sQ = shifted(q->sQ, first * q->r); sc.sQf = shifted(q->sQf, first * q->r);
    sc.roll_ws = a.roll;
    sc.roll_slots = T + 4;
    sc.dual_g = grad_u0 + first * 16;
    sc.s.info = gr->info ? gr->info + first : info_ws;
    a.info = gr->info ? gr->info : info_ws - first;  // indexed by the problem's number in the batch
    if (run_cxt(sc, bf16, st) != hipSuccess) return TTC_ERR_DEVICE;
    const long long groups = (a.count + 15) / 16;  // workgroups' worth of problems
    // slabs of the basis sums: four workgroups per compute unit when the chunk is large, never under the smallest slab
    const long long slab = (a.count + 4LL * ttc::cu_count() - 1) / (4LL * ttc::cu_count());
    a.basis_slab = (int)(slab < ttc::CXT_BASIS_SLAB ? ttc::CXT_BASIS_SLAB : slab > 4096 ? 4096 : slab);
    if (ttc::launch_cxt_backward_vec(a, bf16, dim3((unsigned)(groups < vgrid ? groups : vgrid)), st) != hipSuccess)
      return TTC_ERR_DEVICE;
    if (ttc::launch_cxt_basis(a, bf16, st) != hipSuccess) return TTC_ERR_DEVICE;
  }
  return TTC_OK;
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
