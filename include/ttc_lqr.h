/*
 * ttc_lqr.h -- C ABI of the batched finite-horizon LQR solver behind a Test-Time Control (TTC) layer.
 *
 * One independent LQR problem per (batch, head, token), n problems per call.  Each problem is the
 * paper's Eq. "ttc" (Sec. 3.1; formal statement: Def. A.1) with time-invariant parameters (the
 * paper's "Homo." setting): dynamics x_{t+1} = A x_t + B u_t, stage costs x_t^T Q x_t (1 <= t <= T-1)
 * and u_t^T R u_t (0 <= t <= T-1), terminal cost x_T^T Q_T x_T, no cost on the initial state
 * (the paper's Q_0 = 0).  Textbook indexing is used here: x0 = h_0, u0 = u_1^*, K0 = K_1^*.
 *
 * The solve runs the backward Riccati recursion (Prop. 3.1) through the reverse symplectic
 * iteration of Thm 3.3: the pair [Y1 Y2] is multiplied by the factored symplectic matrices
 * Sigma_t (App. C "Kernel Fusion") and P = Y1^{-1} Y2 is recovered by a pivoted dense solve.
 * Because cond(Y1) grows geometrically with the number of accumulated factors, the T factors are
 * applied in groups and the pair is re-based to [I P] after each group: rebase_every = k asks for
 * ceil(T/k) groups of nearly equal length (the paper's algorithm is one group, rebase_every >= T).
 * A growth guard watches max |Y1| inside every group (Y1 starts a group as the identity): a group that
 * is about to pass the limit is ended early, and a problem whose pair has passed it is solved instead
 * by the recursion of Prop. 3.1 in its printed form (one positive definite solve per step, as
 * ttc_lqr_solve_tv does), inside the same launch.  The accuracy therefore does not depend on the inputs
 * resembling those the default grouping was measured on; what remains is float32 itself: with state
 * costs some 1e4 times the control costs P0 is a small difference of large terms and every float32
 * evaluation of the recursion loses digits in proportion.
 *
 * Conventions
 *   - All matrix arguments are DEVICE pointers to row-major, problem-major arrays: problem p of A
 *     starts at A + p*sA elements.  A stride of 0 shares one matrix between all problems.
 *   - Inputs are borrowed and read-only; outputs and the workspace are caller-owned.  The library
 *     never allocates device memory, never synchronises the stream, and launches asynchronously on
 *     the HIP stream passed as `hip_stream` (a hipStream_t cast to void*; NULL = default stream).
 *   - Q, R and Q_T are read as their symmetric parts (M + M^T)/2.  R must be positive definite and
 *     A invertible (the paper's parameterisation A = I + ... guarantees it, Sec. 4).
 *   - Inputs may be float32 or bfloat16 (in_dtype); every on-chip quantity and every output is
 *     float32 (App. C "Mixed Precision").
 *   - Supported shapes: d = m in {16, 32, 64, 128}, T >= 1.  Anything else returns
 *     TTC_ERR_UNSUPPORTED and launches nothing.  Pointers of float32 inputs/outputs must be 16-byte
 *     aligned (8-byte for bfloat16 inputs) and strides multiples of 4 elements, else
 *     TTC_ERR_INVALID_ARG.
 *   - Argument errors are reported by the return code and nothing is launched.  Numerical breakdown
 *     (a zero or non-finite pivot: R not positive definite, singular A, singular Y1) is reported
 *     per problem in info[] and that problem's outputs are NaN; the call still returns TTC_OK.
 */
#ifndef TTC_LQR_H
#define TTC_LQR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TTC_OK = 0,
  TTC_ERR_INVALID_ARG = 1, /* NULL/misaligned pointer, n < 0, T < 1, bad stride or enum value   */
  TTC_ERR_UNSUPPORTED = 2, /* shape outside the supported set                                    */
  TTC_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than ttc_lqr_workspace_bytes()           */
  TTC_ERR_DEVICE = 4       /* the HIP runtime refused the launch (no device, bad stream, ...)    */
} ttc_status_t;

typedef enum { TTC_F32 = 0, TTC_BF16 = 1 } ttc_dtype_t;

enum {
  /* P0 += Q: charge the stage cost on x0 as textbooks do.  Default 0 is the paper's Q_0 = 0
   * (Sec. 3.1, Thm A.3).  K0 and u0 do not depend on it. */
  TTC_FLAG_STAGE_COST_AT_X0 = 1,
  /* Never re-base inside the horizon: accumulate all T factors Sigma_T..Sigma_1 with row
   * normalisation after every step (App. C "Numerical Stability") and do the dense solve once,
   * as Alg. 4 does, without the growth guard.  For study: accuracy degrades quickly with T on dense
   * problems. */
  TTC_FLAG_PURE_SYMPLECTIC = 2,
  /* Long-horizon path (ttc_lqr_solve only): the parameters are time-invariant (the paper's "Homo."
   * setting), so the T factors of Thm 3.3 are T copies of one matrix and their product (Sec. 3.3)
   * is formed by repeated squaring, about log2(T) dense solves instead of one per group of factors.
   * Each factor is held as the triple (A_e, G_e, H_e) of the map P -> H_e + A_e^T P (I + G_e P)^{-1} A_e
   * (Prop. 3.1 in that form), which composes without A^{-1} and needs no re-basing.  Same outputs and
   * tolerances; rebase_every is ignored; cannot be combined with TTC_FLAG_PURE_SYMPLECTIC.
   * info: 1 = R^{-1}B^T, then every dense solve in program order, the last one being the final step. */
  TTC_FLAG_DOUBLING = 4
};

/* Problem statement: the (A, B, Q, R, Q_T, x0, T) of Eq. "ttc" for n problems. */
typedef struct {
  int64_t n;            /* number of problems (batch*heads*tokens), n >= 0                        */
  int32_t d, m, T;      /* state size, control size, horizon                                       */
  int32_t in_dtype;     /* ttc_dtype_t of A, B, Q, R, QT, x0                                       */
  int32_t flags;        /* TTC_FLAG_*                                                              */
  int32_t rebase_every; /* at most this many factors between re-bases; 0 = library default         */
  const void *A;        /* (n, d, d)                                                               */
  const void *B;        /* (n, d, m)                                                               */
  const void *Q;        /* (n, d, d)                                                               */
  const void *R;        /* (n, m, m)                                                               */
  const void *QT;       /* (n, d, d) or NULL meaning Q_T = Q                                       */
  const void *x0;       /* (n, d)                                                                  */
  int64_t sA, sB, sQ, sR, sQT, sx0; /* elements between consecutive problems; 0 = shared           */
} ttc_lqr_problem_t;

/* Outputs of ttc_lqr_solve, float32, DEVICE pointers; P0, K0, value and info may be NULL. */
typedef struct {
  float *P0;     /* (n, d, d) value matrix at x0: lambda_0 = P0 x0 (Alg. 4: P = Y1^{-1} Y2)         */
  float *K0;     /* (n, m, d) first gain, Eq. "decode" at t = 1                                     */
  float *u0;     /* (n, m)    first optimal control u0 = K0 x0 (the layer's output o)               */
  float *value;  /* (n)       x0^T P0 x0 = 2x the optimal objective of Eq. "ttc"                    */
  int32_t *info; /* (n)       0 = ok; s > 0 = the s-th dense solve of that problem broke down
                               (1: R^{-1}B^T, 2: A^{-1}, 3..: re-bases in order; the last yields P0;
                               for a problem the growth guard handed to the recursion of Prop. 3.1:
                               2 + the index of the step, counted from the end of the horizon)      */
} ttc_lqr_solution_t;

/* Bytes of device workspace ttc_lqr_solve (for_rollout = 0) or ttc_lqr_rollout (for_rollout = 1)
 * needs for this problem on the current device.  Returns 0 for an unsupported/invalid problem.
 * Depends only on d, m, T, flags and the device's compute-unit count, never on n. */
size_t ttc_lqr_workspace_bytes(const ttc_lqr_problem_t *problem, int for_rollout);

/* Solve n problems: P0, K0, u0, value (Prop. 3.1 via Thm 3.3 / Alg. 4, see the file header).
 * `workspace` is a DEVICE buffer of at least ttc_lqr_workspace_bytes(problem, 0) bytes, 16-byte
 * aligned, used as scratch for the duration of the launch.  Asynchronous on `hip_stream`. */
ttc_status_t ttc_lqr_solve(const ttc_lqr_problem_t *problem, const ttc_lqr_solution_t *solution,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/* ttc_lqr_solve for callers that cannot allocate device memory or pass a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same inputs, outputs, conventions and
 * error behaviour as ttc_lqr_solve; the kernels' workspace (the per-workgroup slots that ttc_lqr_solve takes
 * from the caller) is a fixed array of ttc_lqr_noalloc_scratch_bytes() = 24 MiB inside the library's device
 * image, one copy per GPU, held until the process ends.  The call allocates nothing and frees nothing, on the
 * host or on the device.  A problem whose workspace (ttc_lqr_workspace_bytes(problem, 0)) exceeds the array
 * returns TTC_ERR_WORKSPACE and launches nothing; TTC_FLAG_DOUBLING, whose six slots per workgroup never fit,
 * returns TTC_ERR_UNSUPPORTED.  Every call on a GPU uses that GPU's one array: calls that overlap in time on the
 * same GPU (two streams, two threads) race on it and must be serialised by the caller; consecutive calls on one
 * stream are fine (nothing in the array needs to start at zero or to survive between calls). */
ttc_status_t ttc_lqr_solve_noalloc(const ttc_lqr_problem_t *problem, const ttc_lqr_solution_t *solution,
                                   void *hip_stream);
size_t ttc_lqr_noalloc_scratch_bytes(void);

/* Full optimal trajectory (Alg. 1, forward loop, r = 0): U (n, T, m) controls u_0..u_{T-1},
 * X (n, T+1, d) states x_0..x_T, cost (n) = sum_t u_t^T R u_t + sum_{t=1}^{T-1} x_t^T Q x_t +
 * x_T^T Q_T x_T (+ x_0^T Q x_0 with TTC_FLAG_STAGE_COST_AT_X0), which equals `value` of
 * ttc_lqr_solve.  The gains K_t are produced by a re-based backward sweep and kept in the
 * workspace.  X, cost and info may be NULL.  Same conventions and error behaviour as above. */
ttc_status_t ttc_lqr_rollout(const ttc_lqr_problem_t *problem, float *U, float *X, float *cost,
                             int32_t *info, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/* Time-heterogeneous problem: Eq. "ttc" as the paper states it in general, with A_t, B_t, Q_t, R_t
 * varying over the horizon (Sec. 4 "time-heterogeneous parameterization"; Prop. 3.1 is written for
 * this case).  Step s = 0..T-1 is the paper's t = s+1:
 *     x_{s+1} = A[s] x_s + B[s] u_s,    cost  sum_s ( u_s^T R[s] u_s + x_{s+1}^T Q[s] x_{s+1} ),
 * so Q[s] is charged on the state the step arrives at, Q[T-1] is the terminal cost Q_T and x_0 carries
 * no cost.  Matrix s of problem p of A starts at A + p*sA + s*tA elements (likewise B, Q, R); a step
 * stride of 0 shares one matrix between all steps, a problem stride of 0 between all problems.
 * Same conventions as ttc_lqr_problem_t otherwise (device pointers, row-major, alignment, d = m in
 * {16, 32, 64, 128}, Q and R read as their symmetric parts, R positive definite); A need not be
 * invertible.  flags must be 0. */
typedef struct {
  int64_t n;
  int32_t d, m, T;
  int32_t in_dtype;  /* ttc_dtype_t */
  int32_t flags;     /* 0 */
  const void *A;     /* (n, T, d, d) */
  const void *B;     /* (n, T, d, m) */
  const void *Q;     /* (n, T, d, d) */
  const void *R;     /* (n, T, m, m) */
  const void *x0;    /* (n, d)       */
  int64_t sA, sB, sQ, sR, sx0; /* elements between consecutive problems */
  int64_t tA, tB, tQ, tR;      /* elements between consecutive steps of one problem */
} ttc_lqr_tv_problem_t;

/* P0, K0, u0, value, info of n time-heterogeneous problems (same solution struct and error behaviour
 * as ttc_lqr_solve).  With every factor Sigma_t of Thm 3.3 different, the iteration is re-based after
 * every factor, which is the backward recursion of Prop. 3.1 as printed, one step per factor:
 *     S_s = R[s] + B[s]^T P_{s+1} B[s],  K_s = -S_s^{-1} B[s]^T P_{s+1} A[s]                  (Eq. "decode")
 *     P_s = Q[s-1] + A[s]^T P_{s+1} A[s] - (B[s]^T P_{s+1} A[s])^T S_s^{-1} (B[s]^T P_{s+1} A[s])   (Eq. "riccati")
 * with P_T = Q[T-1] and no Q on x_0.  One dense solve per step, S_s positive definite (no pivoting; a
 * pivot that is not positive is a breakdown): info = T - s for the step s whose solve broke down.
 * No workspace is needed: `workspace` may be NULL. */
ttc_status_t ttc_lqr_solve_tv(const ttc_lqr_tv_problem_t *problem, const ttc_lqr_solution_t *solution,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Roll-out of n time-heterogeneous problems (Alg. 1, forward loop, r = 0): U (n, T, m), X (n, T+1, d) and
 * cost (n) = sum_s u_s^T R[s] u_s + x_{s+1}^T Q[s] x_{s+1}, which equals `value` of ttc_lqr_solve_tv.
 * The gains K_s are produced by the backward sweep of ttc_lqr_solve_tv and kept in the workspace, a DEVICE
 * buffer of at least ttc_lqr_tv_rollout_workspace_bytes(problem) bytes, 16-byte aligned.  X, cost and
 * info may be NULL.  Same conventions and error behaviour as ttc_lqr_rollout. */
size_t ttc_lqr_tv_rollout_workspace_bytes(const ttc_lqr_tv_problem_t *problem);
ttc_status_t ttc_lqr_rollout_tv(const ttc_lqr_tv_problem_t *problem, float *U, float *X, float *cost,
                                int32_t *info, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same outputs as ttc_lqr_solve_tv with the product of the T factors of Thm 3.3 formed pairwise instead
 * of one after the other (the paper's product is sequential, Sec. 3.3; composition of the factors is
 * associative): every step becomes an element (A_s, G_s = B_s R_s^{-1} B_s^T, Q_{s-1}) of the map
 * P -> Q_{s-1} + A_s^T P (I + G_s P)^{-1} A_s, neighbouring elements are composed in ceil(log2 T) rounds of
 * one launch each, and the step s = 0 is taken as printed (Prop. 3.1) to obtain K_0.  For small batches
 * with long horizons, where ttc_lqr_solve_tv leaves most of the chip idle: the rounds run n*T/2, n*T/4, ...
 * compositions side by side.  It does about three times the arithmetic of ttc_lqr_solve_tv and needs a
 * workspace of ttc_lqr_tv_scan_workspace_bytes(problem) = n*T*3*d*d*4 bytes (DEVICE, 16-byte aligned;
 * TTC_ERR_WORKSPACE otherwise).  info is 1 for a problem with a breakdown anywhere (an R[s] that is not
 * positive definite, a singular I + G_1 H_2 in a composition, S_0 not positive definite), outputs NaN.
 * Launches 2 + ceil(log2 T) kernels on hip_stream; allocates nothing; asynchronous. */
size_t ttc_lqr_tv_scan_workspace_bytes(const ttc_lqr_tv_problem_t *problem);
ttc_status_t ttc_lqr_solve_tv_scan(const ttc_lqr_tv_problem_t *problem, const ttc_lqr_solution_t *solution,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Every value matrix and every gain of n time-heterogeneous problems, with the work spread over the horizon as
 * well as over the problems (Prop. 3.1, Eq. "riccati" and Eq. "decode"; the factors of Thm 3.3 composed as in
 * ttc_lqr_solve_tv_scan): after the rounds of pairwise compositions a second pass walks the same tree downwards,
 * applying the composition kept at every right child to the value on its right, ceil(log2 T) rounds of one
 * launch each, after which P_t is known for every t.  For small batches with long horizons whose roll-out or
 * backward pass needs all of them.
 *   P  (n, T, d, d) or NULL: P[:, k] = P_{k+1}, the value matrix after step k + 1 (P[:, T-1] = the terminal cost);
 *                            symmetric parts.
 *   K  (n, T, m, d) or NULL: K[:, s] = K_s, the gain of step s, u_s = K_s x_s (computed from P_{s+1} as n*T one-step
 *                            problems; needs sA = T*tA, sB = T*tB, sR = T*tR, TTC_ERR_UNSUPPORTED otherwise).
 * DEVICE pointers, 16-byte aligned, written; at least one of them.  workspace: DEVICE, 16-byte aligned,
 * ttc_lqr_tv_scan_values_workspace_bytes(problem) bytes (TTC_ERR_WORKSPACE otherwise).  A breakdown (an R[s] that is
 * not positive definite, a singular matrix in a composition) shows as NaN in the matrices it reaches.
 * Launches up to 3 + 2 ceil(log2 T) kernels on hip_stream; allocates nothing; asynchronous. */
size_t ttc_lqr_tv_scan_values_workspace_bytes(const ttc_lqr_tv_problem_t *problem);
ttc_status_t ttc_lqr_tv_scan_values(const ttc_lqr_tv_problem_t *problem, float *P, float *K, void *workspace,
                                    size_t workspace_bytes, void *hip_stream);

/* Structured, contextualised problems (Sec. 4, "Contextualization" and "Parameterization"; Sec. 3.3,
 * "Structured Parameterization"): the T steps of a problem are not stored anywhere; the kernel builds them
 * from per-problem vectors and two groups of r basis matrices shared by all problems.  With t = 1..T the
 * paper's step index (step s = t - 1 of ttc_lqr_solve_tv) and Gamma_X^t = diag(exp(-t * lgX)):
 *     A_t = I + Gamma_A^t diag(sA)                                   (diagonal)
 *     B_t = (sum_i sB[i] Bbasis[i]) Gamma_B^t                        (columns scaled)
 *     Q_t = Gamma_Q^t (sum_i sQ[i] Qbasis[i]) Gamma_Q^t   for t < T
 *     Q_T = sum_i sQf[i] Qbasis[i]                                   (terminal cost, not modulated)
 *     R_t = diag(1 / rinv)                                           (the diagonal of R^{-1} is the input)
 * All pointers are DEVICE pointers, borrowed and read-only, of element type in_dtype, contiguous:
 * sA, rinv, lgA, lgB, lgQ, x0 are (n, d); sB, sQ, sQf are (n, r); Bbasis, Qbasis are (r, d, d) row-major.
 * The problem solved needs rinv > 0 and the combined Q matrices positive semi-definite (they are read as
 * their symmetric parts); lgX >= 0 gives the discounting of the paper, any finite value is accepted.
 * Accuracy: float32 throughout; when control is nearly free (rinv several orders of magnitude above the
 * state costs) P_0 is a small difference of large terms in the recursion of Prop. 3.1 and digits are lost
 * in proportion, as in any float32 evaluation of it. */
typedef struct {
  int64_t n;        /* problems = batch * heads * tokens */
  int32_t d;        /* state = control dimension; 16 is supported */
  int32_t r;        /* basis matrices per group, 1..64 */
  int32_t T;        /* horizon, >= 1 */
  int32_t in_dtype; /* ttc_dtype_t */
  int32_t flags;    /* 0 */
  const void *sA, *sB, *sQ, *sQf, *rinv, *lgA, *lgB, *lgQ, *x0;
  const void *Bbasis, *Qbasis;
} ttc_lqr_cxt_problem_t;

/* P0, K0, u0, value, info of n structured problems: the recursion of ttc_lqr_solve_tv (Prop. 3.1) on the
 * steps defined above, with the same solution struct, conventions (no cost on x_0) and error behaviour;
 * info = T - s for the step whose S_s = R + B^T P B was not positive definite.  Needs no workspace,
 * allocates nothing, is asynchronous on hip_stream.  d other than 16 or r above 64: TTC_ERR_UNSUPPORTED. */
ttc_status_t ttc_lqr_solve_cxt(const ttc_lqr_cxt_problem_t *problem, const ttc_lqr_solution_t *solution,
                               void *hip_stream);

/* Roll-out of n structured problems (Alg. 1, forward loop, r = 0) under the optimal feedback: U (n, T, d),
 * X (n, T+1, d) and cost (n) = sum_t u_t^T R_t u_t + x_t^T Q_t x_t over t = 1..T, which equals `value` of
 * ttc_lqr_solve_cxt.  Two launches: the backward sweep of ttc_lqr_solve_cxt keeping every gain K_t, then the
 * closed loop forward.  The workspace is a DEVICE buffer of at least
 * ttc_lqr_cxt_rollout_workspace_bytes(problem) bytes (n*(T+3)*d*d floats and n flags), 16-byte aligned
 * (TTC_ERR_WORKSPACE otherwise).  X, cost and info may be NULL; info and NaN outputs as for ttc_lqr_solve_cxt. */
size_t ttc_lqr_cxt_rollout_workspace_bytes(const ttc_lqr_cxt_problem_t *problem);
ttc_status_t ttc_lqr_rollout_cxt(const ttc_lqr_cxt_problem_t *problem, float *U, float *X, float *cost,
                                 int32_t *info, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backward pass of the layer (Thm 3.2; appendix: Thm A.6, Alg. 5): gradients of a loss l of the layer's output
 * u0 = u_1^* with respect to the parameters and the initial state, given grad_u0 = dl/du0 (n, m), float32.
 * With (x, u, lam) the states, controls and co-states of the problem itself (the "primal LQR") and (xt, ut, lamt)
 * those of the "dual LQR" (the same dynamics and quadratic costs from the initial state 0, plus the linear cost
 * grad_u0^T ut_0 on the first control), step s = 0..T-1 being the paper's t = s+1:
 *     dl/dA[s] = lam_{s+1} xt_s^T + lamt_{s+1} x_s^T          dl/dB[s] = lam_{s+1} ut_s^T + lamt_{s+1} u_s^T
 *     dl/dQ[s] = (xt_{s+1} x_{s+1}^T + x_{s+1} xt_{s+1}^T)/2    dl/dR[s] = (ut_s u_s^T + u_s ut_s^T)/2
 *     dl/dx0   = lamt_0
 * (Q and R are read as their symmetric parts; their gradients are the symmetric ones of Thm 3.2).  The call is
 * self-contained: it repeats the backward recursion of Prop. 3.1 (keeping the gains of the problems in flight in
 * the workspace), rolls both closed loops forward (Alg. 1) and the co-states backward (Alg. 2), instead of running
 * the forward symplectic recursion of Alg. 5 from cached factors, which loses all accuracy in float32 on dense
 * problems.  All gradient pointers are DEVICE pointers, float32, caller-owned, 16-byte aligned, required (info may
 * be NULL).  info and NaN gradients as for ttc_lqr_solve_tv (info = T - s for the step whose solve broke down). */
typedef struct {
  float *gA, *gB, *gQ, *gR; /* ttc_lqr_backward_tv: (n, T, d, d) per step; ttc_lqr_backward: (n, d, d), summed over steps */
  float *gQT;               /* ttc_lqr_backward only: (n, d, d) gradient of the terminal cost; required exactly when
                               the problem gives QT (then gQ sums the steps before the last); NULL otherwise        */
  float *gx0;               /* (n, d)                                                                              */
  int32_t *info;            /* (n) or NULL                                                                         */
} ttc_lqr_grads_t;

/* Time-invariant parameters (ttc_lqr_problem_t, flags must be 0): every matrix serves in all T steps and collects
 * the sum of the steps' gradients.  Workspace: ttc_lqr_backward_workspace_bytes(problem) bytes, DEVICE, 16-byte
 * aligned (per resident workgroup (T-1) d^2 + 6 (T+1) d floats; independent of n). */
size_t ttc_lqr_backward_workspace_bytes(const ttc_lqr_problem_t *problem);
ttc_status_t ttc_lqr_backward(const ttc_lqr_problem_t *problem, const float *grad_u0, const ttc_lqr_grads_t *grads,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Time-heterogeneous parameters (ttc_lqr_tv_problem_t): one gradient per step and matrix. */
size_t ttc_lqr_backward_tv_workspace_bytes(const ttc_lqr_tv_problem_t *problem);
ttc_status_t ttc_lqr_backward_tv(const ttc_lqr_tv_problem_t *problem, const float *grad_u0,
                                 const ttc_lqr_grads_t *grads, void *workspace, size_t workspace_bytes,
                                 void *hip_stream);

/* Backward pass of the structured, contextualised problems (Thm 3.2 carried on to the parameterisation of Sec. 4,
 * "Contextualization", "Parameterization"): gradients of a loss of u0 = u_1^*, given grad_u0 = dl/du0 (n, 16) float32,
 * with respect to the inputs of ttc_lqr_cxt_problem_t, in the quantities the layer hands over (the log-scale
 * modulation coefficients lgA, lgB, lgQ and rinv, the diagonal of R^{-1}).  All outputs DEVICE, float32, contiguous,
 * written: gsA, grinv, glgA, glgB, glgQ, gx0 (n, 16); gsB, gsQ, gsQf (n, r); gBbasis, gQbasis (r, 16, 16), the sums
 * over all n problems (cleared by the call, then accumulated with atomic additions: their last bits may differ from
 * run to run); info (n) or NULL, as ttc_lqr_backward_tv reports it.  The basis gradients are with respect to the
 * matrices as given (every entry on its own); Qbasis has to be symmetric. */
typedef struct {
  float *gsA, *gsB, *gsQ, *gsQf, *grinv, *glgA, *glgB, *glgQ, *gx0;
  float *gBbasis, *gQbasis;
  int32_t *info;
} ttc_lqr_cxt_grads_t;

/* The problems are taken a chunk at a time, three launches per chunk after two that clear the basis gradients: the
 * backward recursion of the forward pass once more, keeping every gain and the dual problem's first control in the workspace; one sweep
 * of sixteen lanes per problem over both closed loops, both co-state recursions and the gradients, contracted straight
 * onto the parameterisation (no dense per-step matrices are formed); the sums for the bases.  Bbasis and Qbasis have to
 * be 16-byte aligned here (TTC_ERR_INVALID_ARG otherwise).  workspace: DEVICE, 16-byte aligned,
 * ttc_lqr_backward_cxt_workspace_bytes(problem) bytes (about 1 GiB for large batches; TTC_ERR_WORKSPACE otherwise).
 * Allocates nothing; asynchronous on hip_stream. */
size_t ttc_lqr_backward_cxt_workspace_bytes(const ttc_lqr_cxt_problem_t *problem);
ttc_status_t ttc_lqr_backward_cxt(const ttc_lqr_cxt_problem_t *problem, const float *grad_u0,
                                  const ttc_lqr_cxt_grads_t *grads, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/* The whole Test-Time Control block for n_tokens token features, each on its own (Sec. 4, "Hybrid with Memory
 * Layers", "Multi-Head Structure", "Contextualization", "Parameterization"), float32:
 *     h_0   = W_in LN(x_in) + b_in, split into H heads of d = 16 numbers;
 *     per head, from its 16 numbers v:  sA = W_A v + b_A,  rinv = softplus(W_R v + b_R),
 *         lgA, lgB, lgQ = softplus(W_g. v + b_g.),  sQf = softplus(W_Qf v + b_Qf)   (maps of the head's own),
 *         sB = W_B v + b_B,  sQ = softplus(W_Q v + b_Q)                              (maps shared by all heads),
 *         Q^(i) = Qc^(i) Qc^(i)^T / sqrt(d);
 *     o     = side by side, the u_1^* of the heads' structured problems (ttc_lqr_cxt_problem_t with these vectors,
 *             Bbasis, Q^(i), x0 = the head's part of h_0, horizon T);
 *     x_out = x_in + W_out LN(o) + b_out.
 * LN normalises over the last axis (biased variance, eps under the root) and applies a gain and an offset per entry.
 * The structured steps are built in the solve kernel, never stored; the per-problem vectors (80 + 3r floats) are.
 * All weights are DEVICE pointers, float32, contiguous, row-major, borrowed and read-only, 16-byte aligned:
 *   ln_in_gain, ln_in_offset (C);  W_in (H*16, C), b_in (H*16);
 *   W_head (H, 80 + r, 16), b_head (H, 80 + r): rows sA, rinv, lgA, lgB, lgQ (16 each), then sQf (r);
 *   W_shared (2r, 16), b_shared (2r): rows sB (r), then sQ (r);
 *   Bbasis, Qc (r, 16, 16);  ln_out_gain, ln_out_offset (H*16);  W_out (C, H*16), b_out (C).
 * d other than 16, r above 64 or not a multiple of 4, C not a multiple of 4: TTC_ERR_UNSUPPORTED.
 * With TTC_BLOCK_FLAG_BF16 in flags the token features x_in, x_out and the two projection matrices W_in, W_out are
 * bfloat16 (everything else stays float32): the projections then run on the bfloat16 matrix cores with float32
 * accumulation, LN(x) rounded to bfloat16 on the way in; C has to be a multiple of 8. */
#define TTC_BLOCK_FLAG_BF16 1
typedef struct {
  int64_t n_tokens;
  int32_t C;     /* width of a token feature */
  int32_t H;     /* heads */
  int32_t d;     /* state and control size of a head: 16 */
  int32_t r;     /* basis matrices per group */
  int32_t T;     /* horizon, >= 1 */
  int32_t flags; /* 0 or TTC_BLOCK_FLAG_BF16 */
  float eps;     /* of both layer normalisations, > 0 */
  const float *ln_in_gain, *ln_in_offset;
  const void *W_in; /* float32, or bfloat16 with TTC_BLOCK_FLAG_BF16 */
  const float *b_in, *W_head, *b_head, *W_shared, *b_shared, *Bbasis, *Qc, *ln_out_gain, *ln_out_offset;
  const void *W_out; /* as W_in */
  const float *b_out;
} ttc_block_t;

/* x_in (n_tokens, C) DEVICE, read; x_out (n_tokens, C) DEVICE, written, may be x_in itself; float32, or bfloat16 with
 * TTC_BLOCK_FLAG_BF16.  Optional DEVICE float32 outputs
 * (NULL to skip): h0 (n_tokens, H*16); o (n_tokens, H*16); info (n_tokens*H), as ttc_lqr_solve_cxt reports it for
 * the problem of token t, head h at [t*H + h] (a problem that broke down gives NaN in its token's x_out).
 * workspace: DEVICE, 16-byte aligned, ttc_block_workspace_bytes(block) bytes (TTC_ERR_WORKSPACE otherwise; the size
 * depends on n_tokens, H, r only).  Seven launches on hip_stream; allocates nothing; asynchronous. */
size_t ttc_block_workspace_bytes(const ttc_block_t *block);
ttc_status_t ttc_block_forward(const ttc_block_t *block, const void *x_in, void *x_out, float *h0, float *o,
                               int32_t *info, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Static, NUL-terminated description of a status code. */
const char *ttc_status_string(ttc_status_t status);

/* Library version: major*10000 + minor*100 + patch. */
int ttc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TTC_LQR_H */
