"""CPU float64 oracle for the finite-horizon LQR solved by the Test-Time Control layer.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the HIP path is
checked against.  It shares no code with the GPU library, never imports it, and must not
be called from the product path (only from tests, the smoke check and the cpu_baseline
leg of the benchmark).

What it computes is the plain definition the paper gives for the layer's output: the
backward Riccati recursion of Prop. 3.1 (Eq. "riccati" for P_t, Eq. "decode" for K_t) and
the closed-loop roll-out of Alg. 1, with no affine cost term (r_t = 0).  The symplectic
iteration of Thm 3.3 is an identity for the same quantity, so the recursion written out
below *is* the reference result; nothing is blocked, fused or reordered.

Notation bridge (paper -> this file).  The paper indexes h_0 (initial state), controls
u_1..u_T and dynamics h_t = A_t h_{t-1} + B_t u_t.  Here the arguments are time-invariant
(A_t = A, B_t = B, R_t = R, Q_t = Q for 1 <= t <= T-1, terminal Q_T) and the outputs are
named after the textbook convention used by the library boundary:

    x0    = h_0                       u0 = u_1^*            K0 = K_1^*
    P[t]  = P_t for t = 0..T          (P[T] = Q_T, P[1] is the paper's P_1)
    P0    = P[0]: the paper never writes P_0 in Riccati form; it is Y_1^{-1} Y_2 of
            Alg. 4 (lambda_0 = P_0 h_0), i.e. one more Riccati step from P_1 with the
            paper's Q_0 = 0 (Sec. 3.1, Thm A.3).  stage_cost_at_x0=True uses Q_0 = Q.
    value = x0^T P0 x0  (twice the paper's objective, which carries a factor 1/2).

All functions accept either one problem (A: (d,d), x0: (d,)) or a stack of problems
(A: (n,d,d), x0: (n,d)); everything is evaluated in float64.

Time-heterogeneous problems (the general statement of Prop. 3.1, with A_t, B_t, Q_t, R_t varying over
the horizon) have their own entry points, riccati_solve_tv / riccati_rollout_tv, below.  The structured,
contextualised parameters of Sec. 4 (diagonal A_t and R_t, B_t and Q_t from shared bases with exponential
time modulation) are expanded to dense steps by contextual_parameters and solved by contextual_solve
(pins: tests/test_oracle_pins_contextual.py: an expansion worked out by hand, ratio properties, a scalar
problem by hand, the time-invariant problem when nothing is modulated, the stacked KKT system).

Pins (tests/test_oracle_pins.py): scalar closed form (Fibonacci ratios), T=1 closed form,
decoupled diagonal problems, brute-force stacked KKT system (Thm A.6's matrix form) and
condensed QP on tiny instances, value == rolled-out cost, DARE fixed point as T grows,
symmetry/PSD of every P_t, the f64 symplectic product of Thm 3.3.  The paper prints no
worked numeric example, so parity against printed values is unpinned.
"""
from __future__ import annotations

import numpy as np


def _t(M):
    """Transpose of the last two axes."""
    return np.swapaxes(M, -1, -2)


def _sym(M):
    return 0.5 * (M + _t(M))


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def _chol_solve(S, Rhs):
    """S^{-1} Rhs for symmetric positive-definite S via Cholesky (raises LinAlgError if not PD)."""
    L = np.linalg.cholesky(S)
    Y = np.linalg.solve(L, Rhs)
    return np.linalg.solve(_t(L), Y)


def riccati_value_matrices(A, B, Q, R, QT, T):
    """Value matrices P[1..T] and gains K[0..T-1] of Prop. 3.1.

    P[T] = Q_T;  P[t] = Q + A^T P[t+1] A - (B^T P[t+1] A)^T (R + B^T P[t+1] B)^{-1} (B^T P[t+1] A)
    for t = T-1..1 (Eq. "riccati"), K[t] = -(R + B^T P[t+1] B)^{-1} B^T P[t+1] A for
    t = 0..T-1 (Eq. "decode"; K[t] multiplies the state x_t and is the paper's K_{t+1}).

    Returns (P, K): lists indexed by t; P[0] is left as None here (see riccati_solve).
    """
    A, B, Q, R = _f64(A), _f64(B), _sym(_f64(Q)), _sym(_f64(R))
    QT = Q if QT is None else _sym(_f64(QT))
    if T < 1:
        raise ValueError("horizon T must be >= 1")
    P = [None] * (T + 1)
    K = [None] * T
    P[T] = QT
    for t in range(T - 1, -1, -1):
        Pn = P[t + 1]
        BtP = _t(B) @ Pn
        S = R + BtP @ B
        F = BtP @ A                      # B^T P A
        W = _chol_solve(S, F)            # S^{-1} B^T P A
        K[t] = -W
        if t >= 1:
            P[t] = _sym(Q + _t(A) @ Pn @ A - _t(F) @ W)
    return P, K


def riccati_solve(A, B, Q, R, QT, x0, T, stage_cost_at_x0=False):
    """First-step solution of the LQR of Eq. "ttc": P0, K0, u0 and value.

    P0 = Q_0 + A^T P_1 A - (B^T P_1 A)^T (R + B^T P_1 B)^{-1} (B^T P_1 A) with Q_0 = 0
    (paper) or Q_0 = Q (stage_cost_at_x0); K0 = K_1^* of Eq. "decode"; u0 = K0 x0;
    value = x0^T P0 x0.
    """
    A, B = _f64(A), _f64(B)
    Qs = _sym(_f64(Q))
    x0 = _f64(x0)
    P, K = riccati_value_matrices(A, B, Q, R, QT, T)
    P1 = P[1]
    F = _t(B) @ P1 @ A
    P0 = _t(A) @ P1 @ A + _t(F) @ K[0]   # K[0] = -S^{-1} F
    if stage_cost_at_x0:
        P0 = P0 + Qs
    P0 = _sym(P0)
    u0 = (K[0] @ x0[..., None])[..., 0]
    value = np.einsum("...i,...ij,...j->...", x0, P0, x0)
    return {"P0": P0, "K0": K[0], "u0": u0, "value": value, "P": P, "K": K}


def riccati_rollout(A, B, Q, R, QT, x0, T, stage_cost_at_x0=False):
    """Closed-loop roll-out of Alg. 1 (forward loop) with r = 0.

    x_0 = x0; u_t = K[t] x_t; x_{t+1} = A x_t + B u_t for t = 0..T-1.
    cost = [x0^T Q x0 if stage_cost_at_x0] + sum_t u_t^T R u_t + sum_{t=1}^{T-1} x_t^T Q x_t
           + x_T^T Q_T x_T   (Eq. "ttc" without its factor 1/2).

    Returns U (..., T, m), X (..., T+1, d), cost (...).
    """
    A, B = _f64(A), _f64(B)
    Qs, Rs = _sym(_f64(Q)), _sym(_f64(R))
    QTs = Qs if QT is None else _sym(_f64(QT))
    x = _f64(x0)
    _, K = riccati_value_matrices(A, B, Q, R, QT, T)
    quad = lambda v, M: np.einsum("...i,...ij,...j->...", v, M, v)
    cost = quad(x, Qs) if stage_cost_at_x0 else np.zeros(x.shape[:-1])
    X, U = [x], []
    for t in range(T):
        u = (K[t] @ x[..., None])[..., 0]
        x = (A @ x[..., None])[..., 0] + (B @ u[..., None])[..., 0]
        cost = cost + quad(u, Rs) + quad(x, QTs if t == T - 1 else Qs)
        U.append(u)
        X.append(x)
    return np.stack(U, axis=-2), np.stack(X, axis=-2), cost


# ------------------------------------------------------------------------------------------------
# Time-heterogeneous parameters: the statement of Prop. 3.1 as printed, with A_t, B_t, Q_t, R_t.
#
# Arrays carry a step axis of length T in front of the matrix axes.  Step s = 0..T-1 is the paper's
# t = s+1:   x_{s+1} = A[s] x_s + B[s] u_s,   cost  sum_s ( u_s^T R[s] u_s + x_{s+1}^T Q[s] x_{s+1} ),
# i.e. Q[s] = Q_{s+1} is charged on the state the step arrives at, Q[T-1] = Q_T is the terminal cost,
# and nothing is charged on x_0 (the paper's Q_0 = 0).


def riccati_value_matrices_tv(A, B, Q, R):
    """P[0..T] and K[0..T-1] for (..., T, d, d)-shaped A, Q, (..., T, d, m) B and (..., T, m, m) R.

    P[T] = Q[T-1];  for s = T-1..0 with Pn = P[s+1]:
        S = R[s] + B[s]^T Pn B[s],  K[s] = -S^{-1} B[s]^T Pn A[s]                       (Eq. "decode")
        P[s] = Qprev + A[s]^T Pn A[s] - (B[s]^T Pn A[s])^T S^{-1} (B[s]^T Pn A[s])      (Eq. "riccati")
    where Qprev = Q[s-1] is the cost on x_s (zero for s = 0).
    """
    A, B, Q, R = _f64(A), _f64(B), _sym(_f64(Q)), _sym(_f64(R))
    T = A.shape[-3]
    if T < 1 or B.shape[-3] != T or Q.shape[-3] != T or R.shape[-3] != T:
        raise ValueError("A, B, Q, R must share a step axis of length T >= 1")
    P = [None] * (T + 1)
    K = [None] * T
    P[T] = Q[..., T - 1, :, :]
    for s in range(T - 1, -1, -1):
        As, Bs, Rs, Pn = A[..., s, :, :], B[..., s, :, :], R[..., s, :, :], P[s + 1]
        BtP = _t(Bs) @ Pn
        S = Rs + BtP @ Bs
        F = BtP @ As
        W = _chol_solve(S, F)
        K[s] = -W
        Ps = _t(As) @ Pn @ As - _t(F) @ W
        if s >= 1:
            Ps = Ps + Q[..., s - 1, :, :]
        P[s] = _sym(Ps)
    return P, K


def riccati_solve_tv(A, B, Q, R, x0):
    """P0, K0, u0 = K0 x0 and value = x0^T P0 x0 of the time-heterogeneous problem."""
    x0 = _f64(x0)
    P, K = riccati_value_matrices_tv(A, B, Q, R)
    u0 = (K[0] @ x0[..., None])[..., 0]
    value = np.einsum("...i,...ij,...j->...", x0, P[0], x0)
    return {"P0": P[0], "K0": K[0], "u0": u0, "value": value, "P": P, "K": K}


def riccati_rollout_tv(A, B, Q, R, x0):
    """Closed-loop roll-out: U (..., T, m), X (..., T+1, d) and the accumulated cost."""
    A, B, Qs, Rs = _f64(A), _f64(B), _sym(_f64(Q)), _sym(_f64(R))
    T = A.shape[-3]
    x = _f64(x0)
    _, K = riccati_value_matrices_tv(A, B, Q, R)
    quad = lambda v, M: np.einsum("...i,...ij,...j->...", v, M, v)
    cost = np.zeros(x.shape[:-1])
    X, U = [x], []
    for s in range(T):
        u = (K[s] @ x[..., None])[..., 0]
        x = (A[..., s, :, :] @ x[..., None])[..., 0] + (B[..., s, :, :] @ u[..., None])[..., 0]
        cost = cost + quad(u, Rs[..., s, :, :]) + quad(x, Qs[..., s, :, :])
        U.append(u)
        X.append(x)
    return np.stack(U, axis=-2), np.stack(X, axis=-2), cost


# ------------------------------------------------------------------------------------------------------
# Contextualised, structured parameters (Sec. 4, "Contextualization" and "Parameterization"; Sec. 3.3,
# "Structured Parameterization"): the T steps of one problem are synthesised from a few per-problem
# vectors and two shared groups of basis matrices,
#     Gamma_X^t = diag(exp(-t * lg_X)),  X in {A, B, Q},                 t = 1..T
#     A_t = I + Gamma_A^t diag(s_A)                       (diagonal)
#     B_t = (sum_i s_B[i] Bbasis[i]) Gamma_B^t            (columns scaled)
#     Q_t = Gamma_Q^t (sum_i s_Q[i] Qbasis[i]) Gamma_Q^t  for t < T,   Q_T = sum_i s_Qf[i] Qbasis[i]
#     R_t = diag(1 / rinv)                                (the layer hands over the diagonal of R^{-1})
# Step s of the arrays below is the paper's t = s + 1.

def contextual_parameters(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, T):
    """Dense A, B, Q, R of shape (..., T, d, d) from the structured inputs.

    sA, rinv, lgA, lgB, lgQ: (..., d);  sB, sQ, sQf: (..., r);  Bbasis, Qbasis: (r, d, d), shared.
    """
    sA, sB, sQ, sQf, rinv = _f64(sA), _f64(sB), _f64(sQ), _f64(sQf), _f64(rinv)
    lgA, lgB, lgQ, Bbasis, Qbasis = _f64(lgA), _f64(lgB), _f64(lgQ), _f64(Bbasis), _f64(Qbasis)
    d = sA.shape[-1]
    eye = np.eye(d)
    Bbar = np.einsum("...i,ijk->...jk", sB, Bbasis)
    Qbar = np.einsum("...i,ijk->...jk", sQ, Qbasis)
    Qf = np.einsum("...i,ijk->...jk", sQf, Qbasis)
    As, Bs, Qs, Rs = [], [], [], []
    for t in range(1, T + 1):
        gA, gB, gQ = np.exp(-t * lgA), np.exp(-t * lgB), np.exp(-t * lgQ)
        As.append(eye + (gA * sA)[..., :, None] * eye)
        Bs.append(Bbar * gB[..., None, :])
        Qs.append(Qf if t == T else gQ[..., :, None] * Qbar * gQ[..., None, :])
        Rs.append((1.0 / rinv)[..., :, None] * eye)
    stack = lambda Ms: np.stack(Ms, axis=-3)
    return stack(As), stack(Bs), stack(Qs), stack(Rs)


def contextual_solve(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T):
    """P0, K0, u0, value of the problem whose steps are contextual_parameters(...)."""
    A, B, Q, R = contextual_parameters(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, T)
    return riccati_solve_tv(A, B, Q, R, x0)


def contextual_rollout(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T):
    """Closed-loop roll-out (U, X, cost) of the problem whose steps are contextual_parameters(...)."""
    A, B, Q, R = contextual_parameters(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, T)
    return riccati_rollout_tv(A, B, Q, R, x0)
