"""CPU float64 oracle for the backward pass of the Test-Time Control layer: gradients of a loss of the layer's
output u_1^* with respect to the LQR parameters and the initial state.

TEST INFRASTRUCTURE ONLY, like lqr_oracle.py: slow, plain, never imported by the product path, shares no code
with the HIP library.

What it computes is Thm 3.2 (appendix: Thm A.6) written out.  With o = u_1^* the layer's output and
g = dl/do given, the gradients are outer products of two KKT solutions,
    dl/dA_t = lam_t ht_{t-1}^T + lamt_t h_{t-1}^T        dl/dB_t = lam_t ut_t^T + lamt_t u_t^T
    dl/dQ_t = (ht_t h_t^T + h_t ht_t^T) / 2              dl/dR_t = (ut_t u_t^T + u_t ut_t^T) / 2
    dl/dh_0 = lamt_0
where (h, u, lam) solve the KKT system of the layer's own problem (the "primal LQR", Eq. "ttc") and
(ht, ut, lamt) that of the "dual LQR": the same dynamics and quadratic costs from the initial state 0, plus the
linear cost g^T ut_1 on the first control.  Each KKT solution is obtained in the paper's order: the backward
recursion with the affine terms of Prop. A.1 (P_t, p_t), the forward roll-out of Alg. 1
(u_t = K_t h_{t-1} + k_t), and the co-state recursion of Alg. 2 (lam_T = Q_T h_T, lam_t = Q_t h_t + A_{t+1}^T lam_{t+1},
lam_0 = A_1^T lam_1).  Nothing is fused or reordered.

Indexing (as in lqr_oracle.py's time-heterogeneous functions): arrays carry a step axis s = 0..T-1 = the paper's
t - 1;  x_{s+1} = A[s] x_s + B[s] u_s;  Q[s] is the cost on x_{s+1} (Q[T-1] the terminal cost), R[s] on u_s; no cost
on x_0.  X has T+1 entries (X[0] = x0), U has T, LAM has T+1 (LAM[t] is the paper's lambda_t).
Q and R are read as their symmetric parts, and the gradients with respect to them are symmetric (the derivative
with respect to the symmetric part, which is what Thm 3.2 states).

Pins (tests/test_grad_oracle_pins.py): central finite differences of lqr_oracle.riccati_solve_tv on tiny
instances, the stacked KKT system of the proof of Thm A.6 solved densely (for both trajectories), a scalar
problem differentiated by hand, dl/dh_0 = K_1^T g, and two invariances of the layer (common scaling of all costs;
change of state coordinates) that force linear identities between the gradients; for the structured parameters
(contextual_gradients, at the end of this file) central finite differences of lqr_oracle.contextual_solve in every
input.  The paper prints no numeric example of a gradient: parity against printed values is unpinned.
"""
from __future__ import annotations

import numpy as np


def _t(M):
    return np.swapaxes(M, -1, -2)


def _sym(M):
    return 0.5 * (M + _t(M))


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def _mv(M, v):
    return (M @ v[..., None])[..., 0]


def kkt_solution_tv(A, B, Q, R, x0, r=None):
    """States X (..., T+1, d), controls U (..., T, m) and co-states LAM (..., T+1, d) of the LQR with an optional
    linear control cost sum_s r[s]^T u_s (Prop. A.1, Alg. 1, Alg. 2).

    Backward:  P_T = Q[T-1], p_T = 0;  for s = T-1..0 with Pn = P_{s+1}, pn = p_{s+1}, S = R[s] + B[s]^T Pn B[s]:
        K_s = -S^{-1} B[s]^T Pn A[s],   k_s = -S^{-1} (B[s]^T pn + r[s])
        P_s = Q[s-1] + A[s]^T Pn A[s] - (B[s]^T Pn A[s])^T S^{-1} (B[s]^T Pn A[s])          (no Q for s = 0)
        p_s = A[s]^T pn - A[s]^T Pn B[s] S^{-1} (B[s]^T pn + r[s])
    Forward:   u_s = K_s x_s + k_s,  x_{s+1} = A[s] x_s + B[s] u_s.
    Co-states: lam_T = Q[T-1] x_T,  lam_t = Q[t-1] x_t + A[t]^T lam_{t+1} (t = T-1..1),  lam_0 = A[0]^T lam_1.
    """
    A, B, Q, R, x0 = _f64(A), _f64(B), _sym(_f64(Q)), _sym(_f64(R)), _f64(x0)
    T = A.shape[-3]
    m = B.shape[-1]
    r = np.zeros(x0.shape[:-1] + (T, m)) if r is None else _f64(r)
    K, k = [None] * T, [None] * T
    P = Q[..., T - 1, :, :]
    p = np.zeros_like(x0)
    for s in range(T - 1, -1, -1):
        As, Bs = A[..., s, :, :], B[..., s, :, :]
        S = R[..., s, :, :] + _t(Bs) @ P @ Bs
        F = _t(Bs) @ P @ As
        aff = _mv(_t(Bs), p) + r[..., s, :]
        K[s] = -np.linalg.solve(S, F)
        k[s] = -_mv(np.linalg.inv(S), aff)
        Pnew = _t(As) @ P @ As + _t(F) @ K[s]
        pnew = _mv(_t(As), p) + _mv(_t(F), k[s])
        if s >= 1:
            Pnew = Pnew + Q[..., s - 1, :, :]
        P, p = _sym(Pnew), pnew
    X, U = [x0], []
    for s in range(T):
        u = _mv(K[s], X[s]) + k[s]
        U.append(u)
        X.append(_mv(A[..., s, :, :], X[s]) + _mv(B[..., s, :, :], u))
    LAM = [None] * (T + 1)
    LAM[T] = _mv(Q[..., T - 1, :, :], X[T])
    for t in range(T - 1, 0, -1):
        LAM[t] = _mv(Q[..., t - 1, :, :], X[t]) + _mv(_t(A[..., t, :, :]), LAM[t + 1])
    LAM[0] = _mv(_t(A[..., 0, :, :]), LAM[1])
    return np.stack(X, axis=-2), np.stack(U, axis=-2), np.stack(LAM, axis=-2)


def _outer(a, b):
    return a[..., :, None] * b[..., None, :]


def lqr_gradients_tv(A, B, Q, R, x0, g):
    """Gradients of a loss l(u_0) with dl/du_0 = g (..., m) for time-heterogeneous parameters (Thm 3.2).

    Returns gA, gB, gQ, gR of the shapes of A, B, Q, R (step axis kept) and gx0 (..., d)."""
    A, B = _f64(A), _f64(B)
    g = _f64(g)
    T = A.shape[-3]
    X, U, LAM = kkt_solution_tv(A, B, Q, R, x0)                       # primal LQR
    r = np.zeros(g.shape[:-1] + (T, g.shape[-1]))
    r[..., 0, :] = g                                                  # dual LQR: g^T ut_1, zero initial state
    Xt, Ut, LAMt = kkt_solution_tv(A, B, Q, R, np.zeros_like(_f64(x0)), r)
    gA = np.stack([_outer(LAM[..., s + 1, :], Xt[..., s, :]) + _outer(LAMt[..., s + 1, :], X[..., s, :])
                   for s in range(T)], axis=-3)
    gB = np.stack([_outer(LAM[..., s + 1, :], Ut[..., s, :]) + _outer(LAMt[..., s + 1, :], U[..., s, :])
                   for s in range(T)], axis=-3)
    gQ = np.stack([0.5 * (_outer(Xt[..., s + 1, :], X[..., s + 1, :]) + _outer(X[..., s + 1, :], Xt[..., s + 1, :]))
                   for s in range(T)], axis=-3)
    gR = np.stack([0.5 * (_outer(Ut[..., s, :], U[..., s, :]) + _outer(U[..., s, :], Ut[..., s, :]))
                   for s in range(T)], axis=-3)
    return {"gA": gA, "gB": gB, "gQ": gQ, "gR": gR, "gx0": LAMt[..., 0, :],
            "X": X, "U": U, "LAM": LAM, "Xt": Xt, "Ut": Ut, "LAMt": LAMt}


def lqr_gradients(A, B, Q, R, QT, x0, T, g):
    """The same for time-invariant parameters (A_t = A, B_t = B, R_t = R, Q_t = Q for t < T, terminal Q_T): a
    parameter used in every step collects the sum of that step's gradients.  gQ sums the steps whose state cost is
    Q; gQT is the terminal step's.  With QT None (Q_T = Q) the terminal term is added to gQ and gQT is None."""
    A, B, Q, R = _f64(A), _f64(B), _f64(Q), _f64(R)
    rep = lambda M: np.repeat(M[..., None, :, :], T, axis=-3)
    Qs = rep(Q)
    if QT is not None:
        Qs[..., T - 1, :, :] = _f64(QT)
    tv = lqr_gradients_tv(rep(A), rep(B), Qs, rep(R), x0, g)
    out = {"gA": tv["gA"].sum(axis=-3), "gB": tv["gB"].sum(axis=-3), "gR": tv["gR"].sum(axis=-3), "gx0": tv["gx0"]}
    if QT is None:
        out["gQ"], out["gQT"] = tv["gQ"].sum(axis=-3), None
    else:
        out["gQ"], out["gQT"] = tv["gQ"][..., :T - 1, :, :].sum(axis=-3), tv["gQ"][..., T - 1, :, :]
    return out


# ------------------------------------------------------------------------------------------------------
# Structured, contextualised parameters (Sec. 4, "Contextualization" and "Parameterization"): the gradients of Thm 3.2
# carried on, by the chain rule, to the per-problem vectors and the shared basis matrices the steps are built from
# (lqr_oracle.contextual_parameters), in the quantities the layer hands over: the log-scale modulation
# coefficients lg_X and the diagonal of R^{-1} (Sec. 4, "Parameterization", last sentence).  With t = 1..T and
# gam_X^t = exp(-t lg_X):
#     A_t = I + diag(gam_A^t sA)                  dl/dsA_i  = sum_t gam_A,i^t gA_t[i,i]
#                                                 dl/dlgA_i = sum_t (-t) gam_A,i^t sA_i gA_t[i,i]
#     B_t = Bbar diag(gam_B^t)                    dl/dBbar  = sum_t gB_t diag(gam_B^t)
#                                                 dl/dlgB_j = sum_t (-t) gam_B,j^t sum_i Bbar[i,j] gB_t[i,j]
#     Q_t = diag(gam_Q^t) Qbar diag(gam_Q^t)      dl/dQbar  = sum_{t<T} diag(gam_Q^t) gQ_t diag(gam_Q^t)
#          (t < T)                                dl/dlgQ_i = sum_{t<T} (-t) (row i + column i sums of Q_t o gQ_t)
#     Q_T = Qf                                    dl/dQf    = gQ_T
#     R_t = diag(1 / rinv)                        dl/drinv_i = -sum_t gR_t[i,i] / rinv_i^2
#     Bbar = sum_k sB_k B^(k) etc.                dl/dsB_k = <B^(k), dl/dBbar>,  dl/dB^(k) = sum over problems sB_k dl/dBbar
# and likewise for sQ, sQf and Q^(k).
# Pin (tests/test_grad_oracle_pins.py): central finite differences of lqr_oracle.contextual_solve in every one of these
# inputs on tiny instances.

def contextual_gradients(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T, g):
    """Gradients of a loss l(u_0), dl/du_0 = g (..., d), for the structured problems of lqr_oracle.contextual_solve.

    Returns gsA, grinv, glgA, glgB, glgQ, gx0 (..., d), gsB, gsQ, gsQf (..., r) and, summed over all leading axes,
    gBbasis, gQbasis (r, d, d)."""
    from . import lqr_oracle
    sA, sB, sQ, sQf, rinv = _f64(sA), _f64(sB), _f64(sQ), _f64(sQf), _f64(rinv)
    lgA, lgB, lgQ, Bbasis, Qbasis = _f64(lgA), _f64(lgB), _f64(lgQ), _f64(Bbasis), _f64(Qbasis)
    A, B, Q, R = lqr_oracle.contextual_parameters(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, T)
    dense = lqr_gradients_tv(A, B, Q, R, x0, g)
    gA, gB, gQ, gR = dense["gA"], dense["gB"], dense["gQ"], dense["gR"]
    Bbar = np.einsum("...k,kij->...ij", sB, Bbasis)
    diag = lambda M: np.diagonal(M, axis1=-2, axis2=-1)
    gsA, glgA, glgB, glgQ = (np.zeros_like(sA) for _ in range(4))
    gBbar, gQbar = np.zeros_like(Bbar), np.zeros_like(Bbar)
    for t in range(1, T + 1):
        s = t - 1
        gamA, gamB, gamQ = np.exp(-t * lgA), np.exp(-t * lgB), np.exp(-t * lgQ)
        gsA += gamA * diag(gA[..., s, :, :])
        glgA += -t * gamA * sA * diag(gA[..., s, :, :])
        gBbar += gB[..., s, :, :] * gamB[..., None, :]
        glgB += -t * gamB * (Bbar * gB[..., s, :, :]).sum(axis=-2)
        if t < T:
            gQbar += gamQ[..., :, None] * gQ[..., s, :, :] * gamQ[..., None, :]
            had = Q[..., s, :, :] * gQ[..., s, :, :]
            glgQ += -t * (had.sum(axis=-1) + had.sum(axis=-2))
    gQf = gQ[..., T - 1, :, :]
    grinv = -diag(gR.sum(axis=-3)) / rinv ** 2
    r, d = Bbasis.shape[0], Bbasis.shape[-1]
    over = lambda c, M: np.einsum("nk,nij->kij", c.reshape(-1, r), M.reshape(-1, d, d))   # sum over the problems
    return {"gsA": gsA, "glgA": glgA, "glgB": glgB, "glgQ": glgQ, "grinv": grinv, "gx0": dense["gx0"],
            "gsB": np.einsum("kij,...ij->...k", Bbasis, gBbar),
            "gsQ": np.einsum("kij,...ij->...k", Qbasis, gQbar),
            "gsQf": np.einsum("kij,...ij->...k", Qbasis, gQf),
            "gBbasis": over(sB, gBbar), "gQbasis": over(sQ, gQbar) + over(sQf, gQf)}
