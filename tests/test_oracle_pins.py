"""Pins for the CPU float64 oracle (no GPU).  Each test checks the oracle against something other
than its own formula: closed forms, brute-force linear systems, scipy's DARE solver, the paper's
symplectic product, structural invariants."""
import os

import numpy as np
import pytest
import scipy.linalg as sla

from oracle import lqr_oracle as orc
from paper_2603_09221_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def draw(d, m, T, seed, n=None, rho=None):
    b = synth.make_batch(1 if n is None else n, d, m, T, seed=seed, rho=rho)
    A, B, Q, R, x0 = b.numpy64()
    if n is None:
        return A[0], B[0], Q[0], R[0], x0[0]
    return A, B, Q, R, x0


# ---------------------------------------------------------------- closed forms
def test_scalar_fibonacci_golden():
    rows = [l.split() for l in open(os.path.join(GOLD, "scalar_fibonacci.txt")) if l.strip() and l[0] != "#"]
    one = np.ones((1, 1))
    for T, p1n, p1d, p0n, p0d in (map(int, r) for r in rows):
        s = orc.riccati_solve(one, one, one, one, one, np.array([2.0]), T)
        assert s["P"][1][0, 0] == pytest.approx(p1n / p1d, rel=1e-14)
        assert s["P0"][0, 0] == pytest.approx(p0n / p0d, rel=1e-14)
        assert s["K0"][0, 0] == pytest.approx(-p0n / p0d, rel=1e-14)
        assert s["u0"][0] == pytest.approx(-2.0 * p0n / p0d, rel=1e-14)
        assert float(s["value"]) == pytest.approx(4.0 * p0n / p0d, rel=1e-14)
        st = orc.riccati_solve(one, one, one, one, one, np.array([2.0]), T, stage_cost_at_x0=True)
        assert st["P0"][0, 0] == pytest.approx(p0n / p0d + 1.0, rel=1e-14)


def test_scalar_general_recursion():
    rng = np.random.default_rng(1)
    for _ in range(20):
        a, b = rng.normal(size=2)
        q, r, qT = rng.uniform(0.1, 3.0, size=3)
        T = int(rng.integers(1, 9))
        p = qT
        for _t in range(T - 1):                      # p_{t} = q + a^2 p r / (r + b^2 p)
            p = q + a * a * p * r / (r + b * b * p)
        k0 = -a * b * p / (r + b * b * p)
        p0 = a * a * p * r / (r + b * b * p)
        m = lambda v: np.array([[v]])
        s = orc.riccati_solve(m(a), m(b), m(q), m(r), m(qT), np.array([1.5]), T)
        assert s["K0"][0, 0] == pytest.approx(k0, rel=1e-12)
        assert s["P0"][0, 0] == pytest.approx(p0, rel=1e-12)


def test_T1_closed_form():
    A, B, Q, R, x0 = draw(5, 3, 1, seed=3)
    QT = Q + 0.3 * np.eye(5)
    s = orc.riccati_solve(A, B, Q, R, QT, x0, 1)
    G = B @ np.linalg.inv(R) @ B.T
    P0 = A.T @ np.linalg.inv(np.eye(5) + QT @ G) @ QT @ A
    K0 = -np.linalg.inv(R + B.T @ QT @ B) @ B.T @ QT @ A
    np.testing.assert_allclose(s["P0"], P0, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(s["K0"], K0, rtol=1e-11, atol=1e-13)


def test_decoupled_diagonal_matches_scalar_problems():
    rng = np.random.default_rng(5)
    d, T = 6, 7
    a, b = rng.normal(size=d), rng.normal(size=d)
    q, r, qT = rng.uniform(0.1, 2, d), rng.uniform(0.5, 2, d), rng.uniform(0.1, 2, d)
    s = orc.riccati_solve(np.diag(a), np.diag(b), np.diag(q), np.diag(r), np.diag(qT), np.ones(d), T)
    for i in range(d):
        m = lambda v: np.array([[v]])
        si = orc.riccati_solve(m(a[i]), m(b[i]), m(q[i]), m(r[i]), m(qT[i]), np.ones(1), T)
        assert s["P0"][i, i] == pytest.approx(si["P0"][0, 0], rel=1e-12)
        assert s["K0"][i, i] == pytest.approx(si["K0"][0, 0], rel=1e-12)
    off = s["P0"] - np.diag(np.diag(s["P0"]))
    assert np.abs(off).max() < 1e-14


# ---------------------------------------------------------------- brute force
def kkt_bruteforce(A, B, Q, R, QT, x0, T):
    """Dense solve of the stacked KKT system in the matrix form used in the proof of Thm A.6:
    x = [h_0..h_T, u_1..u_T], L = 1/2 x^T C x + xi^T (F x - b)."""
    d, m = B.shape
    nh, nu = (T + 1) * d, T * m
    C = np.zeros((nh + nu, nh + nu))
    for t in range(1, T + 1):
        C[t * d:(t + 1) * d, t * d:(t + 1) * d] = QT if t == T else Q
        C[nh + (t - 1) * m: nh + t * m, nh + (t - 1) * m: nh + t * m] = R
    F = np.zeros((nh, nh + nu))
    F[:d, :d] = -np.eye(d)
    for t in range(1, T + 1):
        F[t * d:(t + 1) * d, (t - 1) * d:t * d] = A
        F[t * d:(t + 1) * d, t * d:(t + 1) * d] = -np.eye(d)
        F[t * d:(t + 1) * d, nh + (t - 1) * m: nh + t * m] = B
    b = np.zeros(nh)
    b[:d] = -x0
    KKT = np.block([[C, F.T], [F, np.zeros((nh, nh))]])
    sol = np.linalg.solve(KKT, np.concatenate([np.zeros(nh + nu), b]))
    x, xi = sol[:nh + nu], sol[nh + nu:]
    return x[:nh].reshape(T + 1, d), x[nh:].reshape(T, m), xi.reshape(T + 1, d), float(x @ C @ x)


@pytest.mark.parametrize("d,m,T,seed", [(1, 1, 3, 0), (2, 2, 4, 1), (3, 2, 5, 2), (4, 4, 5, 3), (3, 5, 2, 4), (4, 4, 1, 5)])
def test_kkt_bruteforce(d, m, T, seed):
    A, B, Q, R, x0 = draw(d, m, T, seed)
    QT = Q + 0.5 * np.eye(d)
    s = orc.riccati_solve(A, B, Q, R, QT, x0, T)
    H, U, Lam, xCx = kkt_bruteforce(A, B, Q, R, QT, x0, T)
    np.testing.assert_allclose(s["u0"], U[0], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(s["P0"] @ x0, Lam[0], rtol=1e-9, atol=1e-11)   # lambda_0 = P_0 h_0
    assert float(s["value"]) == pytest.approx(xCx, rel=1e-9)
    Ur, Xr, cost = orc.riccati_rollout(A, B, Q, R, QT, x0, T)
    np.testing.assert_allclose(Ur, U, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(Xr, H, rtol=1e-8, atol=1e-10)
    assert float(cost) == pytest.approx(xCx, rel=1e-9)


def test_condensed_qp():
    d, m, T = 3, 2, 4
    A, B, Q, R, x0 = draw(d, m, T, seed=11)
    QT = 2.0 * Q
    Phi = np.vstack([np.linalg.matrix_power(A, t) for t in range(1, T + 1)])        # x_t = A^t x0 + ...
    Gam = np.zeros((T * d, T * m))
    for t in range(1, T + 1):
        for s_ in range(1, t + 1):
            Gam[(t - 1) * d:t * d, (s_ - 1) * m:s_ * m] = np.linalg.matrix_power(A, t - s_) @ B
    Qbar = sla.block_diag(*([Q] * (T - 1) + [QT]))
    Rbar = sla.block_diag(*([R] * T))
    Ustar = -np.linalg.solve(Gam.T @ Qbar @ Gam + Rbar, Gam.T @ Qbar @ Phi @ x0)
    s = orc.riccati_solve(A, B, Q, R, QT, x0, T)
    np.testing.assert_allclose(s["u0"], Ustar[:m], rtol=1e-10, atol=1e-12)
    xs = Phi @ x0 + Gam @ Ustar
    assert float(s["value"]) == pytest.approx(xs @ Qbar @ xs + Ustar @ Rbar @ Ustar, rel=1e-10)


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("d,T,seed", [(16, 8, 0), (64, 8, 1), (24, 16, 2)])
def test_value_equals_rollout_cost_and_flag(d, T, seed):
    A, B, Q, R, x0 = draw(d, d, T, seed, n=4)
    for flag in (False, True):
        s = orc.riccati_solve(A, B, Q, R, None, x0, T, stage_cost_at_x0=flag)
        U, X, cost = orc.riccati_rollout(A, B, Q, R, None, x0, T, stage_cost_at_x0=flag)
        np.testing.assert_allclose(s["value"], cost, rtol=1e-11)
        np.testing.assert_allclose(U[:, 0], s["u0"], rtol=1e-12, atol=1e-14)
    s0 = orc.riccati_solve(A, B, Q, R, None, x0, T)
    s1 = orc.riccati_solve(A, B, Q, R, None, x0, T, stage_cost_at_x0=True)
    np.testing.assert_allclose(s1["P0"] - s0["P0"], Q, rtol=0, atol=1e-12)
    np.testing.assert_allclose(s1["K0"], s0["K0"], rtol=0, atol=0)


def test_structure_symmetric_psd_and_joseph_form():
    d, T = 16, 8
    A, B, Q, R, x0 = draw(d, d, T, seed=7)
    s = orc.riccati_solve(A, B, Q, R, None, x0, T)
    P, K = s["P"], s["K"]
    for t in range(1, T + 1):
        assert np.abs(P[t] - P[t].T).max() == 0.0
        assert np.linalg.eigvalsh(P[t] - Q).min() > -1e-12 * np.linalg.norm(P[t])
    assert np.linalg.eigvalsh(s["P0"]).min() > -1e-12
    for t in range(1, T):                       # Joseph form of the same step
        Acl = A + B @ K[t]
        J = Q + K[t].T @ R @ K[t] + Acl.T @ P[t + 1] @ Acl
        np.testing.assert_allclose(P[t], J, rtol=1e-11, atol=1e-13)
    Acl = A + B @ K[0]
    np.testing.assert_allclose(s["P0"], K[0].T @ R @ K[0] + Acl.T @ P[1] @ Acl, rtol=1e-11, atol=1e-13)


def test_dare_fixed_point():
    d = 12
    A, B, Q, R, x0 = draw(d, d, 1, seed=9, rho=0.98)
    X = sla.solve_discrete_are(A, B, Q, R)
    errs = []
    for T in (4, 16, 64, 200):
        s = orc.riccati_solve(A, B, Q, R, None, x0, T)
        errs.append(np.linalg.norm(s["P"][1] - X) / np.linalg.norm(X))
    assert all(e1 > e2 for e1, e2 in zip(errs, errs[1:]))
    assert errs[-1] < 1e-9
    s = orc.riccati_solve(A, B, Q, R, None, x0, 200)
    Kinf = -np.linalg.solve(R + B.T @ X @ B, B.T @ X @ A)
    np.testing.assert_allclose(s["K0"], Kinf, rtol=1e-7, atol=1e-9)
    np.testing.assert_allclose(s["P0"], X - Q, rtol=1e-7, atol=1e-9)                     # paper convention
    st = orc.riccati_solve(A, B, Q, R, None, x0, 200, stage_cost_at_x0=True)
    np.testing.assert_allclose(st["P0"], X, rtol=1e-7, atol=1e-9)


# ---------------------------------------------------------------- the paper's symplectic product
def sigma(A, G, Qprev):
    """Sigma_t of Thm 3.3 (time-invariant A, G; Q_{t-1} = Qprev)."""
    AiT = np.linalg.inv(A).T
    return np.block([[AiT, AiT @ Qprev], [G @ AiT, A + G @ AiT @ Qprev]])


@pytest.mark.parametrize("d,T,seed", [(3, 4, 0), (8, 5, 1), (16, 4, 2)])
def test_reverse_symplectic_product(d, T, seed):
    A, B, Q, R, x0 = draw(d, d, T, seed)
    QT = Q + 0.1 * np.eye(d)
    G = B @ np.linalg.inv(R) @ B.T
    Y = np.hstack([np.eye(d), QT])
    J = np.block([[np.zeros((d, d)), np.eye(d)], [-np.eye(d), np.zeros((d, d))]])
    for t in range(T, 0, -1):
        Sg = sigma(A, G, Q if t >= 2 else np.zeros((d, d)))          # Q_0 = 0
        np.testing.assert_allclose(Sg.T @ J @ Sg, J, atol=1e-9)       # Lemma A.5 (transposed inverse of S_t)
        Y = Y @ Sg
        if t == 2:
            P1 = np.linalg.solve(Y[:, :d], Y[:, d:])
    Y1, Y2 = Y[:, :d], Y[:, d:]
    P0 = np.linalg.solve(Y1, Y2)
    Dscale = np.diag(1.0 / np.abs(Y).sum(axis=1))                    # row scaling leaves Y1^{-1} Y2 unchanged
    np.testing.assert_allclose(np.linalg.solve(Dscale @ Y1, Dscale @ Y2), P0, rtol=1e-8, atol=1e-10)
    lam0 = P0 @ x0
    u1 = -np.linalg.solve(R, B.T @ np.linalg.solve(A.T, lam0))
    s = orc.riccati_solve(A, B, Q, R, QT, x0, T)
    np.testing.assert_allclose(s["P0"], P0, rtol=1e-7, atol=1e-9)
    np.testing.assert_allclose(s["u0"], u1, rtol=1e-7, atol=1e-9)
    if T >= 2:
        np.testing.assert_allclose(s["P"][1], P1, rtol=1e-7, atol=1e-9)


# ---------------------------------------------------------------- batching and inputs
def test_batched_equals_single():
    A, B, Q, R, x0 = draw(8, 8, 6, seed=13, n=5)
    s = orc.riccati_solve(A, B, Q, R, None, x0, 6)
    for i in range(5):
        si = orc.riccati_solve(A[i], B[i], Q[i], R[i], None, x0[i], 6)
        np.testing.assert_allclose(s["P0"][i], si["P0"], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(s["u0"][i], si["u0"], rtol=1e-13, atol=1e-15)


def test_non_pd_R_raises():
    A, B, Q, R, x0 = draw(4, 4, 3, seed=2)
    with pytest.raises(np.linalg.LinAlgError):
        orc.riccati_solve(A, B, Q, R - 50.0 * np.eye(4), None, x0, 3)


def test_generators():
    b = synth.make_batch(6, 16, 16, 8, seed=0)
    A, B, Q, R, x0 = b.numpy64()
    assert A.shape == (6, 16, 16) and x0.shape == (6, 16)
    assert np.abs(Q - Q.transpose(0, 2, 1)).max() == 0 and np.abs(R - R.transpose(0, 2, 1)).max() == 0
    assert np.linalg.eigvalsh(Q).min() > 5e-3 and np.linalg.eigvalsh(R).min() > 0.99
    assert np.linalg.cond(R).max() < 1e3
    b2 = synth.make_batch(6, 16, 16, 8, seed=0)
    assert (b2.A == b.A).all() and (b2.x0 == b.x0).all()
    b3 = synth.make_batch(3, 16, 16, 8, seed=1, rho=0.98)
    r = np.abs(np.linalg.eigvals(b3.numpy64()[0])).max(axis=-1)
    np.testing.assert_allclose(r, 0.98, rtol=1e-5)
    bb = synth.make_batch(2, 16, 16, 8, seed=0, dtype="bf16")
    assert bb.A.dtype.is_floating_point and bb.A.element_size() == 2
    assert synth.config_problems("llm_adapter") == 524288
