"""Pins of the time-heterogeneous oracle (oracle.lqr_oracle.riccati_*_tv), against things other than
itself: the stacked KKT system of the problem solved by brute force (the matrix form of the proof of
Thm A.6, with A_t, B_t, Q_t, R_t on the block diagonals), the time-invariant oracle when every step
carries the same matrices, a scalar recursion written out by hand, and value == rolled-out cost."""
import numpy as np
import pytest

from oracle import lqr_oracle as orc


def draw_tv(d, m, T, seed, n=None):
    rng = np.random.default_rng(seed)
    lead = () if n is None else (n,)
    A = np.eye(d) + 0.3 * rng.standard_normal(lead + (T, d, d)) / np.sqrt(d)
    B = rng.standard_normal(lead + (T, d, m)) / np.sqrt(d)
    L = rng.standard_normal(lead + (T, d, d))
    Q = L @ np.swapaxes(L, -1, -2) / d + 1e-2 * np.eye(d)
    M = rng.standard_normal(lead + (T, m, m))
    R = np.eye(m) + M @ np.swapaxes(M, -1, -2) / m
    x0 = rng.standard_normal(lead + (d,))
    return A, B, Q, R, x0


def kkt_bruteforce_tv(A, B, Q, R, x0):
    """min 1/2 sum_s (u_s^T R_s u_s + x_{s+1}^T Q_s x_{s+1})  s.t.  x_{s+1} = A_s x_s + B_s u_s, x_0 given:
    one dense solve of the stacked optimality system in z = [x_0..x_T, u_0..u_{T-1}] and multipliers."""
    T, d, m = B.shape
    nh, nu = (T + 1) * d, T * m
    C = np.zeros((nh + nu, nh + nu))
    F = np.zeros((nh, nh + nu))
    F[:d, :d] = -np.eye(d)
    for s in range(T):
        C[(s + 1) * d:(s + 2) * d, (s + 1) * d:(s + 2) * d] = Q[s]
        C[nh + s * m: nh + (s + 1) * m, nh + s * m: nh + (s + 1) * m] = R[s]
        F[(s + 1) * d:(s + 2) * d, s * d:(s + 1) * d] = A[s]
        F[(s + 1) * d:(s + 2) * d, (s + 1) * d:(s + 2) * d] = -np.eye(d)
        F[(s + 1) * d:(s + 2) * d, nh + s * m: nh + (s + 1) * m] = B[s]
    b = np.zeros(nh)
    b[:d] = -x0
    KKT = np.block([[C, F.T], [F, np.zeros((nh, nh))]])
    sol = np.linalg.solve(KKT, np.concatenate([np.zeros(nh + nu), b]))
    z, xi = sol[:nh + nu], sol[nh + nu:]
    return z[:nh].reshape(T + 1, d), z[nh:].reshape(T, m), xi.reshape(T + 1, d), float(z @ C @ z)


@pytest.mark.parametrize("d,m,T,seed", [(1, 1, 3, 0), (2, 2, 4, 1), (3, 2, 5, 2), (4, 4, 6, 3), (3, 5, 2, 4), (4, 4, 1, 5)])
def test_kkt_bruteforce_tv(d, m, T, seed):
    A, B, Q, R, x0 = draw_tv(d, m, T, seed)
    s = orc.riccati_solve_tv(A, B, Q, R, x0)
    X, U, Lam, zCz = kkt_bruteforce_tv(A, B, Q, R, x0)
    np.testing.assert_allclose(s["u0"], U[0], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(s["P0"] @ x0, Lam[0], rtol=1e-9, atol=1e-11)   # lambda_0 = P_0 x_0
    assert float(s["value"]) == pytest.approx(zCz, rel=1e-9)
    Ur, Xr, cost = orc.riccati_rollout_tv(A, B, Q, R, x0)
    np.testing.assert_allclose(Ur, U, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(Xr, X, rtol=1e-8, atol=1e-10)
    assert float(cost) == pytest.approx(zCz, rel=1e-9)


@pytest.mark.parametrize("T", [1, 2, 5, 9])
def test_constant_steps_reduce_to_the_time_invariant_oracle(T):
    d, m, n = 5, 5, 7
    A, B, Q, R, x0 = draw_tv(d, m, 1, seed=T, n=n)
    QT = 1.7 * Q[:, 0] + 0.1 * np.eye(d)
    rep = lambda M: np.repeat(M, T, axis=1)
    Qtv = rep(Q).copy()
    Qtv[:, T - 1] = QT                                  # the last step arrives at the terminal cost
    tv = orc.riccati_solve_tv(rep(A), rep(B), Qtv, rep(R), x0)
    ti = orc.riccati_solve(A[:, 0], B[:, 0], Q[:, 0], R[:, 0], QT, x0, T)
    for k in ("P0", "K0", "u0", "value"):
        np.testing.assert_allclose(tv[k], ti[k], rtol=1e-12, atol=1e-13)


def test_scalar_recursion_by_hand():
    """d = m = 1: p_s = q_{s-1} + a_s^2 p r_s / (r_s + b_s^2 p), k_s = -a_s b_s p / (r_s + b_s^2 p)."""
    a = np.array([1.1, 0.7, -0.9, 1.3]); b = np.array([0.5, -1.2, 0.8, 1.0])
    q = np.array([0.3, 1.0, 0.2, 2.0]); r = np.array([1.0, 0.5, 2.0, 1.5])
    T = 4
    p = q[T - 1]
    for s in range(T - 1, -1, -1):
        k = -a[s] * b[s] * p / (r[s] + b[s] ** 2 * p)
        p = (q[s - 1] if s >= 1 else 0.0) + a[s] ** 2 * p * r[s] / (r[s] + b[s] ** 2 * p)
    m3 = lambda v: v.reshape(T, 1, 1)
    sol = orc.riccati_solve_tv(m3(a), m3(b), m3(q), m3(r), np.array([2.0]))
    assert float(sol["P0"][0, 0]) == pytest.approx(p, rel=1e-13)
    assert float(sol["K0"][0, 0]) == pytest.approx(k, rel=1e-13)
    assert float(sol["value"]) == pytest.approx(4.0 * p, rel=1e-13)


def test_value_matrices_are_symmetric_psd_and_batched_equals_single():
    A, B, Q, R, x0 = draw_tv(6, 6, 7, seed=9, n=5)
    s = orc.riccati_solve_tv(A, B, Q, R, x0)
    for P in s["P"]:
        assert np.abs(P - np.swapaxes(P, -1, -2)).max() < 1e-12
        assert np.linalg.eigvalsh(P).min() > -1e-10
    one = orc.riccati_solve_tv(A[3], B[3], Q[3], R[3], x0[3])
    np.testing.assert_allclose(one["P0"], s["P0"][3], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(one["u0"], s["u0"][3], rtol=1e-13, atol=1e-14)
