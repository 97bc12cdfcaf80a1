"""Pins of the structured, contextualised parameters (oracle.lqr_oracle.contextual_*) against things other
than the oracle's own formula: an expansion worked out by hand (tests/golden/contextual_d2_T2.txt), ratio
properties that tell row from column scaling and exponent t from t - 1, the scalar problem solved by hand,
the time-invariant oracle when no modulation is applied, and the stacked KKT system solved by brute force."""
import os

import numpy as np
import pytest

from oracle import lqr_oracle as orc
from tests.test_oracle_pins_tv import kkt_bruteforce_tv

GOLD = os.path.join(os.path.dirname(__file__), "golden", "contextual_d2_T2.txt")


def read_golden():
    vals = {}
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = np.array([{"ln2": np.log(2.0), "ln4": np.log(4.0)}.get(x) or float(x) for x in rest])
    return vals


def golden_inputs():
    g = read_golden()
    Bb = np.stack([g["Bbasis0"].reshape(2, 2), g["Bbasis1"].reshape(2, 2)])
    Qb = np.stack([g["Qbasis0"].reshape(2, 2), g["Qbasis1"].reshape(2, 2)])
    return g, (g["sA"], g["sB"], g["sQ"], g["sQf"], g["rinv"], g["lgA"], g["lgB"], g["lgQ"], Bb, Qb)


def test_expansion_matches_hand_worked_example():
    g, args = golden_inputs()
    A, B, Q, R = orc.contextual_parameters(*args, T=2)
    for name, M in (("A", A), ("B", B), ("Q", Q), ("R", R)):
        for t in (1, 2):
            np.testing.assert_allclose(M[t - 1], g[f"{name}{t}"].reshape(2, 2), rtol=1e-14, atol=1e-15, err_msg=f"{name}{t}")


def test_hand_worked_example_solves_like_brute_force():
    g, args = golden_inputs()
    x0 = np.array([1.0, -1.0])
    A = np.stack([g["A1"].reshape(2, 2), g["A2"].reshape(2, 2)])
    B = np.stack([g["B1"].reshape(2, 2), g["B2"].reshape(2, 2)])
    Q = np.stack([g["Q1"].reshape(2, 2), g["Q2"].reshape(2, 2)])
    R = np.stack([g["R1"].reshape(2, 2), g["R2"].reshape(2, 2)])
    X, U, Lam, zCz = kkt_bruteforce_tv(A, B, Q, R, x0)
    s = orc.contextual_solve(*args, x0, 2)
    np.testing.assert_allclose(s["u0"], U[0], rtol=1e-10)
    np.testing.assert_allclose(s["P0"] @ x0, Lam[0], rtol=1e-10)
    assert float(s["value"]) == pytest.approx(zCz, rel=1e-10)


def draw(d, r, seed, n=None):
    rng = np.random.default_rng(seed)
    lead = () if n is None else (n,)
    sp = lambda x: np.log1p(np.exp(x))
    sA = 0.3 * rng.standard_normal(lead + (d,))
    sB = rng.standard_normal(lead + (r,)) / np.sqrt(r)
    sQ, sQf = sp(rng.standard_normal(lead + (r,))) / r, sp(rng.standard_normal(lead + (r,))) / r
    rinv = sp(rng.standard_normal(lead + (d,))) + 0.1
    lgA, lgB, lgQ = (0.3 * sp(rng.standard_normal(lead + (d,))) for _ in range(3))
    Bb = rng.standard_normal((r, d, d)) / np.sqrt(d)
    Qc = rng.standard_normal((r, d, d))
    Qb = Qc @ np.swapaxes(Qc, -1, -2) / np.sqrt(d)
    x0 = rng.standard_normal(lead + (d,))
    return (sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bb, Qb), x0


def test_modulation_ratios():
    """Consecutive steps differ by exactly one factor Gamma: on the diagonal of A - I, on the columns
    (not the rows) of B, on both sides of Q; step 1 already carries one factor (exponent t, not t - 1)."""
    args, _ = draw(5, 3, 0)
    sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bb, Qb = args
    T = 4
    A, B, Q, R = orc.contextual_parameters(*args, T=T)
    gA, gB, gQ = np.exp(-lgA), np.exp(-lgB), np.exp(-lgQ)
    np.testing.assert_allclose(np.diag(A[0]) - 1.0, gA * sA, rtol=1e-13)
    np.testing.assert_allclose(B[0] / gB[None, :], np.tensordot(sB, Bb, 1), rtol=1e-13)
    for s in range(1, T):
        assert np.count_nonzero(A[s] - np.diag(np.diag(A[s]))) == 0
        np.testing.assert_allclose((np.diag(A[s]) - 1.0) / (np.diag(A[s - 1]) - 1.0), gA, rtol=1e-12)
        np.testing.assert_allclose(B[s] / B[s - 1], np.broadcast_to(gB[None, :], B[s].shape), rtol=1e-12)
        if s < T - 1:
            np.testing.assert_allclose(Q[s] / Q[s - 1], np.outer(gQ, gQ), rtol=1e-12)
        np.testing.assert_array_equal(R[s], R[0])
    np.testing.assert_allclose(Q[T - 1], np.tensordot(sQf, Qb, 1), rtol=1e-13)   # the terminal override, unmodulated
    np.testing.assert_allclose(np.diag(R[0]) * rinv, np.ones(5), rtol=1e-14)
    for s in range(T):
        np.testing.assert_allclose(Q[s], Q[s].T, rtol=1e-13)
        assert np.linalg.eigvalsh(Q[s]).min() > -1e-12


def test_scalar_problem_by_hand():
    """d = r = 1, T = 2: two Riccati steps written out for scalars."""
    sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, b1, q1, x0 = 0.4, -0.7, 1.3, 0.9, 2.5, 0.2, 0.5, 0.3, 1.7, 0.6, -1.1
    a = [1 + np.exp(-t * lgA) * sA for t in (1, 2)]
    b = [sB * b1 * np.exp(-t * lgB) for t in (1, 2)]
    qq1 = np.exp(-2 * lgQ) * sQ * q1            # Q_1: one factor Gamma_Q on each side
    R = 1 / rinv
    P2 = sQf * q1
    P1 = qq1 + a[1] ** 2 * P2 * R / (R + b[1] ** 2 * P2)
    P0 = a[0] ** 2 * P1 * R / (R + b[0] ** 2 * P1)
    K0 = -b[0] * P1 * a[0] / (R + b[0] ** 2 * P1)
    v = lambda x: np.array([x])
    s = orc.contextual_solve(v(sA), v(sB), v(sQ), v(sQf), v(rinv), v(lgA), v(lgB), v(lgQ),
                             np.array([[[b1]]]), np.array([[[q1]]]), v(x0), 2)
    assert float(s["P0"][0, 0]) == pytest.approx(P0, rel=1e-13)
    assert float(s["K0"][0, 0]) == pytest.approx(K0, rel=1e-13)
    assert float(s["u0"][0]) == pytest.approx(K0 * x0, rel=1e-13)
    assert float(s["value"]) == pytest.approx(P0 * x0 * x0, rel=1e-13)


@pytest.mark.parametrize("T", [1, 3, 6])
def test_no_modulation_is_the_time_invariant_problem(T):
    args, x0 = draw(4, 3, 1, n=5)
    sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bb, Qb = args
    z = np.zeros_like(lgA)
    s = orc.contextual_solve(sA, sB, sQ, sQf, rinv, z, z, z, Bb, Qb, x0, T)
    eye = np.eye(4)
    A = eye + sA[:, :, None] * eye
    B = np.einsum("ni,ijk->njk", sB, Bb)
    Q = np.einsum("ni,ijk->njk", sQ, Qb)
    QT = np.einsum("ni,ijk->njk", sQf, Qb)
    R = (1 / rinv)[:, :, None] * eye
    ref = orc.riccati_solve(A, B, Q, R, QT, x0, T)
    for k in ("P0", "K0", "u0", "value"):
        np.testing.assert_allclose(s[k], ref[k], rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("d,r,T,seed", [(2, 1, 3, 0), (3, 4, 5, 1), (4, 2, 1, 2)])
def test_contextual_solve_vs_kkt(d, r, T, seed):
    args, x0 = draw(d, r, seed)
    A, B, Q, R = orc.contextual_parameters(*args, T=T)
    X, U, Lam, zCz = kkt_bruteforce_tv(A, B, Q, R, x0)
    s = orc.contextual_solve(*args, x0, T)
    np.testing.assert_allclose(s["u0"], U[0], rtol=1e-9, atol=1e-11)
    assert float(s["value"]) == pytest.approx(zCz, rel=1e-9)


def test_batched_equals_single():
    args, x0 = draw(3, 2, 4, n=6)
    s = orc.contextual_solve(*args, x0, 4)
    for j in (0, 5):
        one = orc.contextual_solve(*(a[j] if a.ndim == 2 and a.shape[0] == 6 else a for a in args), x0[j], 4)
        np.testing.assert_allclose(s["P0"][j], one["P0"], rtol=1e-12)
        np.testing.assert_allclose(s["u0"][j], one["u0"], rtol=1e-12)


def test_rollout_cost_is_the_value_and_follows_the_dynamics():
    args, x0 = draw(4, 3, 7, n=5)
    T = 6
    U, X, cost = orc.contextual_rollout(*args, x0, T)
    s = orc.contextual_solve(*args, x0, T)
    np.testing.assert_allclose(cost, s["value"], rtol=1e-10)
    np.testing.assert_allclose(U[:, 0], s["u0"], rtol=1e-12)
    A, B, Q, R = orc.contextual_parameters(*args, T=T)
    for t in range(T):
        np.testing.assert_allclose(X[:, t + 1], np.einsum("nij,nj->ni", A[:, t], X[:, t]) +
                                   np.einsum("nij,nj->ni", B[:, t], U[:, t]), rtol=1e-12, atol=1e-13)
