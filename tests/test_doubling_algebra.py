"""CPU check of the algebra the long-horizon (squaring) path rests on, written out in float64 numpy and
compared with the oracle's backward Riccati recursion (Prop. 3.1): the one-step map
f_e(P) = H + A^T P (I + G P)^{-1} A of e = (A, G, Q), its square e o e, and the bit schedule that turns
T steps into squarings and applications.  This is test-side arithmetic: the HIP path shares no code with it."""
import numpy as np
import pytest

from oracle import lqr_oracle
from paper_2603_09221_amd import synth


def square(e):
    A, G, H = e
    I = np.eye(A.shape[-1])
    M = np.linalg.inv(I + G @ H)
    At = np.swapaxes(A, -1, -2)
    return A @ M @ A, G + A @ M @ G @ At, H + At @ H @ M @ A


def apply(e, P):
    A, G, H = e
    I = np.eye(A.shape[-1])
    return H + np.swapaxes(A, -1, -2) @ P @ np.linalg.solve(I + G @ P, A)


def p1_by_squaring(A, G, Q, QT, T, qt_is_q):
    """P_1 = f^(T-1)(Q_T); with Q_T = Q = f(0) it is f^T(0).  Bits of the count from the lowest."""
    m, P = (T, None) if qt_is_q else (T - 1, QT)
    e = (A, G, Q)
    while m:
        if m & 1:
            P = e[2] if P is None else apply(e, P)
        m >>= 1
        if m:
            e = square(e)
    return P


@pytest.mark.parametrize("T", [1, 2, 3, 4, 7, 8, 13, 16, 64])
@pytest.mark.parametrize("qt_is_q", [True, False])
def test_squaring_reproduces_the_riccati_recursion(T, qt_is_q):
    b = synth.make_batch(6, 16, 16, T, seed=T)
    A, B, Q, R, x0 = b.numpy64()
    rng = np.random.default_rng(T)
    L = rng.standard_normal(Q.shape)
    QT = Q if qt_is_q else L @ np.swapaxes(L, -1, -2) / 32
    ref = lqr_oracle.riccati_solve(A, B, Q, R, QT, x0, T)
    X = np.linalg.solve(R, np.swapaxes(B, -1, -2))
    G = B @ X
    P1 = p1_by_squaring(A, G, Q, QT, T, qt_is_q)
    np.testing.assert_allclose(P1, ref["P"][1], rtol=0, atol=1e-11 * np.abs(ref["P"][1]).max())
    I = np.eye(16)
    M1 = np.linalg.solve(I + P1 @ G, P1 @ A)          # (I + P_1 G)^{-1} P_1 A
    np.testing.assert_allclose(np.swapaxes(A, -1, -2) @ M1, ref["P0"], rtol=0, atol=1e-11 * np.abs(ref["P0"]).max())
    np.testing.assert_allclose(-X @ M1, ref["K0"], rtol=0, atol=1e-11 * np.abs(ref["K0"]).max())


def test_square_is_the_map_applied_twice():
    b = synth.make_batch(4, 16, 16, 2, seed=3)
    A, B, Q, R, _ = b.numpy64()
    G = B @ np.linalg.solve(R, np.swapaxes(B, -1, -2))
    e = (A, G, Q)
    rng = np.random.default_rng(0)
    L = rng.standard_normal(Q.shape)
    P = L @ np.swapaxes(L, -1, -2)
    np.testing.assert_allclose(apply(square(e), P), apply(e, apply(e, P)), rtol=1e-10, atol=1e-10)


def compose(e1, e2):
    """f_{e1} o f_{e2}: e1 is the earlier step (applied last in the backward recursion)."""
    A1, G1, H1 = e1
    A2, G2, H2 = e2
    I = np.eye(A1.shape[-1])
    M = np.linalg.inv(I + G1 @ H2)
    return A2 @ M @ A1, G2 + A2 @ M @ G1 @ np.swapaxes(A2, -1, -2), H1 + np.swapaxes(A1, -1, -2) @ H2 @ M @ A1


@pytest.mark.parametrize("T", [1, 2, 3, 5, 8, 13, 33])
def test_pairwise_composition_of_distinct_steps_reproduces_the_recursion(T):
    """The tree the time-heterogeneous long-horizon entry point walks: elements of the steps s = 1..T-1 and the
    terminal cost as the constant map (0, 0, Q_T), composed pairwise with strides 1, 2, 4, ...; H of the first
    element is then P_1 of the oracle."""
    tv = synth.make_tv_batch(3, 8, 8, T, seed=T)
    A, B, Q, R, x0 = tv.numpy64()
    ref = lqr_oracle.riccati_solve_tv(A, B, Q, R, x0)
    els = [(A[:, s], B[:, s] @ np.linalg.solve(R[:, s], np.swapaxes(B[:, s], -1, -2)), Q[:, s - 1]) for s in range(1, T)]
    Z = np.zeros_like(Q[:, 0])
    els.append((Z, Z, Q[:, T - 1]))
    st = 1
    while st < len(els):
        for j in range(0, len(els), 2 * st):
            if j + st < len(els):
                els[j] = compose(els[j], els[j + st])
        st *= 2
    np.testing.assert_allclose(els[0][2], ref["P"][1], rtol=0, atol=1e-11 * np.abs(ref["P"][1]).max())
    e = (A[:, 1], els[0][1] * 0 + B[:, 1] @ np.linalg.solve(R[:, 1], np.swapaxes(B[:, 1], -1, -2)), Q[:, 0]) if T > 2 else None
    if e is not None:   # composition agrees with applying the two maps one after the other
        P3 = ref["P"][3]
        e12 = compose(e, (A[:, 2], B[:, 2] @ np.linalg.solve(R[:, 2], np.swapaxes(B[:, 2], -1, -2)), Q[:, 1]))
        np.testing.assert_allclose(apply(e12, P3), ref["P"][1], rtol=0, atol=1e-11 * np.abs(ref["P"][1]).max())
