"""Pins of the gradient oracle (oracle/lqr_grad_oracle.py) against what the mathematics fixes: finite differences
of the forward oracle, the stacked KKT system of the proof of Thm A.6, a scalar problem differentiated by hand,
and invariances of the layer.  CPU only."""
import numpy as np
import pytest

from oracle import lqr_grad_oracle as go
from oracle import lqr_oracle


def random_tv(rng, d, m, T, batch=()):
    A = np.eye(d) + 0.3 * rng.standard_normal(batch + (T, d, d)) / np.sqrt(d)
    B = rng.standard_normal(batch + (T, d, m)) / np.sqrt(d)
    L = rng.standard_normal(batch + (T, d, d))
    Q = L @ np.swapaxes(L, -1, -2) / d + 0.05 * np.eye(d)
    M = rng.standard_normal(batch + (T, m, m))
    R = np.eye(m) + M @ np.swapaxes(M, -1, -2) / m
    x0 = rng.standard_normal(batch + (d,))
    g = rng.standard_normal(batch + (m,))
    return A, B, Q, R, x0, g


def loss(A, B, Q, R, x0, g):
    return float(g @ lqr_oracle.riccati_solve_tv(A, B, Q, R, x0)["u0"])


@pytest.mark.parametrize("d,m,T,seed", [(3, 3, 3, 0), (2, 3, 4, 1), (4, 2, 2, 2), (3, 3, 1, 3)])
def test_central_finite_differences_of_the_forward_oracle(d, m, T, seed):
    """Every entry of every A_t, B_t, Q_t, R_t and of h_0, perturbed one at a time.  Q and R are read as their
    symmetric parts, so an off-diagonal entry moves the loss by the symmetric gradient's entry."""
    rng = np.random.default_rng(seed)
    A, B, Q, R, x0, g = random_tv(rng, d, m, T)
    G = go.lqr_gradients_tv(A, B, Q, R, x0, g)
    eps = 1e-6
    args = {"A": A, "B": B, "Q": Q, "R": R, "x0": x0}
    for name, key in (("A", "gA"), ("B", "gB"), ("Q", "gQ"), ("R", "gR"), ("x0", "gx0")):
        base = args[name]
        fd = np.zeros_like(base)
        for idx in np.ndindex(base.shape):
            hi, lo = base.copy(), base.copy()
            hi[idx] += eps
            lo[idx] -= eps
            fd[idx] = (loss(**{**args, name: hi}, g=g) - loss(**{**args, name: lo}, g=g)) / (2 * eps)
        scale = max(1.0, np.abs(fd).max())
        assert np.abs(fd - G[key]).max() <= 2e-7 * scale, (name, np.abs(fd - G[key]).max())


def stacked_kkt(A, B, Q, R, T, d, m):
    """C, F of the proof of Thm A.6: x = [h_0..h_T, u_1..u_T], xi = [lam_0..lam_T]."""
    nx, nxi = (T + 1) * d + T * m, (T + 1) * d
    C = np.zeros((nx, nx))
    F = np.zeros((nxi, nx))
    for t in range(1, T + 1):
        C[t * d:(t + 1) * d, t * d:(t + 1) * d] = 0.5 * (Q[t - 1] + Q[t - 1].T)
        o = (T + 1) * d + (t - 1) * m
        C[o:o + m, o:o + m] = 0.5 * (R[t - 1] + R[t - 1].T)
    F[:d, :d] = -np.eye(d)
    for t in range(1, T + 1):
        F[t * d:(t + 1) * d, (t - 1) * d:t * d] = A[t - 1]
        F[t * d:(t + 1) * d, t * d:(t + 1) * d] = -np.eye(d)
        o = (T + 1) * d + (t - 1) * m
        F[t * d:(t + 1) * d, o:o + m] = B[t - 1]
    return C, F


@pytest.mark.parametrize("d,m,T,seed", [(3, 2, 3, 5), (2, 2, 4, 6)])
def test_both_trajectories_solve_the_stacked_kkt_systems(d, m, T, seed):
    """Primal: [[C, F^T], [F, 0]] [x; xi] = [0; b] with b = [-h_init, 0, ...].  Dual (the adjoint system of the
    proof): the same matrix with right-hand side [-dl/dx; 0], dl/dx non-zero only in the u_1 block."""
    rng = np.random.default_rng(seed)
    A, B, Q, R, x0, g = random_tv(rng, d, m, T)
    G = go.lqr_gradients_tv(A, B, Q, R, x0, g)
    C, F = stacked_kkt(A, B, Q, R, T, d, m)
    nx, nxi = C.shape[0], F.shape[0]
    KKT = np.block([[C, F.T], [F, np.zeros((nxi, nxi))]])
    b = np.zeros(nxi)
    b[:d] = -x0
    z = np.linalg.solve(KKT, np.concatenate([np.zeros(nx), b]))
    pack = lambda X, U, LAM: np.concatenate([X.reshape(-1), U.reshape(-1), LAM.reshape(-1)])
    assert np.abs(z - pack(G["X"], G["U"], G["LAM"])).max() <= 1e-10
    dl = np.zeros(nx)
    dl[(T + 1) * d:(T + 1) * d + m] = g
    zt = np.linalg.solve(KKT, np.concatenate([-dl, np.zeros(nxi)]))
    assert np.abs(zt - pack(G["Xt"], G["Ut"], G["LAMt"])).max() <= 1e-10
    # the gradient with respect to one entry of A_t, straight from the proof: xi_{td+i} xt_{(t-1)d+j} + xit_{td+i} x_{(t-1)d+j}
    xi, xit = z[nx:], zt[nx:]
    t, i, j = 2, 1, 0
    want = xi[t * d + i] * zt[(t - 1) * d + j] + xit[t * d + i] * z[(t - 1) * d + j]
    assert abs(G["gA"][t - 1, i, j] - want) <= 1e-12


def test_scalar_problem_by_hand():
    """d = m = 1, T = 1: u_0 = -b q a x0 / (r + b^2 q) with q the terminal cost; l = g u_0.  With a = 2, b = 3,
    q = 5, r = 7, x0 = 11, g = 13: r + b^2 q = 52, u_0 = -330/52.  Differentiating the quotient by hand:
      dl/da = g (-b q x0 / 52) = -13 * 165 / 52           dl/dx0 = g (-b q a / 52) = -13 * 30 / 52
      dl/db = g (-q a x0 (r - b^2 q) / 52^2) = 13 * 110 * 38 / 2704
      dl/dq = g (-b a x0 r / 52^2) = -13 * 66 * 7 / 2704   dl/dr = g (b q a x0 / 52^2) = 13 * 330 / 2704"""
    A, B, Q, R = (np.array([[[v]]], dtype=float) for v in (2.0, 3.0, 5.0, 7.0))
    G = go.lqr_gradients_tv(A, B, Q, R, np.array([11.0]), np.array([13.0]))
    assert G["gA"].item() == pytest.approx(-13 * 165 / 52, rel=1e-13)
    assert G["gx0"].item() == pytest.approx(-13 * 30 / 52, rel=1e-13)
    assert G["gB"].item() == pytest.approx(13 * 110 * 38 / 2704, rel=1e-13)
    assert G["gQ"].item() == pytest.approx(-13 * 66 * 7 / 2704, rel=1e-13)
    assert G["gR"].item() == pytest.approx(13 * 330 / 2704, rel=1e-13)


def test_gradient_with_respect_to_the_initial_state_is_the_transposed_gain():
    rng = np.random.default_rng(7)
    A, B, Q, R, x0, g = random_tv(rng, 4, 3, 5, batch=(6,))
    G = go.lqr_gradients_tv(A, B, Q, R, x0, g)
    K0 = lqr_oracle.riccati_solve_tv(A, B, Q, R, x0)["K0"]
    assert np.abs(G["gx0"] - np.einsum("nij,ni->nj", K0, g)).max() <= 1e-12


def test_invariances_of_the_layer_bind_the_gradients():
    """(1) Multiplying every Q_t and R_t by the same factor leaves u_0 unchanged: sum <gQ, Q> + <gR, R> = 0.
    (2) A change of state coordinates h -> (I + eps X) h, i.e. A_t -> A_t + eps (X A_t - A_t X),
    B_t -> B_t + eps X B_t, Q_t -> Q_t - eps (X^T Q_t + Q_t X), h_0 -> h_0 + eps X h_0, leaves u_0 unchanged."""
    rng = np.random.default_rng(8)
    d, m, T = 4, 3, 4
    A, B, Q, R, x0, g = random_tv(rng, d, m, T)
    G = go.lqr_gradients_tv(A, B, Q, R, x0, g)
    size = np.abs(G["gQ"] * Q).sum() + np.abs(G["gR"] * R).sum()
    assert abs((G["gQ"] * Q).sum() + (G["gR"] * R).sum()) <= 1e-12 * size
    X = rng.standard_normal((d, d))
    dA = X @ A - A @ X
    dB = X @ B
    dQ = -(X.T @ Q + Q @ X)
    lie = (G["gA"] * dA).sum() + (G["gB"] * dB).sum() + (G["gQ"] * dQ).sum() + G["gx0"] @ (X @ x0)
    size = np.abs(G["gA"] * dA).sum() + np.abs(G["gB"] * dB).sum() + np.abs(G["gQ"] * dQ).sum()
    assert abs(lie) <= 1e-12 * size


def test_time_invariant_gradients_against_finite_differences():
    rng = np.random.default_rng(9)
    d, T = 3, 4
    A = np.eye(d) + 0.3 * rng.standard_normal((d, d))
    B = rng.standard_normal((d, d))
    L, M = rng.standard_normal((d, d)), rng.standard_normal((d, d))
    Q, R, QT = L @ L.T + 0.1 * np.eye(d), np.eye(d) + M @ M.T, 2.0 * L @ L.T + np.eye(d)
    x0, g = rng.standard_normal(d), rng.standard_normal(d)
    eps = 1e-6
    for qt in (None, QT):
        G = go.lqr_gradients(A, B, Q, R, qt, x0, T, g)
        args = {"A": A, "B": B, "Q": Q, "R": R}
        if qt is not None:
            args["QT"] = qt
        f = lambda a: float(g @ lqr_oracle.riccati_solve(a["A"], a["B"], a["Q"], a["R"], a.get("QT"), x0, T)["u0"])
        for name in args:
            fd = np.zeros((d, d))
            for idx in np.ndindex(d, d):
                hi, lo = args[name].copy(), args[name].copy()
                hi[idx] += eps
                lo[idx] -= eps
                fd[idx] = (f({**args, name: hi}) - f({**args, name: lo})) / (2 * eps)
            assert np.abs(fd - G["g" + name]).max() <= 2e-7 * max(1.0, np.abs(fd).max()), name
        if qt is None:
            assert G["gQT"] is None


@pytest.mark.parametrize("d,r,T,seed", [(3, 2, 3, 0), (2, 3, 1, 1), (4, 2, 2, 2)])
def test_structured_gradients_against_finite_differences(d, r, T, seed):
    """contextual_gradients against central differences of contextual_solve's u0 in every input: the per-problem
    vectors (the log-scale modulation coefficients and the diagonal of R^{-1} among them), x0 and both groups of
    basis matrices (whose gradients sum over the problems)."""
    from oracle import lqr_oracle
    rng = np.random.default_rng(seed)
    n = 2
    sp = lambda z: np.logaddexp(0.0, z)
    args = {"sA": 0.3 * rng.normal(size=(n, d)), "sB": rng.normal(size=(n, r)), "sQ": sp(rng.normal(size=(n, r))),
            "sQf": sp(rng.normal(size=(n, r))), "rinv": sp(rng.normal(size=(n, d))) + 0.2,
            "lgA": 0.3 * sp(rng.normal(size=(n, d))), "lgB": 0.3 * sp(rng.normal(size=(n, d))),
            "lgQ": 0.3 * sp(rng.normal(size=(n, d))), "Bbasis": rng.normal(size=(r, d, d)) / np.sqrt(d)}
    Qc = rng.normal(size=(r, d, d))
    args["Qbasis"] = Qc @ np.swapaxes(Qc, -1, -2) / np.sqrt(d)
    args["x0"] = rng.normal(size=(n, d))
    g = rng.normal(size=(n, d))
    order = ("sA", "sB", "sQ", "sQf", "rinv", "lgA", "lgB", "lgQ", "Bbasis", "Qbasis", "x0")
    loss = lambda a: float((lqr_oracle.contextual_solve(*(a[k] for k in order), T)["u0"] * g).sum())
    got = go.contextual_gradients(*(args[k] for k in order), T, g)
    names = {"sA": "gsA", "sB": "gsB", "sQ": "gsQ", "sQf": "gsQf", "rinv": "grinv", "lgA": "glgA", "lgB": "glgB",
             "lgQ": "glgQ", "Bbasis": "gBbasis", "Qbasis": "gQbasis", "x0": "gx0"}
    eps = 1e-6
    for key, gname in names.items():
        fd = np.zeros_like(args[key])
        for idx in np.ndindex(*args[key].shape):
            if key == "Qbasis" and idx[1] > idx[2]:
                continue                       # Q^(k) is symmetric: move the pair of entries together
            hi, lo = {k: v.copy() for k, v in args.items()}, {k: v.copy() for k, v in args.items()}
            pairs = [idx] if key != "Qbasis" or idx[1] == idx[2] else [idx, (idx[0], idx[2], idx[1])]
            for ix in pairs:
                hi[key][ix] += eps
                lo[key][ix] -= eps
            fd[idx] = (loss(hi) - loss(lo)) / (2 * eps)
        want = got[gname]
        if key == "Qbasis":                     # the derivative along a symmetric pair is the sum of the two entries
            want = np.triu(want + np.swapaxes(want, -1, -2)) - np.einsum("kij,ij->kij", want, np.eye(d))
        scale = max(np.abs(want).max(), 1e-12)
        assert np.abs(fd - want).max() <= 2e-6 * scale + 1e-9, (key, np.abs(fd - want).max(), scale)
