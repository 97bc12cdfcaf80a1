"""How long may a group of reverse symplectic factors (Thm 3.3) be in float32 on the structured, contextualised
parameters of Sec. 4?  With diagonal A_t and R_t the factors need no dense inverse (Sec. 3.3 "Structured
Parameterization"), so the only dense solve left is the re-base Y1^{-1} Y2 after a group; this test emulates the
grouped iteration in numpy float32 on the generator's problems and tabulates the error of P_0 against the float64
oracle.  Outcome (2000 problems, d = 16, r = 16; max / share of problems above 1e-4):
    T = 8:   k=1 1.7e-6   k=2 3.4e-6   k=3 3.6e-6   k=4 1.4e-4 / 0.1 %   k=6 3.8e-4 / 0.5 %   k=8 2.9e-1 / 36 %
    T = 16:  k=1 1.9e-6   k=2 3.2e-6   k=3 5.4e-6   k=4 1.8e-4 / 0.1 %   k=8 2.4e-2 / 20 %
    T = 32:  k=1 2.4e-6   k=2 3.8e-6   k=3 4.1e-6   k=4 1.4e-4 / 0.1 %   k=8 2.2e-2 / 19 %
Groups of up to three factors hold the float32 tolerance with a factor of twenty to spare; groups of four are at its
edge; the printed algorithm (one solve after all T factors, row normalisation being an exact scaling that does not
change Y1^{-1} Y2) loses a third of the problems at T = 8.
That margin belongs to the generator's parameter scales, not to the method: with control thirty times cheaper
(rinv x 30), or the state costs thirty times larger, groups of three lose 85 % of the problems (T = 16), with the
input matrices four times larger half of them; and the growth of Y1 does not separate the lost problems from the
good ones (good problems reach 3.6e3 on the generator's scales, lost ones start at 40 when the dynamics are
scaled), so a grouped kernel would need a fallback it cannot trigger reliably.  The structured kernel therefore
keeps the Riccati form of Prop. 3.1 (one 16 x 16 positive definite inverse per step), whose accuracy does not
depend on these scales."""
import numpy as np

from oracle import lqr_oracle
from paper_2603_09221_amd import synth


def grouped_symplectic_f32(A, B, Q, R, k):
    """P_0 by the reverse symplectic iteration in float32, re-based every k factors.  A, B, Q, R: (n, T, d, d);
    step s carries the paper's factor of t = s + 1: Y1 <- (Y1 + Y2 G_t) A_t^{-T}, Y2 <- Y2 A_t + Y1 Q_{t-1}, Q_0 = 0."""
    A, B, Q, R = (x.astype(np.float32) for x in (A, B, Q, R))
    n, T, d, _ = A.shape
    eye = np.broadcast_to(np.eye(d, dtype=np.float32), (n, d, d))
    Y1, Y2 = eye.copy(), Q[:, T - 1].copy()
    in_group = 0
    for s in range(T - 1, -1, -1):
        rinv = 1.0 / np.diagonal(R[:, s], axis1=-2, axis2=-1)            # R_t is diagonal
        ainv = 1.0 / np.diagonal(A[:, s], axis1=-2, axis2=-1)            # A_t is diagonal
        G = (B[:, s] * rinv[:, None, :]) @ np.swapaxes(B[:, s], -1, -2)
        Y1 = (Y1 + Y2 @ G) * ainv[:, None, :]
        Y2 = Y2 * np.diagonal(A[:, s], axis1=-2, axis2=-1)[:, None, :]
        if s > 0:
            Y2 = Y2 + Y1 @ Q[:, s - 1]
        in_group += 1
        if in_group == k or s == 0:
            P = np.linalg.solve(Y1, Y2)
            Y1, Y2 = eye.copy(), (0.5 * (P + np.swapaxes(P, -1, -2))).astype(np.float32)
            in_group = 0
    return Y2


def errors(n, T, k, seed=3, rinv_scale=1.0):
    b = synth.make_contextual_batch(n, 16, 16, T, seed=seed)
    f = lambda t: t.double().numpy()
    A, B, Q, R = lqr_oracle.contextual_parameters(f(b.sA), f(b.sB), f(b.sQ), f(b.sQf), rinv_scale * f(b.rinv), f(b.lgA),
                                                  f(b.lgB), f(b.lgQ), f(b.Bbasis), f(b.Qbasis), T)
    assert np.abs(A - A * np.eye(16)).max() == 0 and np.abs(R - R * np.eye(16)).max() == 0   # diagonal, as Sec. 4 says
    ref = lqr_oracle.riccati_solve_tv(A, B, Q, R, f(b.x0))["P0"]
    got = grouped_symplectic_f32(A, B, Q, R, k)
    return np.linalg.norm((got - ref).reshape(n, -1), axis=1) / np.linalg.norm(ref.reshape(n, -1), axis=1)


def test_short_groups_hold_the_float32_tolerance_on_structured_parameters():
    for T in (8, 16):
        for k in (1, 2, 3):
            assert errors(400, T, k).max() < 2e-5, (T, k)


def test_the_product_over_the_whole_horizon_does_not():
    e = errors(400, 8, 8)
    assert (e > 1e-4).mean() > 0.05 and e.max() > 1e-2


def test_cheaper_control_breaks_groups_of_three():
    assert (errors(400, 16, 3, rinv_scale=30.0) > 5e-5).mean() > 0.5
    assert errors(400, 16, 1, rinv_scale=30.0).max() < 1e-4     # one factor per group: the Riccati recursion
