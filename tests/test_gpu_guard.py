"""The default path's accuracy must be a property of the code, not of the benchmark generator: inputs whose pair
[Y1 Y2] (Thm 3.3) grows faster than the grouping assumes are caught by the growth guard and solved by the
recursion of Prop. 3.1 in its printed form.  Sweep of cost scales and open-loop spectral radii against the oracle."""
import itertools

import numpy as np
import pytest
import torch

from paper_2603_09221_amd import binding, synth
from tests.parity import oracle_solve, rel_err, solve_errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_F32 = 1e-4


def riccati_float32(A, B, Q, R, T):
    """Prop. 3.1 evaluated in float32 by numpy (Cholesky of S): what float32 arithmetic can deliver on these
    inputs, as a yardstick for the cases whose conditioning puts 1e-4 out of reach."""
    f = np.float32
    A, B, Q, R = (x.astype(f) for x in (A, B, Q, R))
    P = Q.copy()
    for t in range(T):
        BtP = np.swapaxes(B, -1, -2) @ P
        S = R + BtP @ B
        F = BtP @ A
        L = np.linalg.cholesky(S)
        W = np.linalg.solve(np.swapaxes(L, -1, -2), np.linalg.solve(L, F)).astype(f)
        P = (np.swapaxes(A, -1, -2) @ P @ A - np.swapaxes(F, -1, -2) @ W).astype(f)
        if t < T - 1:
            P = P + Q
        P = f(0.5) * (P + np.swapaxes(P, -1, -2))
    return P


def solve(b, **kw):
    out = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T, **kw)
    torch.cuda.synchronize()
    return out


SCALES = (1e-2, 1.0, 1e2)


@pytest.mark.parametrize("d,n,T", [(16, 3100, 9), (16, 60, 9), (64, 80, 9), (128, 24, 6)])
@pytest.mark.parametrize("rho", [0.5, None, 1.2])
def test_cost_scales_and_spectral_radii(d, n, T, rho):
    """R and Q scaled by 1e-2 .. 1e2 (all nine combinations), rho(A) from 0.5 to 1.2: 1e-4 with info == 0
    wherever the ratio of the scales is at most 1e2.  At 1e4 (state cost 1e2, control cost 1e-2) P_0 is a small
    difference of large terms in any float32 evaluation; there the bound is four times the error of numpy's
    float32 evaluation of Prop. 3.1 on the same inputs, and at least 1e-4."""
    for qs, rs in itertools.product(SCALES, SCALES):
        b = synth.make_batch(n, d, d, T, seed=int(d + 10 * T), device=DEV, rho=rho, q_scale=qs, r_scale=rs)
        out = solve(b)
        assert int(out["info"].abs().max()) == 0, (qs, rs)
        ref = oracle_solve(b)
        errs = solve_errors(out, ref)
        tol = TOL_F32
        if qs / rs > 1e3:
            A, B, Q, R, _ = b.numpy64()
            m = min(n, 64)
            P32 = riccati_float32(A[:m], B[:m], Q[:m], R[:m], T)
            # P_1-type recursion above charges no cost on x_0 as well: compare its P_0 with the oracle's
            floor = float(rel_err(P32, ref["P0"][:m]).max())
            tol = max(TOL_F32, 4.0 * floor)
        print(d, rho, qs, rs, {k: "%.1e" % v for k, v in errs.items()}, "tol %.1e" % tol)
        for k, v in errs.items():
            assert v <= tol, (d, rho, qs, rs, k, v)


@pytest.mark.parametrize("d,n", [(16, 3100), (16, 40), (64, 64), (128, 20)])
def test_fast_growing_problems_take_the_riccati_recursion(d, n):
    """Cheap control (R scaled by 1e-2): the pair grows a thousandfold per factor, far beyond the guard's limit,
    so every problem must come out as ttc_lqr_solve_tv computes it on the same matrices repeated over the horizon
    (the same code runs: P0 and K0 bit for bit; u0 and value are sums over the wavefronts of a workgroup, and the two
    kernels may be built with different numbers of wavefronts per problem, so these agree to rounding); on the
    benchmark inputs the guard must stay silent and the symplectic path's own results differ from that recursion in
    the last bits."""
    T = 7
    hard = synth.make_batch(n, d, d, T, seed=3, device=DEV, r_scale=1e-2)
    out = solve(hard)
    rep = lambda t: t.unsqueeze(1).expand(-1, T, -1, -1)
    tv = binding.ttc_lqr_solve_tv(rep(hard.A), rep(hard.B), rep(hard.Q), rep(hard.R), hard.x0)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0
    for k in ("P0", "K0"):
        assert torch.equal(out[k], tv[k]), k
    for k in ("u0", "value"):
        assert float(rel_err(out[k].cpu().numpy(), tv[k].cpu().numpy()).max()) <= 2e-6, k
    easy = synth.make_batch(n, d, d, T, seed=3, device=DEV)
    out = solve(easy)
    tv = binding.ttc_lqr_solve_tv(rep(easy.A), rep(easy.B), rep(easy.Q), rep(easy.R), easy.x0)
    torch.cuda.synchronize()
    assert not torch.equal(out["P0"], tv["P0"])
    assert float(rel_err(out["P0"].cpu().numpy(), tv["P0"].cpu().numpy()).max()) <= 1e-4


@pytest.mark.parametrize("d,n", [(16, 2101), (64, 70)])
def test_hard_and_easy_problems_side_by_side(d, n):
    """Every third problem has cheap control; at d = 16 such a problem shares its wavefront with three easy
    ones.  Each problem must be right, with a given terminal cost and the stage-cost flag too."""
    T = 8
    easy = synth.make_batch(n, d, d, T, seed=5, device=DEV)
    hard = synth.make_batch(n, d, d, T, seed=5, device=DEV, r_scale=1e-2)
    pick = (torch.arange(n, device=DEV) % 3 == 1)
    R = torch.where(pick[:, None, None], hard.R, easy.R).contiguous()
    b = synth.LqrBatch(easy.A, easy.B, easy.Q, R, easy.x0, T)
    QT = (1.5 * b.Q + 0.2 * torch.eye(d, device=DEV)).contiguous()
    for qt, flag in ((None, False), (QT, True)):
        out = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, qt, b.x0, T,
                                    flags=binding.TTC_FLAG_STAGE_COST_AT_X0 if flag else 0)
        torch.cuda.synchronize()
        assert int(out["info"].abs().max()) == 0
        for k, v in solve_errors(out, oracle_solve(b, QT=qt, flag=flag)).items():
            assert v <= TOL_F32, (k, v)


def test_breakdown_next_to_a_hard_problem_keeps_its_report():
    """A singular A (set-up breakdown, info = 2, NaN outputs) in the same wavefront as a problem the guard hands
    to the Riccati recursion."""
    n, d, T = 3100, 16, 6
    b = synth.make_batch(n, d, d, T, seed=8, device=DEV)
    A, R = b.A.clone(), b.R.clone()
    A[1001] = 0.0
    R[1002] *= 1e-2
    out = solve(synth.LqrBatch(A, b.B, b.Q, R, b.x0, T))
    info = out["info"].cpu().numpy()
    assert info[1001] == 2 and (np.delete(info, 1001) == 0).all()
    assert torch.isnan(out["u0"][1001]).all() and torch.isnan(out["P0"][1001]).all()
    keep = torch.tensor([1000, 1002, 1003, 5], device=DEV)
    ref = oracle_solve(synth.LqrBatch(A, b.B, b.Q, R, b.x0, T).take(keep))
    sub = {k: out[k][keep] for k in ("P0", "K0", "u0", "value")}
    for k, v in solve_errors(sub, ref).items():
        assert v <= TOL_F32, (k, v)
