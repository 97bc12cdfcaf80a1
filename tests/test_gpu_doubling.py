"""GPU parity of the long-horizon (squaring) path, TTC_FLAG_DOUBLING, against the CPU float64 oracle:
same inputs, same outputs and same tolerances as the default path (relative error <= 1e-4 for float32
inputs, <= 2e-2 for bfloat16 inputs, on P0, K0, u0 and the value, per problem)."""
import numpy as np
import pytest
import torch

from paper_2603_09221_amd import binding, synth
from tests.parity import oracle_solve, rel_err, solve_errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DBL = binding.TTC_FLAG_DOUBLING
TOL_F32, TOL_BF16 = 1e-4, 2e-2


def check(batch, tol, QT=None, flag=False):
    flags = DBL | (binding.TTC_FLAG_STAGE_COST_AT_X0 if flag else 0)
    out = binding.ttc_lqr_solve(batch.A, batch.B, batch.Q, batch.R, QT, batch.x0, batch.T, flags=flags)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0
    errs = solve_errors(out, oracle_solve(batch, QT=QT, flag=flag))
    print({k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)
    return out


@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 6, 7, 8, 11, 16, 21])
def test_every_bit_pattern_of_the_horizon(T):
    """Q_T = Q: T maps applied to 0.  Covers powers of two (squarings only), all-ones patterns and mixed ones."""
    check(synth.make_batch(70, 16, 16, T, seed=T, device=DEV), TOL_F32)
    check(synth.make_batch(5, 64, 64, T, seed=100 + T, device=DEV), TOL_F32)


@pytest.mark.parametrize("T", [1, 2, 3, 5, 8, 16, 17])
def test_given_terminal_cost(T):
    """A separate Q_T: T-1 maps applied to Q_T (T = 1: none at all), with and without the stage cost at x0."""
    b = synth.make_batch(40, 32, 32, T, seed=T, device=DEV)
    g = torch.Generator().manual_seed(T)
    L = torch.randn((40, 32, 32), generator=g).to(DEV)
    QT = (L @ L.transpose(1, 2) / 64 + 0.05 * torch.eye(32, device=DEV)).contiguous()
    check(b, TOL_F32, QT=QT)
    check(b, TOL_F32, QT=QT, flag=True)


def test_aliased_terminal_cost_is_recognised():
    """Passing Q itself as Q_T must give bit-identical results to passing no Q_T."""
    b = synth.make_batch(24, 64, 64, 12, seed=2, device=DEV)
    a = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T, flags=DBL)
    c = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, b.Q, b.x0, b.T, flags=DBL)
    torch.cuda.synchronize()
    assert torch.equal(a["P0"], c["P0"]) and torch.equal(a["u0"], c["u0"])


@pytest.mark.parametrize("d,T,n", [(128, 16, 300), (128, 13, 20), (128, 1, 9), (64, 64, 600), (32, 40, 37)])
def test_large_shapes_and_ragged_batches(d, T, n):
    check(synth.make_batch(n, d, d, T, seed=d + T, device=DEV), TOL_F32)


def test_long_horizon_config3_sample():
    c = synth.CONFIGS["long_horizon"]
    b = synth.make_batch(96, c["d"], c["m"], c["T"], seed=0, device=DEV, rho=c["rho"])
    check(b, TOL_F32)
    b = synth.make_batch(16, c["d"], c["m"], 1000, seed=1, device=DEV, rho=c["rho"])
    check(b, TOL_F32)     # ten squarings: converged to the stationary solution


def test_agrees_with_default_path():
    b = synth.make_batch(64, 128, 128, 16, seed=3, device=DEV)
    a = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T)
    c = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T, flags=DBL)
    torch.cuda.synchronize()
    for k in ("P0", "K0", "u0"):
        assert rel_err(a[k].cpu().numpy(), c[k].double().cpu().numpy()).max() <= 2e-4


def test_bf16_inputs():
    for d, T, n in [(16, 8, 64), (64, 8, 64), (128, 32, 24)]:
        check(synth.make_batch(n, d, d, T, seed=8, device=DEV, dtype="bf16"), TOL_BF16)


def test_shared_matrices_stride_zero():
    b = synth.make_batch(50, 32, 32, 9, seed=7, device=DEV)
    A0, R0 = b.A[:1].contiguous(), b.R[:1].contiguous()
    shared = synth.LqrBatch(A0.expand(50, -1, -1), b.B, b.Q, R0.expand(50, -1, -1), b.x0, b.T)
    out = binding.ttc_lqr_solve(shared.A, shared.B, shared.Q, shared.R, None, shared.x0, shared.T, flags=DBL)
    ref = oracle_solve(synth.LqrBatch(A0.repeat(50, 1, 1), b.B, b.Q, R0.repeat(50, 1, 1), b.x0, b.T))
    for k, v in solve_errors(out, ref).items():
        assert v <= TOL_F32, (k, v)


def test_singular_A_is_fine_here():
    """No A^{-1} on this path: a singular A is an ordinary problem (the default path reports info = 2)."""
    b = synth.make_batch(6, 16, 16, 6, seed=10, device=DEV)
    A = b.A.clone()
    A[2, :, 3] = 0.0
    check(synth.LqrBatch(A, b.B, b.Q, b.R, b.x0, b.T), TOL_F32)


def test_info_reports_breakdown():
    b = synth.make_batch(6, 16, 16, 4, seed=10, device=DEV)
    R = b.R.clone()
    R[4] = 0.0                                  # R not positive definite: the first solve must fail
    out = binding.ttc_lqr_solve(b.A, b.B, b.Q, R, None, b.x0, b.T, flags=DBL)
    info = out["info"].cpu().numpy()
    assert info[4] == 1 and (np.delete(info, 4) == 0).all()
    assert torch.isnan(out["u0"][4]).all() and torch.isnan(out["P0"][4]).all()
    good = [0, 1, 2, 3, 5]
    ref = oracle_solve(b.take(torch.tensor(good, device=DEV)))
    assert rel_err(out["u0"][good].cpu().numpy(), ref["u0"]).max() <= TOL_F32


def test_determinism_and_optional_outputs():
    b = synth.make_batch(33, 64, 64, 24, seed=11, device=DEV)
    full = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T, flags=DBL)
    slim = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T, flags=DBL, want_P0=False, want_K0=False)
    again = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T, flags=DBL)
    torch.cuda.synchronize()
    assert "P0" not in slim and torch.equal(slim["u0"], full["u0"]) and torch.equal(slim["value"], full["value"])
    assert torch.equal(again["P0"], full["P0"]) and torch.equal(again["K0"], full["K0"])
