"""GPU parity of the time-heterogeneous solve (ttc_lqr_solve_tv) against the CPU float64 oracle
(oracle.lqr_oracle.riccati_solve_tv), element by element on the same seeded inputs; tolerances as for the
time-invariant solve (1e-4 float32 inputs, 2e-2 bfloat16 inputs; per problem, Frobenius / 2-norm)."""
import numpy as np
import pytest
import torch

from oracle import lqr_oracle
from paper_2603_09221_amd import binding, synth
from tests.parity import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_F32, TOL_BF16 = 1e-4, 2e-2


def errors(out, batch):
    ref = lqr_oracle.riccati_solve_tv(*batch.numpy64())
    return {k: float(rel_err(out[k].detach().cpu().numpy(), ref[k]).max()) for k in ("P0", "K0", "u0", "value")}


def check(batch, tol):
    out = binding.ttc_lqr_solve_tv(batch.A, batch.B, batch.Q, batch.R, batch.x0)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0
    errs = errors(out, batch)
    print({k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)
    return out


@pytest.mark.parametrize("d,T,n", [(16, 1, 5), (16, 8, 70), (32, 5, 37), (64, 8, 300), (128, 1, 3), (128, 6, 20),
                                    (128, 16, 260), (64, 40, 17)])
def test_shapes_horizons_and_ragged_batches(d, T, n):
    check(synth.make_tv_batch(n, d, d, T, seed=d + T, device=DEV), TOL_F32)


def test_d16_large_batches_four_problems_per_wavefront():
    """From 24 x CUs problems on, d = 16 runs four problems per wavefront: ragged last quad, bfloat16 inputs, a
    horizon of one, and a breakdown that must stay with its own problem."""
    n = 6144 + 37
    b = synth.make_tv_batch(n, 16, 16, 6, seed=21, device=DEV)
    out = check(b, TOL_F32)
    check(synth.make_tv_batch(n, 16, 16, 1, seed=22, device=DEV), TOL_F32)
    check(synth.make_tv_batch(n + 2, 16, 16, 9, seed=23, device=DEV, dtype="bf16"), TOL_BF16)
    R = b.R.clone()
    R[1001, 2] = -100.0 * torch.eye(16, device=DEV)        # S not positive definite at step 2, the fourth solve
    bad = binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, R, b.x0)
    info = bad["info"].cpu().numpy()
    assert info[1001] == 4 and (np.delete(info, 1001) == 0).all()
    keep = torch.tensor([1000, 1002, 1003, n - 1], device=DEV)
    assert torch.equal(bad["u0"][keep], out["u0"][keep]) and torch.isnan(bad["u0"][1001]).all()


def test_bf16_inputs():
    for d, T, n in [(16, 8, 64), (64, 8, 64), (128, 12, 24)]:
        check(synth.make_tv_batch(n, d, d, T, seed=8, device=DEV, dtype="bf16"), TOL_BF16)


def test_constant_steps_agree_with_the_time_invariant_solve():
    """Step stride 0 (one matrix shared by all steps) turns the call into the time-invariant problem."""
    n, d, T = 40, 64, 7
    b = synth.make_batch(n, d, d, T, seed=3, device=DEV)
    ex = lambda M: M[:, None].expand(n, T, *M.shape[1:])
    out = binding.ttc_lqr_solve_tv(ex(b.A), ex(b.B), ex(b.Q), ex(b.R), b.x0)
    ti = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, T)
    torch.cuda.synchronize()
    A, B, Q, R, x0 = b.numpy64()
    ref = lqr_oracle.riccati_solve(A, B, Q, R, None, x0, T)
    for k in ("P0", "K0", "u0", "value"):
        assert rel_err(out[k].cpu().numpy(), ref[k]).max() <= TOL_F32
        assert rel_err(out[k].cpu().numpy(), ti[k].double().cpu().numpy()).max() <= 2e-4


def test_padded_strides_and_singular_A():
    n, d, T = 30, 32, 6
    b = synth.make_tv_batch(n, d, d, T, seed=5, device=DEV)
    A = b.A.clone()
    A[:, 2, :, 4] = 0.0                                    # a singular A_t is an ordinary problem here
    b = synth.LqrTvBatch(A, b.B, b.Q, b.R, b.x0)

    def padded(t, pad_step, pad_prob):
        """The same values with unused (NaN) elements after every matrix and after every problem."""
        step = t[0, 0].numel() + pad_step
        buf = torch.full((n, T * step + pad_prob), float("nan"), dtype=t.dtype, device=DEV)
        v = torch.as_strided(buf, t.shape, (buf.stride(0), step, t.shape[3], 1))
        v.copy_(t)
        return v

    p = synth.LqrTvBatch(padded(b.A, 8, 4), padded(b.B, 4, 8), padded(b.Q, 12, 0), padded(b.R, 0, 16), b.x0)
    assert torch.equal(p.A, b.A) and p.A.stride(1) == d * d + 8
    out = binding.ttc_lqr_solve_tv(p.A, p.B, p.Q, p.R, p.x0)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0
    for k, v in errors(out, b).items():
        assert v <= TOL_F32, (k, v)


def test_info_reports_breakdown_and_outputs_are_optional():
    b = synth.make_tv_batch(6, 16, 16, 4, seed=10, device=DEV)
    R = b.R.clone()
    R[4, 3] = -100.0 * torch.eye(16, device=DEV)           # S = R + B^T P B not positive definite at the last step
    out = binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, R, b.x0, want_P0=False)
    info = out["info"].cpu().numpy()
    assert info[4] == 1 and (np.delete(info, 4) == 0).all() and "P0" not in out
    assert torch.isnan(out["u0"][4]).all()
    good = torch.tensor([0, 1, 2, 3, 5], device=DEV)
    ref = lqr_oracle.riccati_solve_tv(*b.take(good).numpy64())
    assert rel_err(out["u0"][good].cpu().numpy(), ref["u0"]).max() <= TOL_F32


def test_empty_batch():
    b = synth.make_tv_batch(1, 16, 16, 3, seed=0, device=DEV)
    out = binding.ttc_lqr_solve_tv(b.A[:0], b.B[:0], b.Q[:0], b.R[:0], b.x0[:0])
    assert out["u0"].shape == (0, 16)


# ---------------------------------------------------------------- roll-out
def rollout_check(batch, tol):
    out = binding.ttc_lqr_rollout_tv(batch.A, batch.B, batch.Q, batch.R, batch.x0)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0
    U, X, cost = lqr_oracle.riccati_rollout_tv(*batch.numpy64())
    errs = {"U": rel_err(out["U"].cpu().numpy(), U).max(), "X": rel_err(out["X"].cpu().numpy(), X).max(),
            "cost": rel_err(out["cost"].cpu().numpy(), cost).max()}
    print({k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)
    assert torch.equal(out["X"][:, 0], batch.x0.float())
    return out


@pytest.mark.parametrize("d,T,n", [(16, 8, 256), (16, 1, 3), (32, 5, 40), (64, 8, 300), (128, 16, 20)])
def test_rollout_matches_oracle(d, T, n):
    rollout_check(synth.make_tv_batch(n, d, d, T, seed=20 + d, device=DEV), TOL_F32)


def test_rollout_cost_equals_solve_value_and_first_control():
    b = synth.make_tv_batch(48, 64, 64, 6, seed=31, device=DEV)
    ro = rollout_check(b, TOL_F32)
    so = binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, b.R, b.x0)
    torch.cuda.synchronize()
    assert rel_err(ro["cost"].cpu().numpy(), so["value"].double().cpu().numpy()).max() <= 2e-4
    assert rel_err(ro["U"][:, 0].cpu().numpy(), so["u0"].double().cpu().numpy()).max() <= 2e-4


def test_rollout_bf16_and_breakdown():
    rollout_check(synth.make_tv_batch(24, 128, 128, 8, seed=8, device=DEV, dtype="bf16"), TOL_BF16)
    b = synth.make_tv_batch(6, 16, 16, 4, seed=10, device=DEV)
    R = b.R.clone()
    R[4, 3] = -100.0 * torch.eye(16, device=DEV)
    out = binding.ttc_lqr_rollout_tv(b.A, b.B, b.Q, R, b.x0)
    info = out["info"].cpu().numpy()
    assert info[4] == 1 and (np.delete(info, 4) == 0).all()
    assert torch.isnan(out["U"][4]).all() and torch.isnan(out["cost"][4])
