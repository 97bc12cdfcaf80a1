"""GPU parity of ttc_lqr_rollout (Alg. 1 forward loop) against the oracle's closed-loop roll-out."""
import numpy as np
import pytest
import torch

from oracle import lqr_oracle
from paper_2603_09221_amd import binding, synth
from tests.parity import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def rollout_check(batch, tol, QT=None, flag=False):
    flags = binding.TTC_FLAG_STAGE_COST_AT_X0 if flag else 0
    out = binding.ttc_lqr_rollout(batch.A, batch.B, batch.Q, batch.R, QT, batch.x0, batch.T, flags=flags)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0
    A, B, Q, R, x0 = batch.numpy64()
    QT64 = None if QT is None else QT.cpu().double().numpy()
    U, X, cost = lqr_oracle.riccati_rollout(A, B, Q, R, QT64, x0, batch.T, stage_cost_at_x0=flag)
    errs = {"U": rel_err(out["U"].cpu().numpy(), U).max(), "X": rel_err(out["X"].cpu().numpy(), X).max(),
            "cost": rel_err(out["cost"].cpu().numpy(), cost).max()}
    print({k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)
    assert torch.equal(out["X"][:, 0], batch.x0.float())
    return out


@pytest.mark.parametrize("d,T,n", [(16, 8, 256), (16, 1, 3), (32, 5, 40), (64, 8, 300), (128, 16, 20)])
def test_rollout_matches_oracle(d, T, n):
    rollout_check(synth.make_batch(n, d, d, T, seed=20 + d, device=DEV), 1e-4)


def test_rollout_cost_equals_solve_value_and_first_control():
    b = synth.make_batch(48, 64, 64, 6, seed=31, device=DEV)
    QT = (1.5 * b.Q).contiguous()
    for flag in (False, True):
        ro = rollout_check(b, 1e-4, QT=QT, flag=flag)
        so = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, QT, b.x0, b.T,
                                   flags=binding.TTC_FLAG_STAGE_COST_AT_X0 if flag else 0)
        torch.cuda.synchronize()
        assert rel_err(ro["cost"].cpu().numpy(), so["value"].cpu().numpy()).max() <= 1e-4
        assert rel_err(ro["U"][:, 0].cpu().numpy(), so["u0"].cpu().numpy()).max() <= 1e-4


def test_rollout_bf16_inputs():
    rollout_check(synth.make_batch(32, 64, 64, 8, seed=33, device=DEV, dtype="bf16"), 2e-2)
