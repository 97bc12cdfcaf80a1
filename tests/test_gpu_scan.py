"""GPU parity of the time-heterogeneous solve with the factors composed pairwise over the horizon
(ttc_lqr_solve_tv_scan) against the CPU float64 oracle (oracle.lqr_oracle.riccati_solve_tv): the same result as
the sequential recursion, so the same oracle and the same tolerances (1e-4 float32, 2e-2 bfloat16 inputs)."""
import numpy as np
import pytest
import torch

from oracle import lqr_oracle
from paper_2603_09221_amd import binding, synth
from tests.parity import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_F32, TOL_BF16 = 1e-4, 2e-2


def check(batch, tol):
    out = binding.ttc_lqr_solve_tv_scan(batch.A, batch.B, batch.Q, batch.R, batch.x0)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0
    ref = lqr_oracle.riccati_solve_tv(*batch.numpy64())
    errs = {k: float(rel_err(out[k].detach().cpu().numpy(), ref[k]).max()) for k in ("P0", "K0", "u0", "value")}
    print({k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)
    return out


@pytest.mark.parametrize("d,T,n", [(16, 1, 3), (16, 2, 5), (16, 3, 4), (16, 7, 9), (16, 64, 33), (16, 257, 4),
                                    (32, 20, 6), (64, 33, 5), (128, 5, 2), (128, 16, 3)])
def test_shapes_and_horizons_that_are_not_powers_of_two(d, T, n):
    check(synth.make_tv_batch(n, d, d, T, seed=d + T, device=DEV), TOL_F32)


def test_long_horizon_small_batch():
    """The case the pairwise product is for: 16 problems, 2048 steps each."""
    check(synth.make_tv_batch(16, 16, 16, 2048, seed=5, device=DEV), TOL_F32)


def test_bf16_inputs():
    check(synth.make_tv_batch(8, 16, 16, 12, seed=8, device=DEV, dtype="bf16"), TOL_BF16)
    check(synth.make_tv_batch(4, 64, 64, 9, seed=9, device=DEV, dtype="bf16"), TOL_BF16)


def test_agrees_with_the_sequential_solve_and_isolates_a_breakdown():
    b = synth.make_tv_batch(12, 32, 32, 11, seed=3, device=DEV)
    seq = binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, b.R, b.x0)
    par = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, b.R, b.x0)
    torch.cuda.synchronize()
    for k in ("P0", "K0", "u0", "value"):
        assert float(rel_err(par[k].cpu().numpy(), seq[k].cpu().numpy()).max()) <= 2e-5, k
    R = b.R.clone()
    R[7, 4] = -100.0 * torch.eye(32, device=DEV)      # R_4 of problem 7 is not positive definite
    bad = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, R, b.x0)
    torch.cuda.synchronize()
    info = bad["info"].cpu().numpy()
    assert info[7] == 1 and (np.delete(info, 7) == 0).all()
    keep = torch.tensor([0, 6, 8, 11], device=DEV)
    assert torch.equal(bad["u0"][keep], par["u0"][keep]) and torch.isnan(bad["u0"][7]).all()
    assert torch.isnan(bad["P0"][7]).all()


def test_workspace_is_checked_and_empty_batches_pass():
    b = synth.make_tv_batch(4, 16, 16, 6, seed=1, device=DEV)
    small = torch.empty((4 * 6 * 3 * 256 * 4 - 16,), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.TtcError) as e:
        binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, b.R, b.x0, workspace=small)
    assert e.value.status == binding.TTC_ERR_WORKSPACE
    e0 = synth.make_tv_batch(0, 16, 16, 6, seed=1, device=DEV)
    out = binding.ttc_lqr_solve_tv_scan(e0.A, e0.B, e0.Q, e0.R, e0.x0)
    assert out["u0"].shape == (0, 16)


def check_values(batch, tol):
    """ttc_lqr_tv_scan_values: every P_t (t = 1..T) and every gain K_s (s = 0..T-1) against the oracle's recursion."""
    out = binding.ttc_lqr_tv_scan_values(batch.A, batch.B, batch.Q, batch.R, batch.x0)
    torch.cuda.synchronize()
    P_ref, K_ref = lqr_oracle.riccati_value_matrices_tv(*batch.numpy64()[:4])
    n, T = batch.A.shape[0], batch.A.shape[1]
    P = out["P"].cpu().numpy()
    K = out["K"].cpu().numpy()
    eP = max(float(rel_err(P[:, k], P_ref[k + 1]).max()) for k in range(T))
    eK = max(float(rel_err(K[:, s], K_ref[s]).max()) for s in range(T))
    print(f"P {eP:.2e} K {eK:.2e}")
    assert eP <= tol and eK <= tol, (eP, eK)
    return out


@pytest.mark.parametrize("d,T,n", [(16, 1, 3), (16, 2, 5), (16, 3, 4), (16, 7, 9), (16, 64, 33), (16, 300, 3),
                                    (32, 20, 6), (64, 33, 5), (128, 5, 2), (128, 16, 3)])
def test_all_value_matrices_and_gains(d, T, n):
    check_values(synth.make_tv_batch(n, d, d, T, seed=2 * d + T, device=DEV), TOL_F32)


def test_all_value_matrices_long_horizon_small_batch():
    check_values(synth.make_tv_batch(16, 16, 16, 2048, seed=6, device=DEV), TOL_F32)


def test_values_bf16_inputs_and_single_outputs():
    b = synth.make_tv_batch(6, 16, 16, 13, seed=4, device=DEV, dtype="bf16")
    check_values(b, TOL_BF16)
    b = synth.make_tv_batch(5, 32, 32, 9, seed=5, device=DEV)
    both = binding.ttc_lqr_tv_scan_values(b.A, b.B, b.Q, b.R, b.x0)
    onlyP = binding.ttc_lqr_tv_scan_values(b.A, b.B, b.Q, b.R, b.x0, want_K=False)
    onlyK = binding.ttc_lqr_tv_scan_values(b.A, b.B, b.Q, b.R, b.x0, want_P=False)
    torch.cuda.synchronize()
    assert "K" not in onlyP and "P" not in onlyK
    assert torch.equal(onlyP["P"], both["P"]) and torch.equal(onlyK["K"], both["K"])
    # the first gain and the first value matrix agree with the reduction's outputs
    red = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, b.R, b.x0)
    torch.cuda.synchronize()
    assert float(rel_err(both["K"][:, 0].cpu().numpy(), red["K0"].cpu().numpy()).max()) <= 1e-6


def test_many_items_at_d16_four_per_wavefront():
    """Rounds with more items than twice the resident workgroups run the kernels that take four items per wavefront
    (d = 16): a ragged last group, terminal elements inside a group, bfloat16 inputs, and a breakdown that must stay
    with its problem."""
    b = synth.make_tv_batch(41, 16, 16, 333, seed=12, device=DEV)      # 13653 items, not a multiple of four
    check(b, TOL_F32)
    check_values(b, TOL_F32)
    check(synth.make_tv_batch(41, 16, 16, 333, seed=13, device=DEV, dtype="bf16"), TOL_BF16)
    good = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, b.R, b.x0)
    R = b.R.clone()
    R[17, 200] = -100.0 * torch.eye(16, device=DEV)
    bad = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, R, b.x0)
    torch.cuda.synchronize()
    info = bad["info"].cpu().numpy()
    assert info[17] == 1 and (np.delete(info, 17) == 0).all()
    keep = torch.tensor([k for k in range(41) if k != 17], device=DEV)
    assert torch.equal(bad["u0"][keep], good["u0"][keep]) and torch.isnan(bad["u0"][17]).all()


def test_many_items_even_horizon():
    """As test_many_items_at_d16_four_per_wavefront with an even horizon (no odd element left over in the first
    round) and a ragged last group of pairs."""
    b = synth.make_tv_batch(41, 16, 16, 334, seed=14, device=DEV)      # 6847 pairs, not a multiple of four
    check(b, TOL_F32)
    check_values(b, TOL_F32)
    check(synth.make_tv_batch(41, 16, 16, 334, seed=15, device=DEV, dtype="bf16"), TOL_BF16)
    good = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, b.R, b.x0)
    R = b.R.clone()
    R[23, 201] = -100.0 * torch.eye(16, device=DEV)
    bad = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, R, b.x0)
    torch.cuda.synchronize()
    info = bad["info"].cpu().numpy()
    assert info[23] == 1 and (np.delete(info, 23) == 0).all()
    keep = torch.tensor([k for k in range(41) if k != 23], device=DEV)
    assert torch.equal(bad["u0"][keep], good["u0"][keep]) and torch.isnan(bad["u0"][23]).all()
