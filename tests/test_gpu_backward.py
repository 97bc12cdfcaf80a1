"""GPU parity of the backward pass (ttc_lqr_backward, ttc_lqr_backward_tv) against the gradient oracle (Thm 3.2
written out in float64), element by element on the same seeded inputs.  Tolerance 2e-5 per problem on every
gradient (norm-wise and element-wise): the gradients are bilinear in two closed-loop trajectories whose float32
errors add up over the horizon."""
import numpy as np
import pytest
import torch

from oracle import lqr_grad_oracle as go
from paper_2603_09221_amd import binding, synth
from tests.parity import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-5


def draw_g(n, m, seed):
    gen = torch.Generator(device="cpu").manual_seed(seed)
    return torch.randn((n, m), generator=gen).to(DEV)


def check(out, ref, keys, tol=TOL):
    assert int(out["info"].abs().max()) == 0
    errs = {k: float(rel_err(out[k].cpu().numpy().reshape(len(ref[k]), -1), ref[k].reshape(len(ref[k]), -1)).max())
            for k in keys}
    print({k: "%.1e" % v for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)


@pytest.mark.parametrize("d,T,n", [(16, 8, 70), (16, 1, 5), (16, 2, 9), (32, 5, 40), (64, 6, 300), (128, 4, 9),
                                    (128, 9, 270)])
def test_time_heterogeneous_gradients(d, T, n):
    b = synth.make_tv_batch(n, d, d, T, seed=d + T, device=DEV)
    g = draw_g(n, d, 3)
    out = binding.ttc_lqr_backward_tv(b.A, b.B, b.Q, b.R, b.x0, g)
    torch.cuda.synchronize()
    ref = go.lqr_gradients_tv(*b.numpy64(), g.cpu().double().numpy())
    check(out, ref, ("gA", "gB", "gQ", "gR", "gx0"))


@pytest.mark.parametrize("d,T,n", [(16, 8, 64), (64, 8, 200), (128, 16, 40), (32, 1, 7)])
def test_time_invariant_gradients(d, T, n):
    b = synth.make_batch(n, d, d, T, seed=d + T, device=DEV)
    g = draw_g(n, d, 4)
    A, B, Q, R, x0 = b.numpy64()
    out = binding.ttc_lqr_backward(b.A, b.B, b.Q, b.R, None, b.x0, T, g)
    torch.cuda.synchronize()
    ref = go.lqr_gradients(A, B, Q, R, None, x0, T, g.cpu().double().numpy())
    check(out, ref, ("gA", "gB", "gQ", "gR", "gx0"))
    assert "gQT" not in out
    QT = (1.5 * b.Q + 0.2 * torch.eye(d, device=DEV)).contiguous()
    out = binding.ttc_lqr_backward(b.A, b.B, b.Q, b.R, QT, b.x0, T, g)
    torch.cuda.synchronize()
    ref = go.lqr_gradients(A, B, Q, R, QT.cpu().double().numpy(), x0, T, g.cpu().double().numpy())
    keys = ("gA", "gB", "gR", "gQT", "gx0") + (("gQ",) if T > 1 else ())
    check(out, ref, keys)
    if T == 1:
        assert float(out["gQ"].abs().max()) == 0.0      # nothing is charged at Q when the horizon is one step


def test_gradient_of_the_initial_state_is_the_transposed_gain_of_the_forward_pass():
    b = synth.make_batch(50, 64, 64, 7, seed=2, device=DEV)
    g = draw_g(50, 64, 5)
    bw = binding.ttc_lqr_backward(b.A, b.B, b.Q, b.R, None, b.x0, b.T, g)
    fw = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T)
    torch.cuda.synchronize()
    want = torch.einsum("nij,ni->nj", fw["K0"], g)
    assert float(rel_err(bw["gx0"].cpu().numpy(), want.cpu().numpy()).max()) <= 1e-4


def test_bf16_inputs_and_shared_matrices():
    n, d, T = 30, 64, 6
    b = synth.make_tv_batch(n, d, d, T, seed=9, device=DEV, dtype="bf16")
    g = draw_g(n, d, 6)
    out = binding.ttc_lqr_backward_tv(b.A, b.B, b.Q, b.R, b.x0, g)
    torch.cuda.synchronize()
    ref = go.lqr_gradients_tv(*b.numpy64(), g.cpu().double().numpy())     # the oracle consumes the rounded values
    check(out, ref, ("gA", "gB", "gQ", "gR", "gx0"), tol=2e-3)
    f = synth.make_tv_batch(n, d, d, T, seed=10, device=DEV)
    A0 = f.A[:1].contiguous().expand(n, -1, -1, -1)                            # one A sequence shared by all problems
    out = binding.ttc_lqr_backward_tv(A0, f.B, f.Q, f.R, f.x0, g)
    torch.cuda.synchronize()
    A, B, Q, R, x0 = f.numpy64()
    ref = go.lqr_gradients_tv(np.repeat(A[:1], n, axis=0), B, Q, R, x0, g.cpu().double().numpy())
    check(out, ref, ("gA", "gB", "gQ", "gR", "gx0"))


def test_breakdown_and_argument_errors():
    n, d, T = 6, 16, 4
    b = synth.make_tv_batch(n, d, d, T, seed=11, device=DEV)
    g = draw_g(n, d, 7)
    R = b.R.clone()
    R[2, 1] = -100.0 * torch.eye(d, device=DEV)          # S_1 not positive definite for problem 2
    out = binding.ttc_lqr_backward_tv(b.A, b.B, b.Q, R, b.x0, g)
    torch.cuda.synchronize()
    info = out["info"].cpu().numpy()
    assert info[2] != 0 and (np.delete(info, 2) == 0).all()
    assert torch.isnan(out["gx0"][2]).all() and torch.isnan(out["gA"][2]).all()
    good = [0, 1, 3, 4, 5]
    A, B, Q, Rn, x0 = (x[good] for x in b.numpy64())
    ref = go.lqr_gradients_tv(A, B, Q, Rn, x0, g.cpu().double().numpy()[good])
    assert float(rel_err(out["gA"][good].cpu().numpy().reshape(5, -1), ref["gA"].reshape(5, -1)).max()) <= TOL
    with pytest.raises(binding.TtcError):
        binding.ttc_lqr_backward_tv(b.A, b.B, b.Q, b.R, b.x0, g, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    e = binding.ttc_lqr_backward_tv(b.A[:0], b.B[:0], b.Q[:0], b.R[:0], b.x0[:0], g[:0])
    assert e["gx0"].shape == (0, d)
