"""GPU parity: the HIP path, called through the C ABI, against the CPU float64 oracle, element by
element on the same seeded inputs.  Tolerances: relative error <= 1e-4 (float32 inputs) and <= 2e-2
(bfloat16 inputs, float32 accumulation) on P0, K0, u0 and the value, per problem (Frobenius / 2-norm)."""
import numpy as np
import pytest
import torch

from paper_2603_09221_amd import binding, synth
from tests.parity import oracle_solve, rel_err, solve_errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_F32, TOL_BF16 = 1e-4, 2e-2


def run(batch, **kw):
    out = binding.ttc_lqr_solve(batch.A, batch.B, batch.Q, batch.R, kw.pop("QT", None), batch.x0, batch.T, **kw)
    torch.cuda.synchronize()
    return out


def check(batch, tol, QT=None, flag=False, **kw):
    flags = binding.TTC_FLAG_STAGE_COST_AT_X0 if flag else 0
    out = run(batch, QT=QT, flags=flags | kw.pop("flags", 0), **kw)
    assert int(out["info"].abs().max()) == 0
    errs = solve_errors(out, oracle_solve(batch, QT=QT, flag=flag))
    print({k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)
    return errs


def test_config0_tiny_all_problems():
    check(synth.make_config("tiny", device=DEV), TOL_F32)


@pytest.mark.parametrize("d,T,n", [(16, 8, 1), (16, 1, 5), (16, 2, 70), (32, 8, 37), (64, 8, 600), (128, 4, 9),
                                    (128, 16, 300)])
def test_shapes_and_ragged_batches(d, T, n):
    """n spans less than one grid, a ragged tail, and several passes of the persistent workgroups."""
    check(synth.make_batch(n, d, d, T, seed=d + T, device=DEV), TOL_F32)


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_rebase_period(k):
    check(synth.make_batch(64, 64, 64, 8, seed=3, device=DEV), TOL_F32, rebase_every=k)
    check(synth.make_batch(20, 128, 128, 16, seed=4, device=DEV), TOL_F32, rebase_every=k)


def test_pure_symplectic_short_horizon():
    """Alg. 4 as printed (one dense solve for the whole product): accurate only for short horizons."""
    b = synth.make_batch(32, 16, 16, 4, seed=5, device=DEV)
    check(b, 2e-3, flags=binding.TTC_FLAG_PURE_SYMPLECTIC)


@pytest.mark.parametrize("d,n", [(16, 9), (16, 3100), (32, 21), (64, 300), (128, 270)])
@pytest.mark.parametrize("T", [2, 3])
def test_pure_symplectic_row_normalisation_every_size(d, n, T):
    """Alg. 4 with row normalisation after every factor (App. C "Numerical Stability"), at every state size
    (each has its own thread mapping of the normalisation) and over several passes of the persistent grid.
    Two or three factors keep cond(Y1) small enough for the float32 tolerance.  The same product without
    normalisation (one group, rebase_every = T) must agree to rounding: the scales are powers of two, so the
    rows of [Y1 Y2] are the same numbers up to their exponents; the dense solve may then pick other pivots
    (it compares magnitudes across rows), so the two results are close, not bit-identical."""
    b = synth.make_batch(n, d, d, T, seed=40 + d + T, device=DEV)
    check(b, TOL_F32, flags=binding.TTC_FLAG_PURE_SYMPLECTIC)
    pure = run(b, flags=binding.TTC_FLAG_PURE_SYMPLECTIC)
    one_group = run(b, rebase_every=T)
    assert int(pure["info"].abs().max()) == 0 and int(one_group["info"].abs().max()) == 0
    for k in ("P0", "K0", "u0", "value"):
        assert rel_err(pure[k].cpu().numpy(), one_group[k].cpu().numpy()).max() <= 2e-5, k


def test_pure_symplectic_rows_of_very_different_scale():
    """A terminal cost spanning eight orders of magnitude makes the rows of [Y1 Y2] differ by as much; the
    normalisation must bring every row back to order one without changing Y1^{-1} Y2."""
    d, T, n = 64, 2, 40
    b = synth.make_batch(n, d, d, T, seed=77, device=DEV)
    scale = torch.logspace(-4, 4, d, device=DEV)
    QT = (b.Q * scale[None, :, None].sqrt() * scale[None, None, :].sqrt()).contiguous()
    check(b, TOL_F32, QT=QT, flags=binding.TTC_FLAG_PURE_SYMPLECTIC)


def test_terminal_cost_and_stage_flag():
    b = synth.make_batch(40, 64, 64, 6, seed=6, device=DEV)
    QT = (2.0 * b.Q + 0.1 * torch.eye(64, device=DEV)).contiguous()
    check(b, TOL_F32, QT=QT)
    check(b, TOL_F32, QT=QT, flag=True)


def test_shared_matrices_stride_zero():
    b = synth.make_batch(50, 32, 32, 5, seed=7, device=DEV)
    A0, R0 = b.A[:1].contiguous(), b.R[:1].contiguous()
    shared = synth.LqrBatch(A0.expand(50, -1, -1), b.B, b.Q, R0.expand(50, -1, -1), b.x0, b.T)
    out = run(shared)
    ref = oracle_solve(synth.LqrBatch(A0.repeat(50, 1, 1), b.B, b.Q, R0.repeat(50, 1, 1), b.x0, b.T))
    for k, v in solve_errors(out, ref).items():
        assert v <= TOL_F32, (k, v)


def _padded(t, pad):
    """The same values with `pad` unused elements between consecutive problems."""
    n = t.shape[0]
    inner = t[0].numel()
    buf = torch.full((n, inner + pad), float("nan"), dtype=t.dtype, device=t.device)
    buf[:, :inner] = t.reshape(n, inner)
    return buf[:, :inner].view(t.shape)


@pytest.mark.parametrize("d,T,n,flags", [(32, 6, 45, 0), (16, 8, 3100, 0), (64, 9, 30, binding.TTC_FLAG_DOUBLING),
                                         (128, 5, 7, 0)])
def test_padded_problem_strides(d, T, n, flags):
    """Problem-to-problem strides larger than the matrix (and different per argument); the gaps hold NaN."""
    b = synth.make_batch(n, d, d, T, seed=31, device=DEV)
    p = synth.LqrBatch(_padded(b.A, 8), _padded(b.B, 4), _padded(b.Q, 12), _padded(b.R, 8), _padded(b.x0, 3), b.T)
    assert p.A.stride(0) == d * d + 8 and p.x0.stride(0) == d + 3
    out = run(p, flags=flags)
    assert int(out["info"].abs().max()) == 0
    for k, v in solve_errors(out, oracle_solve(b)).items():
        assert v <= TOL_F32, (k, v)


def test_bf16_inputs():
    for d, T, n in [(16, 8, 64), (64, 8, 64), (128, 32, 24)]:
        b = synth.make_batch(n, d, d, T, seed=8, device=DEV, dtype="bf16")
        check(b, TOL_BF16)      # the oracle consumes the same bf16-rounded values


def test_long_horizon_config3_sample():
    c = synth.CONFIGS["long_horizon"]
    b = synth.make_batch(96, c["d"], c["m"], c["T"], seed=0, device=DEV, rho=c["rho"])
    check(b, TOL_F32)


def test_d16_large_batches_four_problems_per_wavefront():
    """From 12 x CUs problems on, d = 16 runs four problems per wavefront: ragged last quad, a given Q_T, the
    stage-cost flag, bfloat16 inputs, a horizon of one, and a breakdown that must stay with its own problem."""
    n = 3072 + 37
    b = synth.make_batch(n, 16, 16, 8, seed=21, device=DEV)
    check(b, TOL_F32)
    QT = (1.5 * b.Q + 0.2 * torch.eye(16, device=DEV)).contiguous()
    check(b, TOL_F32, QT=QT, flag=True)
    check(b, TOL_F32, rebase_every=2)
    check(synth.make_batch(n, 16, 16, 1, seed=22, device=DEV), TOL_F32)
    check(synth.make_batch(n, 16, 16, 4, seed=5, device=DEV), 2e-3, flags=binding.TTC_FLAG_PURE_SYMPLECTIC)
    check(synth.make_batch(n + 1, 16, 16, 12, seed=23, device=DEV, dtype="bf16"), TOL_BF16)
    A = b.A.clone()
    A[1001] = 0.0
    out = run(synth.LqrBatch(A, b.B, b.Q, b.R, b.x0, b.T))
    info = out["info"].cpu().numpy()
    assert info[1001] == 2 and (np.delete(info, 1001) == 0).all()
    assert torch.isnan(out["u0"][1001]).all()
    keep = torch.tensor([1000, 1002, 1003, n - 1], device=DEV)      # its quad neighbours and the ragged tail
    ref = oracle_solve(b.take(keep))
    assert rel_err(out["u0"][keep].cpu().numpy(), ref["u0"]).max() <= TOL_F32


def test_very_long_horizon_keeps_short_groups():
    """Hundreds of factors: the number of groups grows with T (no cap), so every group stays short."""
    check(synth.make_batch(40, 16, 16, 300, seed=12, device=DEV), TOL_F32)
    c = synth.CONFIGS["long_horizon"]
    check(synth.make_batch(12, c["d"], c["m"], 250, seed=13, device=DEV, rho=c["rho"]), TOL_F32)


def test_needs_pivoting():
    """A close to a cyclic shift: its LU has zero leading pivots, so the dense solves must pivot."""
    d, n = 32, 12
    b = synth.make_batch(n, d, d, 5, seed=9, device=DEV)
    shift = torch.roll(torch.eye(d, device=DEV), 1, dims=1)
    A = (0.9 * shift + 0.05 * (b.A - torch.eye(d, device=DEV))).contiguous()
    check(synth.LqrBatch(A, b.B, b.Q, b.R, b.x0, b.T), TOL_F32)


@pytest.mark.parametrize("n", [10, 4100])
def test_needs_pivoting_d16(n):
    """The same at d = 16, where the pivot search prefers the diagonal row when it is large enough (a pivot row in a
    known lane is broadcast without the LDS crossbar) and the choice is made per wavefront: one problem per
    wavefront (small batch), and four per wavefront with every third problem close to a cyclic shift among ordinary
    ones, so that steps of both kinds occur within a wavefront."""
    d = 16
    b = synth.make_batch(n, d, d, 5, seed=19, device=DEV)
    shift = torch.roll(torch.eye(d, device=DEV), 1, dims=1)
    A = b.A.clone()
    A[::3] = 0.9 * shift + 0.05 * (b.A[::3] - torch.eye(d, device=DEV))
    check(synth.LqrBatch(A.contiguous(), b.B, b.Q, b.R, b.x0, b.T), TOL_F32)
    tv = synth.make_tv_batch(n if n < 100 else 4100, d, d, 3, seed=20, device=DEV)
    Atv = tv.A.clone()
    Atv[::3] = 0.9 * shift + 0.05 * (tv.A[::3] - torch.eye(d, device=DEV))
    out = binding.ttc_lqr_solve_tv_scan(Atv.contiguous(), tv.B, tv.Q, tv.R, tv.x0)   # the compositions solve with I + G H
    seq = binding.ttc_lqr_solve_tv(Atv.contiguous(), tv.B, tv.Q, tv.R, tv.x0)
    torch.cuda.synchronize()
    assert int(out["info"].abs().max()) == 0 and int(seq["info"].abs().max()) == 0
    for k in ("P0", "K0", "u0", "value"):
        assert float(rel_err(out[k].cpu().numpy(), seq[k].cpu().numpy()).max()) <= 2e-5, k


def test_info_reports_breakdown():
    b = synth.make_batch(6, 16, 16, 4, seed=10, device=DEV)
    A = b.A.clone()
    A[2] = 0.0                                  # singular A: the A^{-1} solve must fail
    out = run(synth.LqrBatch(A, b.B, b.Q, b.R, b.x0, b.T))
    info = out["info"].cpu().numpy()
    assert info[2] == 2 and (np.delete(info, 2) == 0).all()
    assert torch.isnan(out["u0"][2]).all() and torch.isnan(out["P0"][2]).all()
    good = [0, 1, 3, 4, 5]
    ref = oracle_solve(b.take(torch.tensor(good, device=DEV)))
    assert rel_err(out["u0"][good].cpu().numpy(), ref["u0"]).max() <= TOL_F32


def test_optional_outputs_and_determinism():
    b = synth.make_batch(33, 64, 64, 8, seed=11, device=DEV)
    full = run(b)
    slim = run(b, want_P0=False, want_K0=False)
    assert "P0" not in slim and torch.equal(slim["u0"], full["u0"]) and torch.equal(slim["value"], full["value"])
    again = run(b)
    assert torch.equal(again["P0"], full["P0"]) and torch.equal(again["K0"], full["K0"])


def test_empty_batch():
    b = synth.make_batch(1, 16, 16, 4, seed=0, device=DEV)
    out = binding.ttc_lqr_solve(b.A[:0], b.B[:0], b.Q[:0], b.R[:0], None, b.x0[:0], 4)
    assert out["u0"].shape == (0, 16)


def test_launch_on_a_side_stream():
    """The call runs on the stream it is given; outputs and the workspace the wrapper allocates must be safe
    to use although that stream is not the current one."""
    b = synth.make_batch(300, 128, 128, 6, seed=14, device=DEV)
    ref = run(b)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    out = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, b.T, stream=side)
    junk = [torch.full((1 << 22,), float("nan"), device=DEV) for _ in range(8)]   # allocator traffic on the current stream
    side.synchronize()
    del junk
    for k in ("P0", "K0", "u0", "value"):
        assert torch.equal(out[k], ref[k]), k
    ro = binding.ttc_lqr_rollout(b.A, b.B, b.Q, b.R, None, b.x0, b.T, stream=side)
    junk = [torch.full((1 << 22,), float("nan"), device=DEV) for _ in range(8)]
    side.synchronize()
    del junk
    ro_ref = binding.ttc_lqr_rollout(b.A, b.B, b.Q, b.R, None, b.x0, b.T)
    torch.cuda.synchronize()
    assert torch.equal(ro["U"], ro_ref["U"]) and torch.equal(ro["cost"], ro_ref["cost"])
