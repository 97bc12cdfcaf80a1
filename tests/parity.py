"""Shared helpers of the GPU parity tests: per-problem relative errors against the CPU oracle."""
import numpy as np

from oracle import lqr_oracle


def rel_err(got, want):
    """Per-problem relative error: Frobenius / 2-norm over all trailing axes, |.| for scalars."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    ax = tuple(range(1, want.ndim))
    if ax:
        num = np.sqrt(((got - want) ** 2).sum(axis=ax))
        den = np.sqrt((want ** 2).sum(axis=ax))
    else:
        num, den = np.abs(got - want), np.abs(want)
    return num / np.maximum(den, 1e-300)


def oracle_solve(batch, QT=None, flag=False):
    A, B, Q, R, x0 = batch.numpy64()
    QT64 = None if QT is None else QT.detach().to("cpu").double().numpy()
    return lqr_oracle.riccati_solve(A, B, Q, R, QT64, x0, batch.T, stage_cost_at_x0=flag)


def solve_errors(out, ref):
    """max relative error over problems for P0, K0, u0, value."""
    return {k: float(rel_err(out[k].detach().cpu().numpy(), ref[k]).max()) for k in ("P0", "K0", "u0", "value")}
