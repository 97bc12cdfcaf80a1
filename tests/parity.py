"""Shared helpers of the GPU parity tests: per-problem errors against the CPU oracle, in norm and element
by element."""
import numpy as np

from oracle import lqr_oracle
from paper_2603_09221_amd import errors

SOLVE_KEYS = ("P0", "K0", "u0", "value")


def oracle_solve(batch, QT=None, flag=False):
    A, B, Q, R, x0 = batch.numpy64()
    QT64 = None if QT is None else QT.detach().to("cpu").double().numpy()
    return lqr_oracle.riccati_solve(A, B, Q, R, QT64, x0, batch.T, stage_cost_at_x0=flag)


def rel_err(got, want):
    """Per-problem error: the larger of the norm-wise relative error (Frobenius / 2-norm over the trailing
    axes) and the element-wise one (max |difference| over max |reference|), so that a single wrong entry
    fails a test even where it is a negligible share of the norm."""
    return np.maximum(errors.rel_err(got, want), errors.elem_err(got, want))


def _np(x):
    return x.detach().cpu().numpy() if hasattr(x, "detach") else np.asarray(x)


def max_errors(out, ref, keys=SOLVE_KEYS):
    """Worst problem's error per output, the larger of the norm-wise and the element-wise measure."""
    errs = {}
    for k in keys:
        got, want = _np(out[k]), ref[k]
        errs[k] = float(rel_err(got, want).max())
    return errs


def solve_errors(out, ref):
    """max over problems of the error of P0, K0, u0, value (norm-wise and element-wise, whichever is larger)."""
    return max_errors(out, ref, SOLVE_KEYS)
