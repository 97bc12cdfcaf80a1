"""Error measures between two stacks of per-problem results (plain numpy; none of the method's arithmetic).

Used by the parity tests and by the benchmark's parity report.
"""
import numpy as np


def rel_err(got, want):
    """Per-problem relative error in norm: Frobenius / 2-norm over all trailing axes, |.| for scalars."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    ax = tuple(range(1, want.ndim))
    if ax:
        num = np.sqrt(((got - want) ** 2).sum(axis=ax))
        den = np.sqrt((want ** 2).sum(axis=ax))
    else:
        num, den = np.abs(got - want), np.abs(want)
    return num / np.maximum(den, 1e-300)


def elem_err(got, want):
    """Per-problem element-wise error: max_ij |got_ij - want_ij| / max_ij |want_ij| (so that one wrong entry,
    however small its share of the norm, shows)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    ax = tuple(range(1, want.ndim))
    if ax:
        num = np.abs(got - want).max(axis=ax)
        den = np.abs(want).max(axis=ax)
    else:
        num, den = np.abs(got - want), np.abs(want)
    return num / np.maximum(den, 1e-300)
