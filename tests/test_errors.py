"""The error measures of the parity tests (CPU): the element-wise one must catch what the norm hides."""
import numpy as np

from paper_2603_09221_amd.errors import elem_err, rel_err
from tests import parity


def test_one_wrong_small_entry_fails_elementwise_but_not_in_norm():
    rng = np.random.default_rng(0)
    want = rng.standard_normal((3, 128, 128)) * 1e-3
    want[:, np.arange(128), np.arange(128)] += 10.0          # a dominant diagonal, as a value matrix has
    got = want.copy()
    got[1, 5, 77] += 3e-3                                    # 300 % of that entry, 0.03 % of the largest one
    assert rel_err(got, want).max() < 1e-4                   # invisible in the Frobenius norm
    assert elem_err(got, want)[1] > 2.9e-4 and elem_err(got, want)[[0, 2]].max() == 0.0
    assert parity.rel_err(got, want)[1] > 1e-4               # the tests' measure takes the larger of the two


def test_scalars_and_vectors():
    assert np.allclose(rel_err(np.array([1.1, 2.0]), np.array([1.0, 2.0])), [0.1, 0.0])
    assert np.allclose(elem_err(np.array([[1.0, 2.2]]), np.array([[1.0, 2.0]])), [0.1])
    assert np.allclose(rel_err(np.array([[3.0, 4.0]]), np.array([[3.0, 0.0]])), [4.0 / 3.0])
