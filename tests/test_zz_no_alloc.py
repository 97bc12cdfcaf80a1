"""The entry point that allocates nothing (ttc_lqr_solve_noalloc), called through the C ABI: two calls in a row,
the second on a smaller input, each checked against ttc_lqr_solve on the same inputs.  The same kernel runs on
the same grid, only the workspace differs (the library's fixed scratch array instead of a caller's buffer), so
the outputs must agree bit for bit; both are also held to the oracle's tolerance."""
import ctypes

import pytest
import torch

from paper_2603_09221_amd import binding, synth
from tests.parity import oracle_solve, solve_errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def outputs(n, d):
    f32 = dict(dtype=torch.float32, device=DEV)
    return {"P0": torch.full((n, d, d), float("nan"), **f32), "K0": torch.full((n, d, d), float("nan"), **f32),
            "u0": torch.full((n, d), float("nan"), **f32), "value": torch.full((n,), float("nan"), **f32),
            "info": torch.full((n,), -1, dtype=torch.int32, device=DEV)}


def call_noalloc(lib, b, out):
    prob = binding.make_problem(b.A, b.B, b.Q, b.R, None, b.x0, b.T)
    sol = binding.Solution(*(out[k].data_ptr() for k in ("P0", "K0", "u0", "value", "info")))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return lib.ttc_lqr_solve_noalloc(ctypes.byref(prob), ctypes.byref(sol), stream)


def test_two_calls_in_a_row_second_one_smaller():
    lib = binding.load()
    assert lib.ttc_lqr_noalloc_scratch_bytes() == 24 << 20
    for n, d, T, seed in ((700, 128, 6, 1), (37, 128, 5, 2), (900, 64, 7, 3), (5, 32, 4, 4), (3100, 16, 8, 5)):
        b = synth.make_batch(n, d, d, T, seed=seed, device=DEV)
        out = outputs(n, d)
        assert call_noalloc(lib, b, out) == binding.TTC_OK
        torch.cuda.synchronize()
        ref = binding.ttc_lqr_solve(b.A, b.B, b.Q, b.R, None, b.x0, T)
        torch.cuda.synchronize()
        assert int(out["info"].abs().max()) == 0
        for k in ("P0", "K0", "u0", "value"):
            assert torch.equal(out[k], ref[k]), (n, d, k)
        for k, v in solve_errors(out, oracle_solve(b)).items():
            assert v <= 1e-4, (n, d, k, v)


def test_rejections_launch_nothing():
    lib = binding.load()
    b = synth.make_batch(8, 64, 64, 4, seed=6, device=DEV)
    out = outputs(8, 64)
    prob = binding.make_problem(b.A, b.B, b.Q, b.R, None, b.x0, b.T, flags=binding.TTC_FLAG_DOUBLING)
    sol = binding.Solution(*(out[k].data_ptr() for k in ("P0", "K0", "u0", "value", "info")))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert lib.ttc_lqr_solve_noalloc(ctypes.byref(prob), ctypes.byref(sol), stream) == binding.TTC_ERR_UNSUPPORTED
    prob = binding.make_problem(b.A, b.B, b.Q, b.R, None, b.x0, 0)
    assert lib.ttc_lqr_solve_noalloc(ctypes.byref(prob), ctypes.byref(sol), stream) == binding.TTC_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.isnan(out["u0"]).all() and int((out["info"] != -1).sum()) == 0
