"""C-ABI boundary checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest
import torch

from paper_2603_09221_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load()


def header_functions():
    text = open(os.path.join(ROOT, "include", "ttc_lqr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ttc_[a-z_0-9]+)\s*\(", text)))


def test_exports_match_header(lib):
    names = header_functions()
    assert names == sorted(binding.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert binding.ttc_version() >= 100
    texts = {binding.ttc_status_string(s) for s in range(5)}
    assert len(texts) == 5 and all(texts)
    assert binding.ttc_status_string(99) == "unknown status"


def _problem(**kw):
    p = binding.Problem()
    p.n, p.d, p.m, p.T = 4, 16, 16, 8
    fake = 0x1000  # never dereferenced: validation fails or n == 0 before any launch
    p.A = p.B = p.Q = p.R = p.x0 = fake
    p.sA = p.sB = p.sQ = p.sR = 256
    p.sx0 = 16
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def _solve(lib, p, sol=None, ws=0x1000, ws_bytes=1 << 40):
    sol = sol or binding.Solution(0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    return lib.ttc_lqr_solve(ctypes.byref(p), ctypes.byref(sol), ctypes.c_void_p(ws), ws_bytes, None)


def test_argument_validation_without_device(lib):
    assert _solve(lib, _problem(T=0)) == binding.TTC_ERR_INVALID_ARG
    assert _solve(lib, _problem(n=-1)) == binding.TTC_ERR_INVALID_ARG
    assert _solve(lib, _problem(in_dtype=7)) == binding.TTC_ERR_INVALID_ARG
    assert _solve(lib, _problem(flags=64)) == binding.TTC_ERR_INVALID_ARG
    assert _solve(lib, _problem(flags=binding.TTC_FLAG_DOUBLING | binding.TTC_FLAG_PURE_SYMPLECTIC)) \
        == binding.TTC_ERR_INVALID_ARG
    assert _solve(lib, _problem(A=None)) == binding.TTC_ERR_INVALID_ARG
    assert _solve(lib, _problem(A=0x1004)) == binding.TTC_ERR_INVALID_ARG      # misaligned
    assert _solve(lib, _problem(sQ=255)) == binding.TTC_ERR_INVALID_ARG        # stride not a multiple of 4
    assert _solve(lib, _problem(d=48, m=48)) == binding.TTC_ERR_UNSUPPORTED
    assert _solve(lib, _problem(m=8)) == binding.TTC_ERR_UNSUPPORTED
    assert _solve(lib, _problem(), sol=binding.Solution(None, None, None, None, None)) == binding.TTC_ERR_INVALID_ARG
    assert _solve(lib, _problem(), ws=None) == binding.TTC_ERR_WORKSPACE
    assert _solve(lib, _problem(), ws_bytes=16) == binding.TTC_ERR_WORKSPACE
    assert _solve(lib, _problem(n=0)) == binding.TTC_OK                          # empty batch: nothing launched
    assert lib.ttc_lqr_solve(None, None, None, 0, None) == binding.TTC_ERR_INVALID_ARG


def test_workspace_bytes(lib):
    p = _problem(d=128, m=128, T=16)
    w = binding.ttc_lqr_workspace_bytes(p)
    assert w > 0 and w % (128 * 128 * 4) == 0                                   # one matrix per resident workgroup
    assert binding.ttc_lqr_workspace_bytes(p, for_rollout=True) == w * 19       # T + 3 of them for the roll-out
    assert binding.ttc_lqr_workspace_bytes(_problem(d=48, m=48)) == 0
    p.n = 10 ** 9
    assert binding.ttc_lqr_workspace_bytes(p) == w                               # independent of n
    p.flags = binding.TTC_FLAG_DOUBLING                                          # six matrices per workgroup
    assert binding.ttc_lqr_workspace_bytes(p) == w * 6


def test_binding_rejects_mixed_dtypes():
    import torch
    A = torch.zeros(1, 16, 16)
    with pytest.raises(ValueError):
        binding.make_problem(A, A.bfloat16(), A, A, None, torch.zeros(1, 16), 4)
    with pytest.raises(ValueError):
        binding.make_problem(A.double(), A.double(), A.double(), A.double(), None, torch.zeros(1, 16).double(), 4)


def _tv_problem(**kw):
    p = binding.TvProblem()
    p.n, p.d, p.m, p.T = 4, 16, 16, 8
    fake = 0x1000  # never dereferenced: validation fails or n == 0 before any launch
    p.A = p.B = p.Q = p.R = p.x0 = fake
    p.sA = p.sB = p.sQ = p.sR = 8 * 256
    p.tA = p.tB = p.tQ = p.tR = 256
    p.sx0 = 16
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_time_heterogeneous_argument_validation_without_device(lib):
    sol = binding.Solution(0x1000, 0x1000, 0x1000, 0x1000, 0x1000)

    def solve(p, s=sol):
        return lib.ttc_lqr_solve_tv(ctypes.byref(p), ctypes.byref(s), None, 0, None)

    def rollout(p, U=0x1000, ws=0x1000, ws_bytes=1 << 40):
        return lib.ttc_lqr_rollout_tv(ctypes.byref(p), U, None, None, None, ws, ws_bytes, None)

    for call in (solve, rollout):
        assert call(_tv_problem(T=0)) == binding.TTC_ERR_INVALID_ARG
        assert call(_tv_problem(flags=1)) == binding.TTC_ERR_INVALID_ARG           # no flags on this entry point
        assert call(_tv_problem(in_dtype=3)) == binding.TTC_ERR_INVALID_ARG
        assert call(_tv_problem(R=None)) == binding.TTC_ERR_INVALID_ARG
        assert call(_tv_problem(B=0x1008)) == binding.TTC_ERR_INVALID_ARG          # misaligned
        assert call(_tv_problem(tQ=250)) == binding.TTC_ERR_INVALID_ARG            # step stride not a multiple of 4
        assert call(_tv_problem(d=48, m=48)) == binding.TTC_ERR_UNSUPPORTED
        assert call(_tv_problem(n=0)) == binding.TTC_OK
    assert solve(_tv_problem(), binding.Solution(None, None, None, None, None)) == binding.TTC_ERR_INVALID_ARG
    assert rollout(_tv_problem(), U=None) == binding.TTC_ERR_INVALID_ARG
    assert rollout(_tv_problem(), ws=None) == binding.TTC_ERR_WORKSPACE
    assert rollout(_tv_problem(), ws_bytes=64) == binding.TTC_ERR_WORKSPACE
    w = lib.ttc_lqr_tv_rollout_workspace_bytes(ctypes.byref(_tv_problem(d=128, m=128, T=16)))
    assert w > 0 and w % (16 * 128 * 128 * 4) == 0                                   # T matrices per resident workgroup
    assert lib.ttc_lqr_tv_rollout_workspace_bytes(ctypes.byref(_tv_problem(d=48, m=48))) == 0


def _cxt_problem(**kw):
    p = binding.CxtProblem()
    p.n, p.d, p.r, p.T, p.in_dtype, p.flags = 8, 16, 16, 4, binding.TTC_F32, 0
    for k in ("sA", "sB", "sQ", "sQf", "rinv", "lgA", "lgB", "lgQ", "x0", "Bbasis", "Qbasis"):
        setattr(p, k, 0x1000)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_structured_argument_validation_without_device(lib):
    s = binding.Solution(0x2000, 0x3000, 0x4000, 0x5000, 0x6000)
    call = lambda p, sol=s: lib.ttc_lqr_solve_cxt(ctypes.byref(p), ctypes.byref(sol), None)
    assert call(_cxt_problem(T=0)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(r=0)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(flags=4)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(in_dtype=2)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(n=-1)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(lgB=None)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(Qbasis=0x1002)) == binding.TTC_ERR_INVALID_ARG        # misaligned for float32
    assert call(_cxt_problem(Qbasis=0x1002, in_dtype=binding.TTC_BF16, n=0)) == binding.TTC_OK
    assert call(_cxt_problem(d=32)) == binding.TTC_ERR_UNSUPPORTED
    assert call(_cxt_problem(r=65)) == binding.TTC_ERR_UNSUPPORTED
    assert call(_cxt_problem(n=0)) == binding.TTC_OK
    assert call(_cxt_problem(), binding.Solution(None, None, None, None, None)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(), binding.Solution(0x2004, 0x3000, 0x4000, None, None)) == binding.TTC_ERR_INVALID_ARG


def test_structured_binding_checks_shapes():
    b = synth.make_contextual_batch(6, 16, 4, 5, seed=0)
    keys = synth.ContextualBatch.PER_PROBLEM + ("Bbasis", "Qbasis", "x0")
    args = {k: getattr(b, k) for k in keys}
    p = binding.make_cxt_problem(*(args[k] for k in keys), 5)
    assert (p.n, p.d, p.r, p.T, p.in_dtype) == (6, 16, 4, 5, binding.TTC_F32)
    bad = dict(args, sQ=args["sQ"][:, :3].contiguous())
    with pytest.raises(ValueError):
        binding.make_cxt_problem(*(bad[k] for k in keys), 5)
    bad = dict(args, lgA=args["lgA"].to(torch.bfloat16))
    with pytest.raises(ValueError):
        binding.make_cxt_problem(*(bad[k] for k in keys), 5)


def test_pairwise_long_horizon_argument_validation_without_device(lib):
    s = binding.Solution(0x2000, 0x3000, 0x4000, 0x5000, 0x6000)
    call = lambda p, sol=s, ws=0x1000, nbytes=1 << 40: lib.ttc_lqr_solve_tv_scan(ctypes.byref(p), ctypes.byref(sol), ws,
                                                                                nbytes, None)
    need = lib.ttc_lqr_tv_scan_workspace_bytes(ctypes.byref(_tv_problem()))
    assert need == 4 * 8 * 3 * 256 * 4                      # n * T * 3 * d * d floats
    assert lib.ttc_lqr_tv_scan_workspace_bytes(ctypes.byref(_tv_problem(d=48, m=48))) == 0
    assert call(_tv_problem(T=0)) == binding.TTC_ERR_INVALID_ARG
    assert call(_tv_problem(flags=1)) == binding.TTC_ERR_INVALID_ARG
    assert call(_tv_problem(A=None)) == binding.TTC_ERR_INVALID_ARG
    assert call(_tv_problem(d=48, m=48)) == binding.TTC_ERR_UNSUPPORTED
    assert call(_tv_problem(n=0)) == binding.TTC_OK
    assert call(_tv_problem(), ws=None) == binding.TTC_ERR_WORKSPACE
    assert call(_tv_problem(), ws=0x1008) == binding.TTC_ERR_WORKSPACE          # misaligned
    assert call(_tv_problem(), nbytes=need - 1) == binding.TTC_ERR_WORKSPACE
    assert call(_tv_problem(), binding.Solution(None, None, None, None, None)) == binding.TTC_ERR_INVALID_ARG


def test_structured_rollout_argument_validation_without_device(lib):
    call = lambda p, U=0x2000, ws=0x1000, nbytes=1 << 40: lib.ttc_lqr_rollout_cxt(ctypes.byref(p), U, None, None, None, ws,
                                                                                 nbytes, None)
    need = lib.ttc_lqr_cxt_rollout_workspace_bytes(ctypes.byref(_cxt_problem()))
    assert need == 8 * (4 + 3) * 256 * 4 + 32              # gains and combined bases, then 8 flags rounded to 16 bytes
    assert lib.ttc_lqr_cxt_rollout_workspace_bytes(ctypes.byref(_cxt_problem(d=32))) == 0
    assert call(_cxt_problem(T=0)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(d=32)) == binding.TTC_ERR_UNSUPPORTED
    assert call(_cxt_problem(n=0)) == binding.TTC_OK
    assert call(_cxt_problem(), U=None) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(), ws=None) == binding.TTC_ERR_WORKSPACE
    assert call(_cxt_problem(), nbytes=need - 1) == binding.TTC_ERR_WORKSPACE


def test_structured_backward_argument_validation_without_device(lib):
    def grads(**kw):
        g = binding.CxtGrads()
        for k in binding.CXT_GRADS:
            setattr(g, k, 0x8000)
        for k, v in kw.items():
            setattr(g, k, v)
        return g
    call = lambda p, g=None, gu=0x7000, ws=0x1000, nbytes=1 << 40: lib.ttc_lqr_backward_cxt(
        ctypes.byref(p), gu, ctypes.byref(g if g is not None else grads()), ws, nbytes, None)
    need = lib.ttc_lqr_backward_cxt_workspace_bytes(ctypes.byref(_cxt_problem()))
    per_problem = (4 + 4) * 256 + 4 * (4 + 1) * 16 + 768 + 1   # kept matrices, trajectories, rows for the bases, info
    assert need == (8 * per_problem + 63) // 64 * 64 * 4   # floats, rounded up to a multiple of 64
    assert lib.ttc_lqr_backward_cxt_workspace_bytes(ctypes.byref(_cxt_problem(d=32))) == 0
    assert call(_cxt_problem(T=0)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(r=0)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(d=32)) == binding.TTC_ERR_UNSUPPORTED
    assert call(_cxt_problem(sQ=None)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(), gu=None) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(), grads(gBbasis=None)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(), grads(glgB=None)) == binding.TTC_ERR_INVALID_ARG
    assert call(_cxt_problem(), grads(gsA=0x8002)) == binding.TTC_ERR_INVALID_ARG            # misaligned output
    assert call(_cxt_problem(Bbasis=0x1004)) == binding.TTC_ERR_INVALID_ARG                  # the bases' rows are read 16 bytes at a time
    assert call(_cxt_problem(Qbasis=0x1008)) == binding.TTC_ERR_INVALID_ARG


def test_block_argument_validation_without_device(lib):
    def block(**kw):
        b = binding.Block()
        b.n_tokens, b.C, b.H, b.d, b.r, b.T, b.flags, b.eps = 12, 64, 4, 16, 8, 3, 0, 1e-5
        for k in binding.BLOCK_WEIGHTS:
            setattr(b, k, 0x1000)
        for k, v in kw.items():
            setattr(b, k, v)
        return b
    call = lambda b, x=0x2000, y=0x3000, ws=0x4000, nbytes=1 << 40: lib.ttc_block_forward(ctypes.byref(b), x, y, None, None,
                                                                                         None, ws, nbytes, None)
    need = lib.ttc_block_workspace_bytes(ctypes.byref(block()))
    assert need > 0 and need % 16 == 0
    assert lib.ttc_block_workspace_bytes(ctypes.byref(block(d=32))) == 0
    assert call(block(T=0)) == binding.TTC_ERR_INVALID_ARG
    assert call(block(eps=0.0)) == binding.TTC_ERR_INVALID_ARG
    assert call(block(flags=2)) == binding.TTC_ERR_INVALID_ARG
    assert call(block(d=32)) == binding.TTC_ERR_UNSUPPORTED
    assert call(block(r=6)) == binding.TTC_ERR_UNSUPPORTED                               # r is a multiple of four
    assert call(block(C=62)) == binding.TTC_ERR_UNSUPPORTED                              # so is C
    assert call(block(C=68, flags=binding.TTC_BLOCK_FLAG_BF16)) == binding.TTC_ERR_UNSUPPORTED   # of eight for bfloat16
    assert call(block(n_tokens=0)) == binding.TTC_OK
    assert call(block(W_out=None)) == binding.TTC_ERR_INVALID_ARG
    assert call(block(W_head=0x1004)) == binding.TTC_ERR_INVALID_ARG                     # misaligned
    assert call(block(), x=None) == binding.TTC_ERR_INVALID_ARG
    assert call(block(), ws=None) == binding.TTC_ERR_WORKSPACE
    assert call(block(), nbytes=need - 1) == binding.TTC_ERR_WORKSPACE
