"""ctypes binding of the C-ABI library (include/ttc_lqr.h): argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the HIP library.
The library must have been built (``python -c "import __graft_entry__ as g; g.build()"``); there is
no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libttc_lqr.so")

TTC_OK, TTC_ERR_INVALID_ARG, TTC_ERR_UNSUPPORTED, TTC_ERR_WORKSPACE, TTC_ERR_DEVICE = range(5)
TTC_F32, TTC_BF16 = 0, 1
TTC_FLAG_STAGE_COST_AT_X0 = 1
TTC_FLAG_PURE_SYMPLECTIC = 2
TTC_FLAG_DOUBLING = 4

EXPORTS = ("ttc_lqr_workspace_bytes", "ttc_lqr_solve", "ttc_lqr_solve_noalloc", "ttc_lqr_noalloc_scratch_bytes",
           "ttc_lqr_rollout", "ttc_lqr_solve_tv", "ttc_lqr_rollout_tv",
           "ttc_lqr_tv_rollout_workspace_bytes", "ttc_lqr_solve_cxt", "ttc_lqr_rollout_cxt",
           "ttc_lqr_cxt_rollout_workspace_bytes", "ttc_lqr_solve_tv_scan",
           "ttc_lqr_tv_scan_workspace_bytes", "ttc_lqr_tv_scan_values", "ttc_lqr_tv_scan_values_workspace_bytes",
           "ttc_lqr_backward", "ttc_lqr_backward_workspace_bytes",
           "ttc_lqr_backward_tv", "ttc_lqr_backward_tv_workspace_bytes", "ttc_lqr_backward_cxt", "ttc_lqr_backward_cxt_workspace_bytes", "ttc_block_workspace_bytes", "ttc_block_forward",
           "ttc_status_string", "ttc_version")


class Problem(ctypes.Structure):
    _fields_ = [("n", c_int64), ("d", c_int32), ("m", c_int32), ("T", c_int32), ("in_dtype", c_int32),
                ("flags", c_int32), ("rebase_every", c_int32),
                ("A", c_void_p), ("B", c_void_p), ("Q", c_void_p), ("R", c_void_p), ("QT", c_void_p),
                ("x0", c_void_p),
                ("sA", c_int64), ("sB", c_int64), ("sQ", c_int64), ("sR", c_int64), ("sQT", c_int64),
                ("sx0", c_int64)]


class TvProblem(ctypes.Structure):
    _fields_ = [("n", c_int64), ("d", c_int32), ("m", c_int32), ("T", c_int32), ("in_dtype", c_int32),
                ("flags", c_int32),
                ("A", c_void_p), ("B", c_void_p), ("Q", c_void_p), ("R", c_void_p), ("x0", c_void_p),
                ("sA", c_int64), ("sB", c_int64), ("sQ", c_int64), ("sR", c_int64), ("sx0", c_int64),
                ("tA", c_int64), ("tB", c_int64), ("tQ", c_int64), ("tR", c_int64)]


class CxtProblem(ctypes.Structure):
    _fields_ = [("n", c_int64), ("d", c_int32), ("r", c_int32), ("T", c_int32), ("in_dtype", c_int32),
                ("flags", c_int32),
                ("sA", c_void_p), ("sB", c_void_p), ("sQ", c_void_p), ("sQf", c_void_p), ("rinv", c_void_p),
                ("lgA", c_void_p), ("lgB", c_void_p), ("lgQ", c_void_p), ("x0", c_void_p),
                ("Bbasis", c_void_p), ("Qbasis", c_void_p)]


BLOCK_WEIGHTS = ("ln_in_gain", "ln_in_offset", "W_in", "b_in", "W_head", "b_head", "W_shared", "b_shared", "Bbasis", "Qc",
                 "ln_out_gain", "ln_out_offset", "W_out", "b_out")


class Block(ctypes.Structure):
    _fields_ = [("n_tokens", c_int64), ("C", c_int32), ("H", c_int32), ("d", c_int32), ("r", c_int32), ("T", c_int32),
                ("flags", c_int32), ("eps", ctypes.c_float)] + [(k, c_void_p) for k in BLOCK_WEIGHTS]


class Solution(ctypes.Structure):
    _fields_ = [("P0", c_void_p), ("K0", c_void_p), ("u0", c_void_p), ("value", c_void_p), ("info", c_void_p)]


class Grads(ctypes.Structure):
    _fields_ = [("gA", c_void_p), ("gB", c_void_p), ("gQ", c_void_p), ("gR", c_void_p), ("gQT", c_void_p),
                ("gx0", c_void_p), ("info", c_void_p)]


CXT_GRADS = ("gsA", "gsB", "gsQ", "gsQf", "grinv", "glgA", "glgB", "glgQ", "gx0", "gBbasis", "gQbasis", "info")


class CxtGrads(ctypes.Structure):
    _fields_ = [(k, c_void_p) for k in CXT_GRADS]


class TtcError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"ttc_lqr: {text} (status {status})")
        self.status = status


_lib = None


def load():
    """Load the shared library (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with __graft_entry__.build()")
    lib = ctypes.CDLL(LIB_PATH)
    lib.ttc_lqr_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_workspace_bytes.argtypes = [ctypes.POINTER(Problem), c_int]
    lib.ttc_lqr_solve.restype = c_int
    lib.ttc_lqr_solve.argtypes = [ctypes.POINTER(Problem), ctypes.POINTER(Solution), c_void_p, c_size_t, c_void_p]
    lib.ttc_lqr_solve_noalloc.restype = c_int
    lib.ttc_lqr_solve_noalloc.argtypes = [ctypes.POINTER(Problem), ctypes.POINTER(Solution), c_void_p]
    lib.ttc_lqr_noalloc_scratch_bytes.restype = c_size_t
    lib.ttc_lqr_noalloc_scratch_bytes.argtypes = []
    lib.ttc_lqr_rollout.restype = c_int
    lib.ttc_lqr_rollout.argtypes = [ctypes.POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                    c_size_t, c_void_p]
    lib.ttc_lqr_solve_tv.restype = c_int
    lib.ttc_lqr_solve_tv.argtypes = [ctypes.POINTER(TvProblem), ctypes.POINTER(Solution), c_void_p, c_size_t, c_void_p]
    lib.ttc_lqr_tv_rollout_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_tv_rollout_workspace_bytes.argtypes = [ctypes.POINTER(TvProblem)]
    lib.ttc_lqr_rollout_tv.restype = c_int
    lib.ttc_lqr_rollout_tv.argtypes = [ctypes.POINTER(TvProblem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                       c_size_t, c_void_p]
    lib.ttc_lqr_tv_scan_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_tv_scan_workspace_bytes.argtypes = [ctypes.POINTER(TvProblem)]
    lib.ttc_lqr_solve_tv_scan.restype = c_int
    lib.ttc_lqr_solve_tv_scan.argtypes = [ctypes.POINTER(TvProblem), ctypes.POINTER(Solution), c_void_p, c_size_t,
                                          c_void_p]
    lib.ttc_lqr_tv_scan_values_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_tv_scan_values_workspace_bytes.argtypes = [ctypes.POINTER(TvProblem)]
    lib.ttc_lqr_tv_scan_values.restype = c_int
    lib.ttc_lqr_tv_scan_values.argtypes = [ctypes.POINTER(TvProblem), c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.ttc_lqr_solve_cxt.restype = c_int
    lib.ttc_lqr_solve_cxt.argtypes = [ctypes.POINTER(CxtProblem), ctypes.POINTER(Solution), c_void_p]
    lib.ttc_lqr_cxt_rollout_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_cxt_rollout_workspace_bytes.argtypes = [ctypes.POINTER(CxtProblem)]
    lib.ttc_lqr_rollout_cxt.restype = c_int
    lib.ttc_lqr_rollout_cxt.argtypes = [ctypes.POINTER(CxtProblem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                        c_size_t, c_void_p]
    lib.ttc_lqr_backward_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_backward_workspace_bytes.argtypes = [ctypes.POINTER(Problem)]
    lib.ttc_lqr_backward.restype = c_int
    lib.ttc_lqr_backward.argtypes = [ctypes.POINTER(Problem), c_void_p, ctypes.POINTER(Grads), c_void_p, c_size_t,
                                     c_void_p]
    lib.ttc_lqr_backward_tv_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_backward_tv_workspace_bytes.argtypes = [ctypes.POINTER(TvProblem)]
    lib.ttc_lqr_backward_tv.restype = c_int
    lib.ttc_lqr_backward_tv.argtypes = [ctypes.POINTER(TvProblem), c_void_p, ctypes.POINTER(Grads), c_void_p, c_size_t,
                                        c_void_p]
    lib.ttc_lqr_backward_cxt_workspace_bytes.restype = c_size_t
    lib.ttc_lqr_backward_cxt_workspace_bytes.argtypes = [ctypes.POINTER(CxtProblem)]
    lib.ttc_lqr_backward_cxt.restype = c_int
    lib.ttc_lqr_backward_cxt.argtypes = [ctypes.POINTER(CxtProblem), c_void_p, ctypes.POINTER(CxtGrads), c_void_p, c_size_t,
                                         c_void_p]
    lib.ttc_block_workspace_bytes.restype = c_size_t
    lib.ttc_block_workspace_bytes.argtypes = [ctypes.POINTER(Block)]
    lib.ttc_block_forward.restype = c_int
    lib.ttc_block_forward.argtypes = [ctypes.POINTER(Block), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                      c_size_t, c_void_p]
    lib.ttc_status_string.restype = c_char_p
    lib.ttc_status_string.argtypes = [c_int]
    lib.ttc_version.restype = c_int
    lib.ttc_version.argtypes = []
    _lib = lib
    return lib


def ttc_version() -> int:
    return load().ttc_version()


def ttc_status_string(status: int) -> str:
    return load().ttc_status_string(status).decode()


def _check(status):
    if status != TTC_OK:
        raise TtcError(status, ttc_status_string(status))


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stride(t):
    """Elements between consecutive problems of a (n, ...) tensor whose trailing dims are contiguous."""
    if t is None:
        return 0
    inner = 1
    for k in range(t.dim() - 1, 0, -1):
        if t.shape[k] != 1 and t.stride(k) != inner:
            raise ValueError("per-problem matrices must be contiguous row-major")
        inner *= t.shape[k]
    return t.stride(0)


def make_problem(A, B, Q, R, QT, x0, T, flags=0, rebase_every=0, n=None) -> Problem:
    """Fill the problem descriptor from tensors A (n,d,d), B (n,d,m), Q (n,d,d), R (n,m,m), QT or None,
    x0 (n,d).  A leading dimension expanded with stride 0 is passed through as a shared matrix."""
    dt = A.dtype
    for t in (B, Q, R, x0) + (() if QT is None else (QT,)):
        if t.dtype != dt:
            raise ValueError("all inputs must share one dtype")
    in_dtype = {torch.float32: TTC_F32, torch.bfloat16: TTC_BF16}.get(dt)
    if in_dtype is None:
        raise ValueError("inputs must be float32 or bfloat16")
    p = Problem()
    p.n = A.shape[0] if n is None else n
    p.d, p.m, p.T = A.shape[1], B.shape[2], T
    p.in_dtype, p.flags, p.rebase_every = in_dtype, flags, rebase_every
    p.A, p.B, p.Q, p.R, p.QT, p.x0 = _ptr(A), _ptr(B), _ptr(Q), _ptr(R), _ptr(QT), _ptr(x0)
    p.sA, p.sB, p.sQ, p.sR, p.sQT, p.sx0 = (_stride(t) for t in (A, B, Q, R, QT, x0))
    return p


def ttc_lqr_workspace_bytes(problem: Problem, for_rollout: bool = False) -> int:
    return load().ttc_lqr_workspace_bytes(ctypes.byref(problem), 1 if for_rollout else 0)


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _scratch(nbytes, dev, stream):
    """A workspace the wrapper owns: allocated for, and only released to, the stream the kernels run on (the
    caching allocator would otherwise hand the block to other work on the current stream while the launch,
    on another stream, still uses it)."""
    if stream is None or stream == torch.cuda.current_stream():
        return torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=dev)
    with torch.cuda.stream(stream):
        return torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=dev)


def ttc_lqr_solve(A, B, Q, R, QT, x0, T, *, flags=0, rebase_every=0, want_P0=True, want_K0=True,
                  out=None, workspace=None, stream=None):
    """P0 (n,d,d), K0 (n,m,d), u0 (n,m), value (n), info (n) of n LQR problems; all float32 device tensors.

    `out` may carry preallocated tensors under the same names; `workspace` a uint8 device tensor."""
    lib = load()
    prob = make_problem(A, B, Q, R, QT, x0, T, flags, rebase_every)
    n, d, m, dev = prob.n, prob.d, prob.m, A.device
    out = dict(out or {})
    f32 = dict(dtype=torch.float32, device=dev)
    if want_P0 and "P0" not in out:
        out["P0"] = torch.empty((n, d, d), **f32)
    if want_K0 and "K0" not in out:
        out["K0"] = torch.empty((n, m, d), **f32)
    out.setdefault("u0", torch.empty((n, m), **f32))
    out.setdefault("value", torch.empty((n,), **f32))
    out.setdefault("info", torch.empty((n,), dtype=torch.int32, device=dev))
    sol = Solution(_ptr(out.get("P0")), _ptr(out.get("K0")), _ptr(out["u0"]), _ptr(out["value"]), _ptr(out["info"]))
    need = lib.ttc_lqr_workspace_bytes(ctypes.byref(prob), 0)
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    _check(lib.ttc_lqr_solve(ctypes.byref(prob), ctypes.byref(sol), c_void_p(workspace.data_ptr()),
                             workspace.numel(), _stream_ptr(stream)))
    return out


def ttc_lqr_solve_noalloc(A, B, Q, R, QT, x0, T, out, *, flags=0, rebase_every=0, stream=None):
    """ttc_lqr_solve through the entry point that allocates nothing: `out` must carry preallocated u0 (n,m) and,
    optionally, P0, K0, value, info; the library's own fixed scratch array serves as the workspace."""
    lib = load()
    prob = make_problem(A, B, Q, R, QT, x0, T, flags, rebase_every)
    sol = Solution(_ptr(out.get("P0")), _ptr(out.get("K0")), _ptr(out["u0"]), _ptr(out.get("value")),
                   _ptr(out.get("info")))
    _check(lib.ttc_lqr_solve_noalloc(ctypes.byref(prob), ctypes.byref(sol), _stream_ptr(stream)))
    return out


def ttc_lqr_rollout(A, B, Q, R, QT, x0, T, *, flags=0, rebase_every=0, workspace=None, stream=None):
    """U (n,T,m), X (n,T+1,d), cost (n), info (n) of n LQR problems; float32 device tensors."""
    lib = load()
    prob = make_problem(A, B, Q, R, QT, x0, T, flags, rebase_every)
    n, d, m, dev = prob.n, prob.d, prob.m, A.device
    f32 = dict(dtype=torch.float32, device=dev)
    U = torch.empty((n, T, m), **f32)
    X = torch.empty((n, T + 1, d), **f32)
    cost = torch.empty((n,), **f32)
    info = torch.empty((n,), dtype=torch.int32, device=dev)
    need = lib.ttc_lqr_workspace_bytes(ctypes.byref(prob), 1)
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    _check(lib.ttc_lqr_rollout(ctypes.byref(prob), c_void_p(U.data_ptr()), c_void_p(X.data_ptr()),
                               c_void_p(cost.data_ptr()), c_void_p(info.data_ptr()),
                               c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream)))
    return {"U": U, "X": X, "cost": cost, "info": info}


def _tv_strides(t):
    """(problem stride, step stride) in elements of a (n, T, r, c) tensor whose matrices are contiguous row-major."""
    if t.dim() != 4 or (t.shape[3] != 1 and t.stride(3) != 1) or (t.shape[2] != 1 and t.stride(2) != t.shape[3]):
        raise ValueError("expected (n, T, rows, cols) with contiguous row-major matrices")
    return t.stride(0), t.stride(1)


def make_tv_problem(A, B, Q, R, x0) -> TvProblem:
    """Descriptor of a time-heterogeneous problem from A (n,T,d,d), B (n,T,d,m), Q (n,T,d,d), R (n,T,m,m), x0 (n,d);
    an axis expanded with stride 0 is passed through as shared."""
    dt = A.dtype
    for t in (B, Q, R, x0):
        if t.dtype != dt:
            raise ValueError("all inputs must share one dtype")
    in_dtype = {torch.float32: TTC_F32, torch.bfloat16: TTC_BF16}.get(dt)
    if in_dtype is None:
        raise ValueError("inputs must be float32 or bfloat16")
    p = TvProblem()
    p.n, p.T, p.d, p.m = A.shape[0], A.shape[1], A.shape[2], B.shape[3]
    p.in_dtype, p.flags = in_dtype, 0
    p.A, p.B, p.Q, p.R, p.x0 = _ptr(A), _ptr(B), _ptr(Q), _ptr(R), _ptr(x0)
    (p.sA, p.tA), (p.sB, p.tB), (p.sQ, p.tQ), (p.sR, p.tR) = (_tv_strides(t) for t in (A, B, Q, R))
    p.sx0 = _stride(x0)
    return p


def ttc_lqr_solve_tv(A, B, Q, R, x0, *, want_P0=True, want_K0=True, out=None, stream=None):
    """P0, K0, u0, value, info of n time-heterogeneous problems: A (n,T,d,d), B (n,T,d,m), R (n,T,m,m) and
    Q (n,T,d,d) with Q[:, s] the cost on the state step s arrives at (Q[:, T-1] is the terminal cost)."""
    lib = load()
    prob = make_tv_problem(A, B, Q, R, x0)
    n, d, m, dev = prob.n, prob.d, prob.m, A.device
    out = dict(out or {})
    f32 = dict(dtype=torch.float32, device=dev)
    if want_P0 and "P0" not in out:
        out["P0"] = torch.empty((n, d, d), **f32)
    if want_K0 and "K0" not in out:
        out["K0"] = torch.empty((n, m, d), **f32)
    out.setdefault("u0", torch.empty((n, m), **f32))
    out.setdefault("value", torch.empty((n,), **f32))
    out.setdefault("info", torch.empty((n,), dtype=torch.int32, device=dev))
    sol = Solution(_ptr(out.get("P0")), _ptr(out.get("K0")), _ptr(out["u0"]), _ptr(out["value"]), _ptr(out["info"]))
    _check(lib.ttc_lqr_solve_tv(ctypes.byref(prob), ctypes.byref(sol), None, 0, _stream_ptr(stream)))
    return out


def ttc_lqr_tv_scan_values(A, B, Q, R, x0, *, want_P=True, want_K=True, workspace=None, stream=None):
    """P (n, T, d, d) with P[:, k] = P_{k+1} and K (n, T, m, d) with K[:, s] = K_s of n time-heterogeneous problems,
    by the tree over the horizon (up-sweep and down-sweep)."""
    lib = load()
    prob = make_tv_problem(A, B, Q, R, x0)
    n, d, m, T, dev = prob.n, prob.d, prob.m, prob.T, A.device
    f32 = dict(dtype=torch.float32, device=dev)
    out = {}
    if want_P:
        out["P"] = torch.empty((n, T, d, d), **f32)
    if want_K:
        out["K"] = torch.empty((n, T, m, d), **f32)
    need = lib.ttc_lqr_tv_scan_values_workspace_bytes(ctypes.byref(prob))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    _check(lib.ttc_lqr_tv_scan_values(ctypes.byref(prob), _ptr(out.get("P")), _ptr(out.get("K")),
                                      c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream)))
    return out


def ttc_lqr_solve_tv_scan(A, B, Q, R, x0, *, want_P0=True, want_K0=True, out=None, workspace=None, stream=None):
    """ttc_lqr_solve_tv with the factors composed pairwise over the horizon (small batches, long horizons)."""
    lib = load()
    prob = make_tv_problem(A, B, Q, R, x0)
    n, d, m, dev = prob.n, prob.d, prob.m, A.device
    out = dict(out or {})
    f32 = dict(dtype=torch.float32, device=dev)
    if want_P0 and "P0" not in out:
        out["P0"] = torch.empty((n, d, d), **f32)
    if want_K0 and "K0" not in out:
        out["K0"] = torch.empty((n, m, d), **f32)
    out.setdefault("u0", torch.empty((n, m), **f32))
    out.setdefault("value", torch.empty((n,), **f32))
    out.setdefault("info", torch.empty((n,), dtype=torch.int32, device=dev))
    need = lib.ttc_lqr_tv_scan_workspace_bytes(ctypes.byref(prob))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    sol = Solution(_ptr(out.get("P0")), _ptr(out.get("K0")), _ptr(out["u0"]), _ptr(out["value"]), _ptr(out["info"]))
    _check(lib.ttc_lqr_solve_tv_scan(ctypes.byref(prob), ctypes.byref(sol), c_void_p(workspace.data_ptr()),
                                     workspace.numel(), _stream_ptr(stream)))
    return out


def ttc_lqr_rollout_tv(A, B, Q, R, x0, *, workspace=None, stream=None):
    """U (n,T,m), X (n,T+1,d), cost (n), info (n) of n time-heterogeneous problems; float32 device tensors."""
    lib = load()
    prob = make_tv_problem(A, B, Q, R, x0)
    n, d, m, T, dev = prob.n, prob.d, prob.m, prob.T, A.device
    f32 = dict(dtype=torch.float32, device=dev)
    out = {"U": torch.empty((n, T, m), **f32), "X": torch.empty((n, T + 1, d), **f32),
           "cost": torch.empty((n,), **f32), "info": torch.empty((n,), dtype=torch.int32, device=dev)}
    need = lib.ttc_lqr_tv_rollout_workspace_bytes(ctypes.byref(prob))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    _check(lib.ttc_lqr_rollout_tv(ctypes.byref(prob), _ptr(out["U"]), _ptr(out["X"]), _ptr(out["cost"]),
                                  _ptr(out["info"]), c_void_p(workspace.data_ptr()), workspace.numel(),
                                  _stream_ptr(stream)))
    return out


def make_cxt_problem(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T) -> CxtProblem:
    """Descriptor of n structured problems: sA, rinv, lgA, lgB, lgQ, x0 (n,d); sB, sQ, sQf (n,r); Bbasis, Qbasis
    (r,d,d); all contiguous and of one dtype."""
    n, d = sA.shape
    r = Bbasis.shape[0]
    shapes = {"sA": (n, d), "rinv": (n, d), "lgA": (n, d), "lgB": (n, d), "lgQ": (n, d), "x0": (n, d),
              "sB": (n, r), "sQ": (n, r), "sQf": (n, r), "Bbasis": (r, d, d), "Qbasis": (r, d, d)}
    given = dict(sA=sA, sB=sB, sQ=sQ, sQf=sQf, rinv=rinv, lgA=lgA, lgB=lgB, lgQ=lgQ, Bbasis=Bbasis, Qbasis=Qbasis, x0=x0)
    for k, t in given.items():
        if tuple(t.shape) != shapes[k] or not t.is_contiguous() or t.dtype != sA.dtype:
            raise ValueError(f"{k}: expected a contiguous {shapes[k]} tensor of dtype {sA.dtype}")
    in_dtype = {torch.float32: TTC_F32, torch.bfloat16: TTC_BF16}.get(sA.dtype)
    if in_dtype is None:
        raise ValueError("inputs must be float32 or bfloat16")
    p = CxtProblem()
    p.n, p.d, p.r, p.T, p.in_dtype, p.flags = n, d, r, T, in_dtype, 0
    for k, t in given.items():
        setattr(p, k, _ptr(t))
    return p


def ttc_lqr_solve_cxt(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T, *, want_P0=True, want_K0=True,
                      out=None, stream=None):
    """P0, K0, u0, value, info of n structured, contextualised problems (float32 device tensors)."""
    lib = load()
    prob = make_cxt_problem(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T)
    n, d, dev = prob.n, prob.d, sA.device
    out = dict(out or {})
    f32 = dict(dtype=torch.float32, device=dev)
    if want_P0 and "P0" not in out:
        out["P0"] = torch.empty((n, d, d), **f32)
    if want_K0 and "K0" not in out:
        out["K0"] = torch.empty((n, d, d), **f32)
    out.setdefault("u0", torch.empty((n, d), **f32))
    out.setdefault("value", torch.empty((n,), **f32))
    out.setdefault("info", torch.empty((n,), dtype=torch.int32, device=dev))
    sol = Solution(_ptr(out.get("P0")), _ptr(out.get("K0")), _ptr(out["u0"]), _ptr(out["value"]), _ptr(out["info"]))
    _check(lib.ttc_lqr_solve_cxt(ctypes.byref(prob), ctypes.byref(sol), _stream_ptr(stream)))
    return out


def ttc_lqr_rollout_cxt(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T, *, workspace=None, stream=None):
    """U (n,T,d), X (n,T+1,d), cost (n), info (n) of n structured problems under the optimal feedback."""
    lib = load()
    prob = make_cxt_problem(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T)
    n, d, dev = prob.n, prob.d, sA.device
    f32 = dict(dtype=torch.float32, device=dev)
    out = {"U": torch.empty((n, T, d), **f32), "X": torch.empty((n, T + 1, d), **f32),
           "cost": torch.empty((n,), **f32), "info": torch.empty((n,), dtype=torch.int32, device=dev)}
    need = lib.ttc_lqr_cxt_rollout_workspace_bytes(ctypes.byref(prob))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    _check(lib.ttc_lqr_rollout_cxt(ctypes.byref(prob), _ptr(out["U"]), _ptr(out["X"]), _ptr(out["cost"]),
                                   _ptr(out["info"]), c_void_p(workspace.data_ptr()), workspace.numel(),
                                   _stream_ptr(stream)))
    return out


def _grads_struct(out):
    return Grads(_ptr(out["gA"]), _ptr(out["gB"]), _ptr(out["gQ"]), _ptr(out["gR"]), _ptr(out.get("gQT")),
                 _ptr(out["gx0"]), _ptr(out.get("info")))


def ttc_lqr_backward(A, B, Q, R, QT, x0, T, grad_u0, *, out=None, workspace=None, stream=None):
    """Gradients of a loss of u0 for n time-invariant problems, from grad_u0 = dl/du0 (n,m) float32: gA, gB, gQ, gR
    (n,d,d), summed over the steps, gQT (n,d,d) when QT is given, gx0 (n,d), info (n)."""
    lib = load()
    prob = make_problem(A, B, Q, R, QT, x0, T)
    n, d, dev = prob.n, prob.d, A.device
    f32 = dict(dtype=torch.float32, device=dev)
    out = dict(out or {})
    for k in ("gA", "gB", "gQ", "gR") + (("gQT",) if QT is not None else ()):
        out.setdefault(k, torch.empty((n, d, d), **f32))
    out.setdefault("gx0", torch.empty((n, d), **f32))
    out.setdefault("info", torch.empty((n,), dtype=torch.int32, device=dev))
    need = lib.ttc_lqr_backward_workspace_bytes(ctypes.byref(prob))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    gr = _grads_struct(out)
    _check(lib.ttc_lqr_backward(ctypes.byref(prob), c_void_p(grad_u0.data_ptr()), ctypes.byref(gr),
                                c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream)))
    return out


def ttc_lqr_backward_tv(A, B, Q, R, x0, grad_u0, *, out=None, workspace=None, stream=None):
    """Gradients of a loss of u0 for n time-heterogeneous problems: gA, gB, gQ, gR (n,T,d,d), gx0 (n,d), info (n)."""
    lib = load()
    prob = make_tv_problem(A, B, Q, R, x0)
    n, d, T, dev = prob.n, prob.d, prob.T, A.device
    f32 = dict(dtype=torch.float32, device=dev)
    out = dict(out or {})
    for k in ("gA", "gB", "gQ", "gR"):
        out.setdefault(k, torch.empty((n, T, d, d), **f32))
    out.setdefault("gx0", torch.empty((n, d), **f32))
    out.setdefault("info", torch.empty((n,), dtype=torch.int32, device=dev))
    need = lib.ttc_lqr_backward_tv_workspace_bytes(ctypes.byref(prob))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    gr = _grads_struct(out)
    _check(lib.ttc_lqr_backward_tv(ctypes.byref(prob), c_void_p(grad_u0.data_ptr()), ctypes.byref(gr),
                                   c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream)))
    return out


def ttc_lqr_backward_cxt(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T, grad_u0, *, out=None, workspace=None,
                         stream=None):
    """Gradients of a loss of u0 for n structured problems, from grad_u0 = dl/du0 (n, d) float32: gsA, grinv, glgA,
    glgB, glgQ, gx0 (n, d), gsB, gsQ, gsQf (n, r), gBbasis, gQbasis (r, d, d) summed over the problems, info (n)."""
    lib = load()
    prob = make_cxt_problem(sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, Bbasis, Qbasis, x0, T)
    n, d, r, dev = prob.n, prob.d, prob.r, sA.device
    if grad_u0.dtype != torch.float32 or not grad_u0.is_contiguous() or tuple(grad_u0.shape) != (n, d):
        raise ValueError("grad_u0 must be a contiguous (n, d) float32 tensor")
    f32 = dict(dtype=torch.float32, device=dev)
    out = dict(out or {})
    for k in ("gsA", "grinv", "glgA", "glgB", "glgQ", "gx0"):
        out.setdefault(k, torch.empty((n, d), **f32))
    for k in ("gsB", "gsQ", "gsQf"):
        out.setdefault(k, torch.empty((n, r), **f32))
    for k in ("gBbasis", "gQbasis"):
        out.setdefault(k, torch.empty((r, d, d), **f32))
    out.setdefault("info", torch.empty((n,), dtype=torch.int32, device=dev))
    need = lib.ttc_lqr_backward_cxt_workspace_bytes(ctypes.byref(prob))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    grads = CxtGrads(*(_ptr(out[k]) for k in CXT_GRADS))
    _check(lib.ttc_lqr_backward_cxt(ctypes.byref(prob), _ptr(grad_u0), ctypes.byref(grads), c_void_p(workspace.data_ptr()),
                                    workspace.numel(), _stream_ptr(stream)))
    return out


TTC_BLOCK_FLAG_BF16 = 1


def make_block(weights, n_tokens, T, eps=1e-5) -> Block:
    """Descriptor of a TTC block from a dict of device tensors (keys BLOCK_WEIGHTS), float32 except that W_in and W_out
    may both be bfloat16 (then the block takes bfloat16 token features: TTC_BLOCK_FLAG_BF16); shapes are checked here,
    values never touched."""
    w = weights
    bf16 = w["W_in"].dtype == torch.bfloat16
    for k in BLOCK_WEIGHTS:
        want_dtype = torch.bfloat16 if bf16 and k in ("W_in", "W_out") else torch.float32
        if w[k].dtype != want_dtype or not w[k].is_contiguous():
            raise ValueError("block weight %s must be a contiguous %s tensor" % (k, want_dtype))
    r, d = int(w["Bbasis"].shape[0]), int(w["Bbasis"].shape[-1])
    HD, C = (int(v) for v in w["W_in"].shape)
    H = HD // d
    want = {"ln_in_gain": (C,), "ln_in_offset": (C,), "W_in": (H * d, C), "b_in": (H * d,),
            "W_head": (H, 5 * d + r, d), "b_head": (H, 5 * d + r), "W_shared": (2 * r, d), "b_shared": (2 * r,),
            "Bbasis": (r, d, d), "Qc": (r, d, d), "ln_out_gain": (H * d,), "ln_out_offset": (H * d,),
            "W_out": (C, H * d), "b_out": (C,)}
    for k, shape in want.items():
        if tuple(w[k].shape) != shape:
            raise ValueError("block weight %s has shape %s, expected %s" % (k, tuple(w[k].shape), shape))
    return Block(n_tokens, C, H, d, r, T, TTC_BLOCK_FLAG_BF16 if bf16 else 0, eps, *(w[k].data_ptr() for k in BLOCK_WEIGHTS))


def ttc_block_forward(x_in, weights, T, *, eps=1e-5, want_h0=False, want_o=False, out=None, workspace=None, stream=None):
    """x_out (n_tokens, C) of the whole TTC block for token features x_in (n_tokens, C) on the device, float32 or
    (with bfloat16 W_in, W_out) bfloat16; info (n_tokens, H); optionally the intermediate h0 and o (n_tokens, H*d), float32."""
    lib = load()
    n, dev = int(x_in.shape[0]), x_in.device
    blk = make_block(weights, n, T, eps)
    xdt = torch.bfloat16 if blk.flags & TTC_BLOCK_FLAG_BF16 else torch.float32
    if x_in.dtype != xdt or not x_in.is_contiguous() or x_in.dim() != 2:
        raise ValueError("x_in must be a contiguous (n_tokens, C) %s tensor" % xdt)
    if int(x_in.shape[1]) != blk.C:
        raise ValueError("x_in has %d features, the block expects %d" % (x_in.shape[1], blk.C))
    out = dict(out or {})
    f32 = dict(dtype=torch.float32, device=dev)
    out.setdefault("x_out", torch.empty((n, blk.C), dtype=xdt, device=dev))
    if want_h0:
        out.setdefault("h0", torch.empty((n, blk.H * blk.d), **f32))
    if want_o:
        out.setdefault("o", torch.empty((n, blk.H * blk.d), **f32))
    out.setdefault("info", torch.empty((n, blk.H), dtype=torch.int32, device=dev))
    need = lib.ttc_block_workspace_bytes(ctypes.byref(blk))
    if workspace is None:
        workspace = _scratch(need, dev, stream)
    _check(lib.ttc_block_forward(ctypes.byref(blk), _ptr(x_in), _ptr(out["x_out"]), _ptr(out.get("h0")), _ptr(out.get("o")),
                                 _ptr(out["info"]), c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream)))
    return out
