"""Seeded synthetic TTC-shaped LQR batches.

One LQR problem per (batch, head, token); the recipe stands in for the per-token parameters
a trained TTC-Net would synthesise (no weights or datasets are available).  This module only
draws inputs: it contains none of the solver's arithmetic and is the one piece of code that
both the HIP path's tests/benchmark and the CPU oracle's tests may import.

Per problem, independent draws in the order A, B, L, M, x0 (d = state size, m = control size):
    A  = I + 0.1 * N(0,1)^{d x d} / sqrt(d)         (optionally rescaled to spectral radius rho)
    B  = N(0,1)^{d x m} / sqrt(d)
    Q  = L L^T / d + 1e-2 I,  L ~ N(0,1)^{d x d}    (symmetrised)
    R  = I + M M^T / m,       M ~ N(0,1)^{m x m}    (symmetrised)
    QT = Q (aliased, returned as None),  x0 ~ N(0,1)^d
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

#: The five workload configurations (problems = batch * heads * tokens).
CONFIGS = {
    "tiny": dict(batch=1, heads=1, tokens=256, d=16, m=16, T=8, dtype="f32", rho=None),
    "small_head": dict(batch=4, heads=16, tokens=1024, d=64, m=64, T=8, dtype="f32", rho=None),
    "llm_adapter": dict(batch=2, heads=32, tokens=8192, d=128, m=128, T=16, dtype="f32", rho=None),
    "long_horizon": dict(batch=1, heads=16, tokens=4096, d=64, m=64, T=64, dtype="f32", rho=0.98),
    "mixed_precision": dict(batch=4, heads=32, tokens=8192, d=128, m=128, T=32, dtype="bf16", rho=None),
}


def config_problems(name: str) -> int:
    c = CONFIGS[name]
    return c["batch"] * c["heads"] * c["tokens"]


@dataclass
class LqrBatch:
    """n problems, row-major, problem-major: A (n,d,d), B (n,d,m), Q (n,d,d), R (n,m,m), x0 (n,d)."""
    A: torch.Tensor
    B: torch.Tensor
    Q: torch.Tensor
    R: torch.Tensor
    x0: torch.Tensor
    T: int

    @property
    def n(self):
        return self.A.shape[0]

    @property
    def d(self):
        return self.A.shape[1]

    @property
    def m(self):
        return self.B.shape[2]

    def take(self, index) -> "LqrBatch":
        """Sub-batch (index: slice or LongTensor) on the same device."""
        return LqrBatch(self.A[index], self.B[index], self.Q[index], self.R[index], self.x0[index], self.T)

    def numpy64(self):
        """Stored values widened to float64 numpy arrays on the host: (A, B, Q, R, x0)."""
        return tuple(t.detach().to("cpu", torch.float64).numpy() for t in (self.A, self.B, self.Q, self.R, self.x0))


def _scale_spectral_radius(A: torch.Tensor, rho: float) -> torch.Tensor:
    ev = torch.linalg.eigvals(A.to("cpu", torch.float64))
    r = ev.abs().amax(dim=-1)
    return A * (rho / r).to(A.device, A.dtype)[:, None, None]


def make_batch(n: int, d: int, m: int, T: int, seed: int = 0, device="cpu", dtype: str = "f32",
               rho: float | None = None, chunk: int = 4096, q_scale: float = 1.0, r_scale: float = 1.0) -> LqrBatch:
    """Draw n problems.  Values are generated in float32 (in chunks, to bound temporaries) and,
    for dtype == "bf16", rounded to bfloat16 storage at the end.  q_scale and r_scale multiply the drawn Q and
    R (costly or cheap states and controls: the ratio decides how hard the closed loop pushes)."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    store = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
    A = torch.empty((n, d, d), dtype=store, device=dev)
    B = torch.empty((n, d, m), dtype=store, device=dev)
    Q = torch.empty((n, d, d), dtype=store, device=dev)
    R = torch.empty((n, m, m), dtype=store, device=dev)
    x0 = torch.empty((n, d), dtype=store, device=dev)
    eye_d = torch.eye(d, device=dev)
    eye_m = torch.eye(m, device=dev)
    for lo in range(0, n, chunk):
        c = min(chunk, n - lo)
        rn = lambda *s: torch.randn(*s, generator=gen, device=dev, dtype=torch.float32)
        a = eye_d + 0.1 * rn(c, d, d) / d ** 0.5
        b = rn(c, d, m) / d ** 0.5
        L = rn(c, d, d)
        M = rn(c, m, m)
        x = rn(c, d)
        if rho is not None:
            a = _scale_spectral_radius(a, rho)
        q = L @ L.transpose(1, 2) / d + 1e-2 * eye_d
        r = eye_m + M @ M.transpose(1, 2) / m
        A[lo:lo + c] = a
        B[lo:lo + c] = b
        Q[lo:lo + c] = q_scale * 0.5 * (q + q.transpose(1, 2))
        R[lo:lo + c] = r_scale * 0.5 * (r + r.transpose(1, 2))
        x0[lo:lo + c] = x
    return LqrBatch(A, B, Q, R, x0, T)


def make_config(name: str, n: int | None = None, seed: int = 0, device="cpu") -> LqrBatch:
    """The named configuration (optionally only its first n problems' worth of draws)."""
    c = CONFIGS[name]
    total = config_problems(name)
    return make_batch(total if n is None else n, c["d"], c["m"], c["T"], seed=seed, device=device,
                      dtype=c["dtype"], rho=c["rho"])


@dataclass
class LqrTvBatch:
    """Time-heterogeneous problems: A (n,T,d,d), B (n,T,d,m), Q (n,T,d,d), R (n,T,m,m), x0 (n,d).  Q[:, s] is the
    cost on the state that step s arrives at; Q[:, T-1] is the terminal cost."""
    A: torch.Tensor
    B: torch.Tensor
    Q: torch.Tensor
    R: torch.Tensor
    x0: torch.Tensor

    @property
    def T(self):
        return self.A.shape[1]

    def take(self, idx):
        return LqrTvBatch(self.A[idx], self.B[idx], self.Q[idx], self.R[idx], self.x0[idx])

    def numpy64(self):
        f = lambda t: t.detach().to("cpu").to(torch.float64).numpy()
        return f(self.A), f(self.B), f(self.Q), f(self.R), f(self.x0)


def make_tv_batch(n: int, d: int, m: int, T: int, seed: int = 0, device="cpu", dtype: str = "f32") -> LqrTvBatch:
    """n problems whose T steps each carry their own (A, B, Q, R): the recipe of make_batch, drawn
    independently for every (problem, step); x0 from the first n draws."""
    b = make_batch(n * T, d, m, T, seed=seed, device=device, dtype=dtype)
    return LqrTvBatch(b.A.view(n, T, d, d), b.B.view(n, T, d, m), b.Q.view(n, T, d, d), b.R.view(n, T, m, m),
                      b.x0[:n].contiguous())


@dataclass
class ContextualBatch:
    """n problems in the structured, contextualised parameterisation (Sec. 4): per-problem vectors
    sA, rinv, lgA, lgB, lgQ (n,d), coefficients sB, sQ, sQf (n,r), x0 (n,d) and the two groups of basis
    matrices Bbasis, Qbasis (r,d,d) shared by all problems."""
    sA: torch.Tensor
    sB: torch.Tensor
    sQ: torch.Tensor
    sQf: torch.Tensor
    rinv: torch.Tensor
    lgA: torch.Tensor
    lgB: torch.Tensor
    lgQ: torch.Tensor
    Bbasis: torch.Tensor
    Qbasis: torch.Tensor
    x0: torch.Tensor
    T: int

    PER_PROBLEM = ("sA", "sB", "sQ", "sQf", "rinv", "lgA", "lgB", "lgQ")

    @property
    def n(self):
        return self.sA.shape[0]

    @property
    def d(self):
        return self.sA.shape[1]

    @property
    def r(self):
        return self.sB.shape[1]

    def take(self, index) -> "ContextualBatch":
        kw = {k: getattr(self, k)[index] for k in self.PER_PROBLEM}
        return ContextualBatch(Bbasis=self.Bbasis, Qbasis=self.Qbasis, x0=self.x0[index], T=self.T, **kw)

    def numpy64(self):
        """Stored values widened to float64 numpy arrays, in the oracle's argument order (x0 last)."""
        f = lambda t: t.detach().to("cpu", torch.float64).numpy()
        return tuple(f(getattr(self, k)) for k in self.PER_PROBLEM) + (f(self.Bbasis), f(self.Qbasis), f(self.x0))


def make_contextual_batch(n: int, d: int, r: int, T: int, seed: int = 0, device="cpu",
                          dtype: str = "f32") -> ContextualBatch:
    """Draws standing in for the outputs of the layer's linear maps s_X(h_0) (no trained weights exist):
        sA = 0.1 N(0,1)^d;  sB = N(0,1)^r / sqrt(r);  sQ, sQf = softplus(N(0,1)^r) / r;
        rinv = softplus(N(0,1)^d);  lgA, lgB, lgQ = 0.25 softplus(N(0,1)^d);  x0 = N(0,1)^d;
        Bbasis = N(0,1)^{r x d x d} / sqrt(d);  Qbasis[i] = Qc[i] Qc[i]^T / sqrt(d), Qc ~ N(0,1)^{r x d x d}.
    Draw order: Bbasis, Qc, then sA, sB, sQ, sQf, rinv, lgA, lgB, lgQ, x0 for all problems."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    store = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
    rn = lambda *s: torch.randn(*s, generator=gen, device=dev, dtype=torch.float32)
    sp = torch.nn.functional.softplus
    Bb = rn(r, d, d) / d ** 0.5
    Qc = rn(r, d, d)
    Qb = Qc @ Qc.transpose(1, 2) / d ** 0.5
    Qb = 0.5 * (Qb + Qb.transpose(1, 2))
    sA = 0.1 * rn(n, d)
    sB = rn(n, r) / r ** 0.5
    sQ = sp(rn(n, r)) / r
    sQf = sp(rn(n, r)) / r
    rinv = sp(rn(n, d))
    lgA, lgB, lgQ = (0.25 * sp(rn(n, d)) for _ in range(3))
    x0 = rn(n, d)
    c = lambda t: t.to(store).contiguous()
    return ContextualBatch(c(sA), c(sB), c(sQ), c(sQf), c(rinv), c(lgA), c(lgB), c(lgQ), c(Bb), c(Qb), c(x0), T)


BLOCK_WEIGHTS = ("ln_in_gain", "ln_in_offset", "W_in", "b_in", "W_head", "b_head", "W_shared", "b_shared", "Bbasis", "Qc",
                 "ln_out_gain", "ln_out_offset", "W_out", "b_out")


def make_block_weights(C: int, H: int, d: int, r: int, seed: int = 0, device="cpu") -> dict:
    """Random weights of one TTC block (Sec. 4, "Hybrid with Memory Layers"): no trained weights exist, so the draws
    are scaled to give the solver inputs the ranges of make_contextual_batch.  float32, in the order of BLOCK_WEIGHTS:
        ln_in_gain = 1 + 0.1 N^C, ln_in_offset = 0.1 N^C;  W_in = N^{Hd x C} / sqrt(C), b_in = 0.1 N^{Hd};
        W_head (H, 5d + r, d): rows of s_A 0.1 N / sqrt(d); of s_R, s_Qf N / sqrt(d); of the three s_Gamma 0.5 N / sqrt(d);
        b_head: 0 for s_A, 0.1 N for s_R and s_Qf, -1 + 0.1 N for the three s_Gamma;
        W_shared (2r, d): rows of s_B N / sqrt(d r), of s_Q N / sqrt(d);  b_shared = 0.1 N^{2r};
        Bbasis = N^{r x d x d} / sqrt(d);  Qc = N^{r x d x d} / sqrt(r);
        ln_out_gain = 1 + 0.1 N^{Hd}, ln_out_offset = 0.1 N^{Hd};  W_out = N^{C x Hd} / sqrt(Hd), b_out = 0.1 N^C."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    rn = lambda *s: torch.randn(*s, generator=gen, device=dev, dtype=torch.float32)
    w = {}
    w["ln_in_gain"], w["ln_in_offset"] = 1 + 0.1 * rn(C), 0.1 * rn(C)
    w["W_in"], w["b_in"] = rn(H * d, C) / C ** 0.5, 0.1 * rn(H * d)
    Wh, bh = rn(H, 5 * d + r, d) / d ** 0.5, 0.1 * rn(H, 5 * d + r)
    Wh[:, 0:d] *= 0.1
    bh[:, 0:d] = 0
    Wh[:, 2 * d:5 * d] *= 0.5
    bh[:, 2 * d:5 * d] -= 1
    w["W_head"], w["b_head"] = Wh, bh
    Ws = rn(2 * r, d) / d ** 0.5
    Ws[0:r] /= r ** 0.5
    w["W_shared"], w["b_shared"] = Ws, 0.1 * rn(2 * r)
    w["Bbasis"], w["Qc"] = rn(r, d, d) / d ** 0.5, rn(r, d, d) / r ** 0.5
    w["ln_out_gain"], w["ln_out_offset"] = 1 + 0.1 * rn(H * d), 0.1 * rn(H * d)
    w["W_out"], w["b_out"] = rn(C, H * d) / (H * d) ** 0.5, 0.1 * rn(C)
    return {k: w[k].contiguous() for k in BLOCK_WEIGHTS}


def make_block_input(n_tokens: int, C: int, seed: int = 0, device="cpu") -> torch.Tensor:
    """Token features standing in for the attention output: 0.5 + 2 N(0,1)^{n x C} (a mean away from zero, so that a
    layer normalisation that forgot to centre would show), float32."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed + 7919)
    return (0.5 + 2 * torch.randn(n_tokens, C, generator=gen, device=dev, dtype=torch.float32)).contiguous()
