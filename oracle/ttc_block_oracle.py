"""CPU float64 oracle for the whole Test-Time Control block around the solver.

TEST INFRASTRUCTURE ONLY.  Plain numpy, float64, one statement per equation; shares no code with the GPU library,
never imports it, and is called only from tests, the smoke check and the cpu_baseline leg of the benchmark.

What it computes (Sec. 4, "Hybrid with Memory Layers", "Multi-Head Structure", "Contextualization",
"Parameterization"), for every token feature x_in (C numbers) on its own:

    h_0   = W_in LN(x_in) + b_in                           (H heads of d numbers each)
    per head h, from that head's d numbers h_0^(h):
        sA  = W_A^(h) h_0^(h) + b_A^(h)                    A_t = I + Gamma_A^t diag(sA)
        rinv = softplus(W_R^(h) h_0^(h) + b_R^(h))         R_t = diag(1 / rinv)   (the map hands over diag(R^{-1}))
        lgX = softplus(W_gX^(h) h_0^(h) + b_gX^(h))        Gamma_X = exp(-diag(lgX)),  X in {A, B, Q}
        sQf = softplus(W_Qf^(h) h_0^(h) + b_Qf^(h))        Q_T = sum_i sQf[i] Q^(i)
        sB  = W_B h_0^(h) + b_B                            (W_B, W_Q and the bases are shared by all heads)
        sQ  = softplus(W_Q h_0^(h) + b_Q)
        Q^(i) = Qc^(i) Qc^(i)^T / sqrt(d)
        o^(h) = u_1^* of the problem these parameters define, started from h_0^(h)  (oracle.lqr_oracle.contextual_solve)
    o     = the heads' outputs side by side
    x_out = x_in + W_out LN(o) + b_out

LN is the layer normalisation over the last axis with a biased variance, eps inside the root, then a gain and an
offset per entry.  softplus(z) = log(1 + exp(z)).

Readings where the paper leaves a choice: the activations of s_A and s_B are the identity, that of s_Qf is the
softplus (the terminal cost must be positive semi-definite like the others); every linear map has an offset;
the layer's output o is the first optimal control u_1^*; s_A, s_R, s_Qf and the three s_Gamma are per head.

Pins (tests/test_block_oracle_pins.py): a layer normalisation and a softplus worked by hand (tests/golden/
block_ln_softplus.txt), softplus(z) - softplus(-z) = z, invariance of LN under shift and scale of its input, a zero
output projection leaves the token unchanged (the paper's statement for fine-tuning), a scalar block with T = 1
solved by hand, independence of the heads, and the block assembled from separately pinned pieces.
"""
from __future__ import annotations

import numpy as np

from . import lqr_oracle

HEAD_ROWS = ("sA", "rinv", "lgA", "lgB", "lgQ", "sQf")   # row groups of W_head, in this order; sQf has r rows, the others d
SHARED_ROWS = ("sB", "sQ")                               # row groups of W_shared, r rows each


def layer_norm(x, gain, offset, eps):
    x = np.asarray(x, dtype=np.float64)
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    return (x - mean) / np.sqrt(var + eps) * np.asarray(gain, dtype=np.float64) + np.asarray(offset, dtype=np.float64)


def softplus(z):
    z = np.asarray(z, dtype=np.float64)
    return np.logaddexp(0.0, z)


def contextual_inputs(h0, W_head, b_head, W_shared, b_shared, d, r):
    """The per-problem vectors of the structured parameterisation from the heads' initial states.

    h0: (..., H, d);  W_head: (H, 5d + r, d), b_head: (H, 5d + r), rows in the order HEAD_ROWS;
    W_shared: (2r, d), b_shared: (2r), rows in the order SHARED_ROWS.  Returns a dict of (..., H, d) / (..., H, r)."""
    h0 = np.asarray(h0, dtype=np.float64)
    W_head, b_head = np.asarray(W_head, dtype=np.float64), np.asarray(b_head, dtype=np.float64)
    W_shared, b_shared = np.asarray(W_shared, dtype=np.float64), np.asarray(b_shared, dtype=np.float64)
    zh = np.einsum("hod,...hd->...ho", W_head, h0) + b_head      # each head's own maps
    zs = np.einsum("od,...hd->...ho", W_shared, h0) + b_shared   # the same maps for every head
    out = {}
    out["sA"] = zh[..., 0 * d:1 * d]
    out["rinv"] = softplus(zh[..., 1 * d:2 * d])
    out["lgA"] = softplus(zh[..., 2 * d:3 * d])
    out["lgB"] = softplus(zh[..., 3 * d:4 * d])
    out["lgQ"] = softplus(zh[..., 4 * d:5 * d])
    out["sQf"] = softplus(zh[..., 5 * d:5 * d + r])
    out["sB"] = zs[..., 0:r]
    out["sQ"] = softplus(zs[..., r:2 * r])
    return out


def q_basis(Qc):
    Qc = np.asarray(Qc, dtype=np.float64)
    d = Qc.shape[-1]
    return Qc @ np.swapaxes(Qc, -1, -2) / np.sqrt(d)


def ttc_block(x_in, w, T, eps=1e-5):
    """x_out (..., C) and the intermediate results, for token features x_in (..., C) and the weights w, a dict with
    ln_in_gain, ln_in_offset (C), W_in (H*d, C), b_in (H*d), W_head, b_head, W_shared, b_shared (see
    contextual_inputs), Bbasis, Qc (r, d, d), ln_out_gain, ln_out_offset (H*d), W_out (C, H*d), b_out (C)."""
    x_in = np.asarray(x_in, dtype=np.float64)
    f = lambda k: np.asarray(w[k], dtype=np.float64)
    r, d = f("Bbasis").shape[0], f("Bbasis").shape[-1]
    H = f("W_in").shape[0] // d
    h0 = layer_norm(x_in, f("ln_in_gain"), f("ln_in_offset"), eps) @ f("W_in").T + f("b_in")
    h0 = h0.reshape(x_in.shape[:-1] + (H, d))
    c = contextual_inputs(h0, f("W_head"), f("b_head"), f("W_shared"), f("b_shared"), d, r)
    sol = lqr_oracle.contextual_solve(c["sA"], c["sB"], c["sQ"], c["sQf"], c["rinv"], c["lgA"], c["lgB"], c["lgQ"],
                                      f("Bbasis"), q_basis(f("Qc")), h0, T)
    o = sol["u0"].reshape(x_in.shape[:-1] + (H * d,))
    x_out = x_in + layer_norm(o, f("ln_out_gain"), f("ln_out_offset"), eps) @ f("W_out").T + f("b_out")
    return {"x_out": x_out, "h0": h0, "o": o, "cxt": c}
