"""Pins of the block oracle (oracle.ttc_block_oracle) against things other than its own formulas: a layer
normalisation and softplus values worked by hand (tests/golden/block_ln_softplus.txt), identities of the two
functions, the paper's statement that a zero output projection leaves the token unchanged, a scalar block with
T = 1 solved by hand with plain Python arithmetic, independence of the heads, sharing of s_B, s_Q across heads, and
the block assembled from the separately pinned contextual_solve."""
import math
import os

import numpy as np
import pytest

from oracle import lqr_oracle
from oracle import ttc_block_oracle as blk
from paper_2603_09221_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "block_ln_softplus.txt")


def read_golden():
    vals = {}
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = np.array([float(x) for x in rest])
    return vals


def weights64(C, H, d, r, seed):
    return {k: v.double().numpy() for k, v in synth.make_block_weights(C, H, d, r, seed=seed).items()}


def test_layer_norm_hand_worked():
    g = read_golden()
    eps = float(g["eps"][0])
    np.testing.assert_allclose(blk.layer_norm(g["x"], np.ones(4), np.zeros(4), eps), g["normalised"], rtol=1e-15)
    np.testing.assert_allclose(blk.layer_norm(g["x"], g["gain"], g["offset"], eps), g["ln"], rtol=1e-15)


def test_softplus_hand_worked_and_identities():
    g = read_golden()
    np.testing.assert_allclose(blk.softplus(g["sp_in"]), g["sp_out"], rtol=1e-15)
    z = np.linspace(-30, 30, 61)
    np.testing.assert_allclose(blk.softplus(z) - blk.softplus(-z), z, rtol=0, atol=1e-13)
    assert np.all(blk.softplus(z) > 0) and np.all(np.diff(blk.softplus(z)) > 0)
    np.testing.assert_allclose(blk.softplus(np.array([800.0, -800.0])), [800.0, 0.0])  # no overflow


def test_layer_norm_shift_and_scale_invariance():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(5, 12))
    gain, off = rng.normal(size=12), rng.normal(size=12)
    ref = blk.layer_norm(x, gain, off, 0.0)
    np.testing.assert_allclose(blk.layer_norm(3.0 * x + 7.0, gain, off, 0.0), ref, rtol=1e-12, atol=1e-12)
    y = blk.layer_norm(x, np.ones(12), np.zeros(12), 0.0)
    np.testing.assert_allclose(y.mean(axis=-1), 0, atol=1e-14)
    np.testing.assert_allclose((y ** 2).mean(axis=-1), 1, rtol=1e-13)
    # each row is normalised on its own
    np.testing.assert_allclose(blk.layer_norm(x[2], gain, off, 0.1), blk.layer_norm(x, gain, off, 0.1)[2], rtol=1e-14)


def test_zero_output_projection_is_the_identity():
    C, H, d, r = 24, 2, 4, 3
    w = weights64(C, H, d, r, seed=1)
    x = synth.make_block_input(7, C, seed=1).double().numpy()
    w["W_out"][:] = 0
    w["b_out"][:] = 0
    out = blk.ttc_block(x, w, T=3)
    np.testing.assert_array_equal(out["x_out"], x)
    assert np.abs(out["o"]).max() > 0


@pytest.mark.parametrize("T", [1, 2])
def test_scalar_block_by_hand(T):
    # C = 2, two heads of one state each, one basis matrix, horizon 1 or 2; every number below follows the equations
    # of Sec. 4 and Prop. 3.1 with plain arithmetic
    sp = lambda z: math.log1p(math.exp(z))
    x = [3.0, 1.0]
    eps = 0.25
    g_in, o_in = [1.5, 0.5], [0.1, -0.2]
    W_in, b_in = [[0.7, -0.4], [0.2, 0.9]], [0.05, -0.1]
    # head maps: rows sA, rinv, lgA, lgB, lgQ, sQf
    Wh = [[0.3, 0.8, 0.2, -0.5, 0.4, 0.6], [-0.2, 0.1, 0.7, 0.3, -0.6, 0.9]]
    bh = [[0.01, 0.02, -0.3, -0.4, -0.5, 0.1], [0.0, -0.1, -0.2, 0.3, 0.2, -0.3]]
    Ws, bs = [0.8, -0.7], [0.2, 0.1]      # sB, sQ
    Bb, Qc = 1.3, 0.9
    g_out, o_out = [1.2, 0.8], [0.3, -0.1]
    W_out, b_out = [[0.5, -0.3], [0.25, 0.75]], [0.02, -0.04]

    mean = 2.0
    var = 1.0
    ln = [(x[i] - mean) / math.sqrt(var + eps) * g_in[i] + o_in[i] for i in range(2)]
    h0 = [W_in[h][0] * ln[0] + W_in[h][1] * ln[1] + b_in[h] for h in range(2)]
    o = []
    for h in range(2):
        z = [Wh[h][k] * h0[h] + bh[h][k] for k in range(6)]
        sA, rinv, lgA, lgB, lgQ, sQf = z[0], sp(z[1]), sp(z[2]), sp(z[3]), sp(z[4]), sp(z[5])
        sB = Ws[0] * h0[h] + bs[0]
        sQ = sp(Ws[1] * h0[h] + bs[1])
        A = lambda t: 1 + math.exp(-t * lgA) * sA
        B = lambda t: sB * Bb * math.exp(-t * lgB)
        Qb = Qc * Qc                # d = 1: Qc^2 / sqrt(1)
        R = 1 / rinv
        P = sQf * Qb                # P_T = Q_T
        for t in range(T, 1, -1):   # P_{t-1} = Q_{t-1} + A_t P_t A_t - (B_t P_t A_t)^2 / (R + B_t P_t B_t)
            Qprev = math.exp(-(t - 1) * lgQ) * sQ * Qb * math.exp(-(t - 1) * lgQ)
            P = Qprev + A(t) * P * A(t) - (B(t) * P * A(t)) ** 2 / (R + B(t) * P * B(t))
        K1 = -(B(1) * P * A(1)) / (R + B(1) * P * B(1))
        o.append(K1 * h0[h])
    m2 = 0.5 * (o[0] + o[1])
    v2 = 0.25 * (o[0] - o[1]) ** 2
    lo = [(o[i] - m2) / math.sqrt(v2 + eps) * g_out[i] + o_out[i] for i in range(2)]
    want = [x[c] + W_out[c][0] * lo[0] + W_out[c][1] * lo[1] + b_out[c] for c in range(2)]

    w = dict(ln_in_gain=g_in, ln_in_offset=o_in, W_in=W_in, b_in=b_in,
             W_head=np.array(Wh)[:, :, None], b_head=bh, W_shared=np.array(Ws)[:, None], b_shared=bs,
             Bbasis=[[[Bb]]], Qc=[[[Qc]]], ln_out_gain=g_out, ln_out_offset=o_out, W_out=W_out, b_out=b_out)
    out = blk.ttc_block(np.array(x), w, T=T, eps=eps)
    np.testing.assert_allclose(out["h0"].reshape(2), h0, rtol=1e-14)
    np.testing.assert_allclose(out["o"], o, rtol=1e-13)
    np.testing.assert_allclose(out["x_out"], want, rtol=1e-13)


def test_heads_are_independent_and_share_sB_sQ():
    C, H, d, r = 16, 3, 4, 2
    w = weights64(C, H, d, r, seed=2)
    x = synth.make_block_input(5, C, seed=2).double().numpy()
    base = blk.ttc_block(x, w, T=4)
    w2 = {k: v.copy() for k, v in w.items()}
    w2["W_head"][1] *= 1.5          # only head 1's own maps
    w2["W_in"][2 * d:3 * d] *= -0.5  # and head 2's initial state
    other = blk.ttc_block(x, w2, T=4)
    o0, o1 = base["o"].reshape(5, H, d), other["o"].reshape(5, H, d)
    np.testing.assert_array_equal(o0[:, 0], o1[:, 0])
    assert np.abs(o0[:, 1] - o1[:, 1]).max() > 1e-6 and np.abs(o0[:, 2] - o1[:, 2]).max() > 1e-6
    # two heads with the same initial state and the same own maps get the same shared coefficients and output
    w3 = {k: v.copy() for k, v in w.items()}
    w3["W_in"][d:2 * d], w3["b_in"][d:2 * d] = w3["W_in"][0:d], w3["b_in"][0:d]
    w3["W_head"][1], w3["b_head"][1] = w3["W_head"][0], w3["b_head"][0]
    same = blk.ttc_block(x, w3, T=4)
    np.testing.assert_array_equal(same["o"].reshape(5, H, d)[:, 0], same["o"].reshape(5, H, d)[:, 1])
    np.testing.assert_array_equal(same["cxt"]["sB"][:, 0], same["cxt"]["sB"][:, 1])


def test_block_from_pinned_pieces_and_activation_ranges():
    # the per-head problem is the one contextual_solve (pinned on its own) defines; Q^(i) is positive semi-definite
    C, H, d, r, T = 32, 2, 16, 16, 6
    w = weights64(C, H, d, r, seed=3)
    x = synth.make_block_input(4, C, seed=3).double().numpy()
    out = blk.ttc_block(x, w, T=T)
    c = out["cxt"]
    for k in ("rinv", "lgA", "lgB", "lgQ", "sQf", "sQ"):
        assert np.all(c[k] > 0), k
    assert np.linalg.eigvalsh(blk.q_basis(w["Qc"])).min() > -1e-12
    tok, h = 2, 1
    one = lqr_oracle.contextual_solve(*(c[k][tok, h] for k in ("sA", "sB", "sQ", "sQf", "rinv", "lgA", "lgB", "lgQ")),
                                      w["Bbasis"], blk.q_basis(w["Qc"]), out["h0"][tok, h], T)
    np.testing.assert_allclose(out["o"][tok, h * d:(h + 1) * d], one["u0"], rtol=1e-12, atol=1e-14)
    # the generator's ranges: the structured inputs look like those of make_contextual_batch
    assert 0.3 < np.std(out["h0"]) < 3 and np.abs(c["sA"]).max() < 2 and c["lgA"].max() < 3
