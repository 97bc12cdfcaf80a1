"""GPU parity of the whole TTC block (ttc_block_forward: LN, input projection, contextualisation maps, structured
solve, LN, output projection, residual; Sec. 4) against the CPU float64 oracle (oracle.ttc_block_oracle.ttc_block),
element by element on the same seeded token features and weights.  Tolerance per token, the larger of the 2-norm and
the element-wise measure: 2e-5 for h_0 (one float32 contraction), 1e-4 for o and x_out (the solver's float32 bar)."""
import numpy as np
import pytest
import torch

from oracle import ttc_block_oracle
from paper_2603_09221_amd import binding, synth
from tests.parity import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run(n, C, H, r, T, seed, eps=1e-5, **kw):
    w = synth.make_block_weights(C, H, 16, r, seed=seed, device=DEV)
    x = synth.make_block_input(n, C, seed=seed, device=DEV)
    out = binding.ttc_block_forward(x, w, T, eps=eps, want_h0=True, want_o=True, **kw)
    torch.cuda.synchronize()
    return x, w, out


def oracle(x, w, T, eps=1e-5):
    return ttc_block_oracle.ttc_block(x.cpu().double().numpy(), {k: v.cpu().double().numpy() for k, v in w.items()}, T, eps)


def check(x, w, out, T, eps=1e-5):
    ref = oracle(x, w, T, eps)
    n = x.shape[0]
    assert int(out["info"].abs().max()) == 0
    errs = {"h0": float(rel_err(out["h0"].cpu().numpy(), ref["h0"].reshape(n, -1)).max()),
            "o": float(rel_err(out["o"].cpu().numpy(), ref["o"]).max()),
            "x_out": float(rel_err(out["x_out"].cpu().numpy(), ref["x_out"]).max())}
    print({k: f"{v:.2e}" for k, v in errs.items()})
    assert errs["h0"] <= 2e-5 and errs["o"] <= 1e-4 and errs["x_out"] <= 1e-4, errs
    return ref


@pytest.mark.parametrize("n,C,H,r,T", [(300, 256, 4, 16, 8),      # several row tiles and a ragged one
                                        (1, 64, 1, 16, 4),         # one token, one head: tiles mostly empty
                                        (129, 100, 3, 4, 5),       # C not a multiple of the K slice, H*16 = 48 < a tile
                                        (517, 512, 16, 16, 3),     # two tiles of outputs in the input projection
                                        (70, 36, 9, 64, 2),        # H*16 = 144: a ragged second tile of W_in; most bases
                                        (2050, 128, 2, 8, 16)])    # four problems per wavefront in the solve
def test_block_against_oracle(n, C, H, r, T):
    x, w, out = run(n, C, H, r, T, seed=n + C + H + r + T)
    check(x, w, out, T)


def test_layer_norm_epsilon_and_offset_inputs():
    # a large eps changes both normalisations; token features far from zero mean
    w = synth.make_block_weights(96, 2, 16, 16, seed=5, device=DEV)
    x = 40.0 + synth.make_block_input(65, 96, seed=5, device=DEV)
    out = binding.ttc_block_forward(x, w, 6, eps=0.3, want_h0=True, want_o=True)
    torch.cuda.synchronize()
    check(x, w, out, 6, eps=0.3)


def test_zero_output_projection_returns_the_input_bit_for_bit():
    w = synth.make_block_weights(128, 4, 16, 16, seed=6, device=DEV)
    w["W_out"].zero_()
    w["b_out"].zero_()
    x = synth.make_block_input(200, 128, seed=6, device=DEV)
    out = binding.ttc_block_forward(x, w, 8)
    torch.cuda.synchronize()
    assert torch.equal(out["x_out"], x)


def test_in_place_and_caller_workspace_and_side_stream():
    x, w, ref = run(333, 192, 4, 16, 8, seed=7)
    blk = binding.make_block(w, 333, 8)
    need = binding.load().ttc_block_workspace_bytes(blk)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    y = x.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    out = binding.ttc_block_forward(y, w, 8, out={"x_out": y}, workspace=ws, stream=side)
    side.synchronize()
    assert torch.equal(out["x_out"], ref["x_out"]) and out["x_out"].data_ptr() == y.data_ptr()
    with pytest.raises(binding.TtcError):
        binding.ttc_block_forward(x, w, 8, workspace=ws[: need - 64])


def test_a_bad_token_stays_alone():
    w = synth.make_block_weights(64, 2, 16, 16, seed=8, device=DEV)
    x = synth.make_block_input(260, 64, seed=8, device=DEV)
    good = binding.ttc_block_forward(x, w, 5)
    xb = x.clone()
    xb[131, 7] = float("nan")
    bad = binding.ttc_block_forward(xb, w, 5)
    torch.cuda.synchronize()
    keep = torch.ones(260, dtype=torch.bool, device=DEV)
    keep[131] = False
    assert torch.equal(bad["x_out"][keep], good["x_out"][keep])
    assert bool(torch.isnan(bad["x_out"][131]).all())
    assert int(bad["info"][keep].abs().max()) == 0 and int(bad["info"][131].abs().min()) != 0


def test_unsupported_shapes_are_refused():
    w = synth.make_block_weights(64, 2, 16, 16, seed=9, device=DEV)
    x = synth.make_block_input(4, 64, seed=9, device=DEV)
    w6 = synth.make_block_weights(66, 2, 16, 16, seed=9, device=DEV)       # C not a multiple of 4
    with pytest.raises(binding.TtcError):
        binding.ttc_block_forward(synth.make_block_input(4, 66, seed=9, device=DEV), w6, 5)
    w8 = synth.make_block_weights(64, 2, 8, 16, seed=9, device=DEV)        # heads of 8 states
    with pytest.raises(binding.TtcError):
        binding.ttc_block_forward(x, w8, 5)
    with pytest.raises(binding.TtcError):
        binding.ttc_block_forward(x, w, 0)                                  # no horizon
    assert binding.ttc_block_forward(x[:0], w, 5)["x_out"].shape == (0, 64)  # no tokens: nothing to do


def bf16_case(n, C, H, r, T, seed):
    w = synth.make_block_weights(C, H, 16, r, seed=seed, device=DEV)
    w["W_in"], w["W_out"] = w["W_in"].bfloat16().contiguous(), w["W_out"].bfloat16().contiguous()
    x = synth.make_block_input(n, C, seed=seed, device=DEV).bfloat16().contiguous()
    return x, w


@pytest.mark.parametrize("n,C,H,r,T", [(300, 256, 4, 16, 8), (1, 64, 1, 16, 4), (131, 104, 3, 4, 5), (517, 512, 16, 16, 3),
                                        (70, 40, 9, 64, 2)])
def test_bf16_block_against_oracle(n, C, H, r, T):
    """bfloat16 token features and projection weights (TTC_BLOCK_FLAG_BF16): the oracle consumes the stored (rounded)
    values; 2e-2, the bar for bfloat16 inputs, on h0, o and x_out (x_out is itself rounded to bfloat16)."""
    x, w = bf16_case(n, C, H, r, T, seed=n + C + H + r + T)
    out = binding.ttc_block_forward(x, w, T, want_h0=True, want_o=True)
    torch.cuda.synchronize()
    assert out["x_out"].dtype == torch.bfloat16 and int(out["info"].abs().max()) == 0
    ref = oracle(x.float(), {k: v.float() for k, v in w.items()}, T)
    errs = {"h0": float(rel_err(out["h0"].cpu().numpy(), ref["h0"].reshape(n, -1)).max()),
            "o": float(rel_err(out["o"].cpu().numpy(), ref["o"]).max()),
            "x_out": float(rel_err(out["x_out"].float().cpu().numpy(), ref["x_out"]).max())}
    print({k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= 2e-2, (k, v)


def test_bf16_block_in_place_zero_projection_and_refusals():
    x, w = bf16_case(200, 128, 4, 16, 6, seed=11)
    ref = binding.ttc_block_forward(x, w, 6)
    y = x.clone()
    out = binding.ttc_block_forward(y, w, 6, out={"x_out": y})
    torch.cuda.synchronize()
    assert torch.equal(out["x_out"], ref["x_out"])
    w0 = dict(w)
    w0["W_out"] = torch.zeros_like(w["W_out"])
    w0["b_out"] = torch.zeros_like(w["b_out"])
    same = binding.ttc_block_forward(x, w0, 6)
    torch.cuda.synchronize()
    assert torch.equal(same["x_out"], x)                      # a zero output projection returns the input bit for bit
    with pytest.raises(ValueError):
        binding.ttc_block_forward(x.float(), w, 6)            # float32 features with bfloat16 projections
    xw, ww = bf16_case(4, 68, 2, 16, 3, seed=12)              # C a multiple of 4 but not of 8
    with pytest.raises(binding.TtcError):
        binding.ttc_block_forward(xw, ww, 3)
