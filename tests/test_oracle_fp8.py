"""Pins for the oracle's E4M3 codec and quantisers.  No GPU."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from synth.moe_inputs import MoEConfig, make_inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e4m3_landmarks.txt")


def test_decode_landmarks():
    with open(GOLDEN) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            code_s, val_s = line.split()
            got = float(O.e4m3_decode(np.array([int(code_s, 16)]))[0])
            want = float(val_s)
            if math.isnan(want):
                assert math.isnan(got)
            else:
                assert got == want and math.copysign(1, got) == math.copysign(1, want), code_s


def test_decode_matches_torch_float8_for_all_codes():
    codes = np.arange(256, dtype=np.uint8)
    t = torch.tensor(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = O.e4m3_decode(codes)
    assert np.array_equal(np.isnan(t), np.isnan(ours))
    ok = ~np.isnan(t)
    assert np.array_equal(t[ok], ours[ok])


def test_encode_roundtrip_monotone_midpoints_saturation():
    codes = np.arange(256, dtype=np.uint8)
    vals = O.e4m3_decode(codes)
    finite = ~np.isnan(vals)
    back = O.e4m3_encode(vals[finite])
    assert np.array_equal(back, codes[finite])          # includes -0 -> 0x80
    # monotone on a fine grid
    grid = np.linspace(-460, 460, 200001)
    dec = O.e4m3_decode(O.e4m3_encode(grid))
    assert np.all(np.diff(dec) >= 0)
    # nearest: the decoded value is never farther than half the local spacing
    pos = np.sort(vals[finite & (vals >= 0)])
    g = np.abs(grid[np.abs(grid) <= 448])
    nearest = pos[np.abs(pos[None, :] - g[:, None]).argmin(axis=1)]
    d = O.e4m3_decode(O.e4m3_encode(g))
    assert np.all(np.abs(d - g) <= np.abs(nearest - g) + 1e-15)
    # midpoints go to the even mantissa
    for v, want in ((17.0, 16.0), (19.0, 20.0), (2.0 ** -10, 0.0), (3 * 2.0 ** -10, 2.0 ** -8),
                    (1.0625, 1.0), (1.1875, 1.25), (432.0, 448.0), (15 * 2.0 ** -10, 2.0 ** -6)):
        assert float(O.e4m3_decode(O.e4m3_encode(np.array([v])))[0]) == want, v
        assert float(O.e4m3_decode(O.e4m3_encode(np.array([-v])))[0]) == -want, v
    # saturation, no NaN produced from finite input
    for v in (449.0, 464.0, 500.0, 1e30):
        assert O.e4m3_encode(np.array([v]))[0] == 0x7E
        assert O.e4m3_encode(np.array([-v]))[0] == 0xFE
    assert O.e4m3_encode(np.array([np.nan]))[0] & 0x7F == 0x7F


def test_encode_agrees_with_torch_cast_in_range():
    rng = np.random.default_rng(0)
    v = (rng.standard_normal(200000) * np.exp(rng.uniform(-8, 6, 200000))).astype(np.float32)
    v = v[np.abs(v) <= 448]
    t = torch.tensor(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(O.e4m3_encode(v), t)


def test_quant_rows_properties():
    rng = np.random.default_rng(1)
    v = (rng.standard_normal((33, 64)) * np.exp(rng.uniform(-3, 3, (33, 1)))).astype(np.float32)
    v[5] = 0.0
    codes, scales = O.quant_rows(v)
    assert codes.dtype == np.uint8 and scales.dtype == np.float32
    assert scales[5] == 1.0 and np.all(codes[5] == 0)
    amax = np.abs(v).max(axis=1)
    for r in range(33):
        if r == 5:
            continue
        assert scales[r] == np.float32(amax[r]) / np.float32(448.0)
        j = int(np.abs(v[r]).argmax())
        assert codes[r, j] & 0x7F == 0x7E          # the row maximum lands on +-448
    deq = O.dequant_rows(codes, scales)
    # e4m3 keeps 3 mantissa bits: relative error <= 2^-4 for normals, absolute 2^-10*scale below
    bound = np.maximum(np.abs(v) * 2.0 ** -4, scales[:, None].astype(np.float64) * 2.0 ** -10) * (1 + 1e-6)
    assert np.all(np.abs(deq - v) <= bound)


def test_quant_colgroup128_equals_row_quant_of_transposed_groups():
    rng = np.random.default_rng(2)
    v = rng.standard_normal((300, 16)).astype(np.float32) * 3
    codes, scales = O.quant_colgroup128(v)
    assert scales.shape == (3, 16)
    for g in range(3):
        blk = v[g * 128:(g + 1) * 128]
        c_t, s_t = O.quant_rows(np.ascontiguousarray(blk.T))
        assert np.array_equal(codes[g * 128:(g + 1) * 128], c_t.T)
        assert np.array_equal(scales[g], s_t)
    deq = O.dequant_colgroup128(codes, scales)
    assert np.all(np.abs(deq - v) <= np.abs(v) * 2.0 ** -4 + 1e-2)


def test_fp8_gemm1_exact_when_operands_are_representable():
    """Inputs whose scaled values are exact e4m3 numbers lose nothing, so H of the fp8 layer
    equals H of the plain layer bit for bit."""
    cfg = MoEConfig("t", T=32, d=16, E=3, k=2, f=8, dtype="f32", w_std=1.0, wr_std=1.0)
    rng = np.random.default_rng(3)
    grid = np.array([0, 1, 2, 3, 3.5, 4, 5, 6, 7, -1, -2, -3, -3.5, -4, -5, -6, -7], dtype=np.float32)
    x = rng.choice(grid, size=(cfg.T, cfg.d)).astype(np.float32)
    x[:, 0] = 7.0                                        # amax = 7 -> inv = 64, scale = 1/64
    W1 = rng.choice(grid, size=(cfg.E, 2 * cfg.f, cfg.d)).astype(np.float32) * 0.125
    W1[:, :, 1] = 7.0 * 0.125
    W2 = rng.choice(grid, size=(cfg.E, cfg.d, cfg.f)).astype(np.float32)
    W2[:, :, 0] = 7.0
    z = rng.standard_normal((cfg.T, cfg.E)).astype(np.float32)
    q = O.layer_fwd_fp8(x, z, W1, W2, cfg.k)
    p = O.layer_fwd(x, z, W1, W2, cfg.k)
    assert np.array_equal(q["H"], p["H"])
    assert np.array_equal(q["xp"], p["xp"])


def test_fp8_layer_close_to_plain_layer_and_straight_through_backward():
    cfg = MoEConfig("t", T=64, d=32, E=4, k=2, f=24, dtype="bf16", w_std=0.2, wr_std=0.3)
    inp = make_inputs(cfg, seed=1)
    z = O.router_logits(inp["x"], inp["W_r"]).astype(np.float32)
    q = O.layer_fwd_fp8(inp["x"], z, inp["W1"], inp["W2"], cfg.k)
    p = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k)
    assert np.array_equal(q["idx"], p["idx"]) and np.array_equal(q["perm"], p["perm"])
    err = np.abs(q["y"] - p["y"]).max() / np.abs(p["y"]).max()
    assert 1e-4 < err < 0.15
    gq = O.layer_bwd_fp8(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], q)
    gp = O.layer_bwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], p)
    for name in ("dx", "dW1", "dW2", "dw"):
        e = np.abs(gq[name] - gp[name]).max() / np.abs(gp[name]).max()
        assert e < 0.2, (name, e)
    # straight-through: with casts that change nothing (dy on the e4m3 grid per group, and the
    # forward tensors taken from the fp8 forward) the backward is the plain backward of those tensors
    dy_hat = gq["dy_hat"]
    g2 = O.layer_bwd_fp8(inp["x"], z, inp["W1"], inp["W2"], cfg.k, dy_hat, q)
    assert np.allclose(g2["dy_hat"], dy_hat, rtol=0, atol=0)
    dYp = O.dispatch(dy_hat, q["perm"], cfg.k, row_mul=q["w"])
    dxp, dW1, dW2, _ = O.expert_ffn_bwd(q["xp"], q["H"], dYp, q["offsets"], inp["W1"], inp["W2"], A=q["A"])
    assert np.array_equal(g2["dW1"], dW1) and np.array_equal(g2["dW2"], dW2)
