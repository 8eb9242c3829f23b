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


# ---- FP8 backward GEMMs (Section 7: per-channel quantisation within 128-token groups) --------------------
def test_pow2_exponent_is_the_smallest_power_of_two_that_fits():
    # landmarks worked out by hand: 448 = 1.75 * 2^8
    for amax, k in ((448.0, 0), (448.5, 1), (896.0, 1), (224.0, -1), (225.0, 0), (1.75, -8), (1.76, -7),
                    (0.0, 0), (2.0 ** -20, -28), (3.0e38, 120)):
        assert int(O.pow2_exponent(np.array([amax]))[0]) == k, amax
    rng = np.random.default_rng(5)
    a = np.abs(rng.standard_normal(2000)) * np.exp2(rng.integers(-30, 30, 2000))
    k = O.pow2_exponent(a)
    assert np.all(a * np.exp2(-k.astype(np.float64)) <= 448.0)
    assert np.all(a * np.exp2(-(k - 1).astype(np.float64)) > 448.0)
    assert int(O.pow2_exponent(np.array([1e-45]))[0]) == -126          # clamped


def test_token_groups_never_span_experts():
    assert O.token_groups([0, 130, 130, 386]) == [(0, 0, 128), (0, 128, 130), (2, 130, 258), (2, 258, 386)]
    assert O.token_groups([0, 0, 5]) == [(1, 0, 5)]
    assert O.token_groups([0, 0]) == []


def _nearest_code_brute(p):
    """Nearest e4m3 value by exhaustive search over the 256 codes, ties to the even mantissa."""
    vals = O.e4m3_decode(np.arange(256, dtype=np.uint8))
    best, bd = None, None
    for c in range(256):
        if np.isnan(vals[c]) or (c == 0x80 and p >= 0) or (c == 0x00 and (p < 0 or (p == 0 and np.signbit(p)))):
            continue
        dist = abs(vals[c] - p)
        if bd is None or dist < bd or (dist == bd and (c & 1) == 0 and (best & 1) == 1):
            best, bd = c, dist
    return best


def test_quant_tokengroup_pow2_against_brute_force():
    rng = np.random.default_rng(11)
    offsets = [0, 3, 3, 140, 150]
    v = (rng.standard_normal((150, 5)) * np.exp2(rng.integers(-3, 6, (150, 5)))).astype(np.float32)
    v[10:20, 2] = 0.0
    v[3:140, 4] = 0.0                                     # a whole-zero (group, column): exponent 0, codes 0
    codes, exps = O.quant_tokengroup_pow2(v, offsets)
    groups = [(0, 3), (3, 131), (131, 140), (140, 150)]
    assert exps.shape == (4, 5)
    for gi, (lo, hi) in enumerate(groups):
        for c in range(5):
            amax = float(np.abs(v[lo:hi, c]).max())
            k = 0
            if amax > 0:
                while amax * 2.0 ** -k > 448.0:
                    k += 1
                while amax * 2.0 ** -(k - 1) <= 448.0:
                    k -= 1
            assert exps[gi, c] == k
            for t in range(lo, hi, 7):
                assert codes[t, c] == _nearest_code_brute(float(v[t, c]) * 2.0 ** -k), (t, c)
    deq = O.dequant_tokengroup_pow2(codes, exps, offsets)
    assert np.all(np.abs(deq - v) <= np.abs(v) * 2.0 ** -4 + np.exp2(exps.max()) * 2.0 ** -9)


def test_fp8_backward_gemms_exact_on_representable_operands_and_close_otherwise():
    # (a) exactness: every operand of dA and dW2 lies on its e4m3 grid, so they equal the plain backward bit for bit
    cfg = MoEConfig("t", T=40, d=16, E=3, k=2, f=8, dtype="f32", w_std=1.0, wr_std=1.0)
    rng = np.random.default_rng(4)
    grid = np.array([0, 1, 2, 3, 3.5, 4, 5, 6, 7, -1, -2, -3, -3.5, -4, -5, -6, -7], dtype=np.float32)
    M = cfg.T * cfg.k
    offsets = np.array([0, 30, 30, 80])
    dYp = rng.choice(grid, size=(M, cfg.d)).astype(np.float32)
    dYp[:, 0] = 7.0                                       # row amax 7 -> scale 1/64; column amax 7 -> 2^-6
    dYp[0::2, :] *= 0.5
    A = rng.choice(grid, size=(M, cfg.f)).astype(np.float32)
    A[0, :] = 7.0; A[30, :] = 7.0
    xp = rng.choice(grid, size=(M, cfg.d)).astype(np.float32)
    H = rng.standard_normal((M, 2 * cfg.f))
    W1 = rng.standard_normal((cfg.E, 2 * cfg.f, cfg.d)).astype(np.float32)
    W2 = rng.choice(grid, size=(cfg.E, cfg.d, cfg.f)).astype(np.float32)
    W2[:, 0, :] = 7.0                                     # every row of W2^T has amax 7
    q = O.expert_ffn_bwd_fp8(xp, H, dYp, A, offsets, W1, W2)
    dxp, dW1, dW2, dH = O.expert_ffn_bwd(xp, H, dYp.astype(np.float64), offsets, W1, W2, A=A.astype(np.float64))
    dA_plain = np.zeros((M, cfg.f))
    for e in range(cfg.E):
        lo, hi = offsets[e], offsets[e + 1]
        dA_plain[lo:hi] = dYp[lo:hi].astype(np.float64) @ W2[e].astype(np.float64)
    assert np.array_equal(q["dA"], dA_plain)
    assert np.array_equal(q["dW2"], dW2)
    assert np.array_equal(q["dH"], dH)
    # (b) the rest carries quantisation error only: a transposed operand, a dropped term or a wrong sign would be O(1)
    for name, ref in (("dxp", dxp), ("dW1", dW1)):
        e = np.abs(q[name] - ref).max() / np.abs(ref).max()
        assert 1e-5 < e < 0.12, (name, e)


def test_layer_bwd_fp8_gemm_close_to_straight_through_bf16_backward():
    cfg = MoEConfig("t", T=96, d=32, E=4, k=2, f=24, dtype="bf16", w_std=0.2, wr_std=0.3)
    inp = make_inputs(cfg, seed=2)
    z = O.router_logits(inp["x"], inp["W_r"]).astype(np.float32)
    q = O.layer_fwd_fp8(inp["x"], z, inp["W1"], inp["W2"], cfg.k)
    g8 = O.layer_bwd_fp8_gemm(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], q)
    gs = O.layer_bwd_fp8(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], q)
    assert np.array_equal(g8["dw"], gs["dw"]) and np.array_equal(g8["dYp"], gs["dYp"])
    for name in ("dx", "dW1", "dW2", "dH", "dz"):
        e = np.abs(g8[name] - gs[name]).max() / max(np.abs(gs[name]).max(), 1e-30)
        assert e < 0.12, (name, e)
    assert np.abs(g8["dW1"] - gs["dW1"]).max() > 0


def _exact_fp8_layer_inputs():
    """A layer on which every cast of the fp8 forward is lossless up to the output: all of x, W1, W2, the SwiGLU
    output A and the FC2 output Y lie on the e4m3 grid of their row, and every row maximum is 7 * 2^j (so that
    448 / amax and amax / 448 are powers of two).  G = 64 everywhere, where silu(G) = G exactly in float64
    (1 + e^-64 rounds to 1); U, A = 64 U and Y are small integers times powers of two."""
    T, d, E, k, f = 32, 16, 3, 2, 8
    rng = np.random.default_rng(11)
    pow2 = np.array([0, 1, 2, 4, 8, 16, -1, -2, -4, -8, -16], dtype=np.float32)
    x = rng.choice(pow2, size=(T, d)).astype(np.float32)
    x[:, 0] = 8.0          # drives G
    x[:, 1] = 28.0         # row maximum 7 * 4; no weight reads this column
    x[:, 2] = 0.0          # the weights keep their own row maxima in this column
    x[:, 3] = 16.0         # drives the largest U
    W1 = np.zeros((E, 2 * f, d), dtype=np.float32)
    W2 = np.zeros((E, d, f), dtype=np.float32)
    n_dead, n_top = f - 1, 0
    for e in range(E):
        W1[e, :f, 0] = 8.0                                   # G = 8 * 8 = 64
        W1[e, :f, 2] = 14.0                                  # row maximum 7 * 2 (multiplies x[:, 2] = 0)
        for n in range(f):
            W1[e, f + n, 2] = 7.0                            # row maximum 7
            if n == n_dead:
                continue                                     # U = 0 in this column: FC2's row maxima live here
            p = 3 if n == n_top else int(rng.integers(4, d))
            W1[e, f + n, p] = 7.0 if n == n_top else float(rng.choice([1, 2, 3, 4, 5, 6, 7, -3, -5, -7]))
        for c in range(d):
            W2[e, c, n_dead] = 7.0                           # row maximum 7 (multiplies A[:, n_dead] = 0)
            n = n_top if c == 0 else int(rng.integers(0, f - 1))
            W2[e, c, n] = 4.0 if c == 0 else float(rng.choice([1, 2, 4, -1, -2, -4]))
    z = rng.standard_normal((T, E)).astype(np.float32)
    return x, z, W1, W2, k


def test_fp8_layer_exact_through_fc2_and_output_when_every_cast_is_lossless():
    """Pins the axis of the W2 cast, the placement of the A and Y casts and the gate weight after the dequantised
    Y: on grid-aligned tensors the fp8 layer equals the plain layer bit for bit, up to y."""
    x, z, W1, W2, k = _exact_fp8_layer_inputs()
    q = O.layer_fwd_fp8(x, z, W1, W2, k)
    p = O.layer_fwd(x, z, W1, W2, k)
    assert np.all(p["H"][:, : W1.shape[1] // 2] == 64.0)
    assert np.abs(p["A"]).max() == 64.0 * 112.0 and np.count_nonzero(p["Y"]) > p["Y"].size // 2
    for name in ("xp", "H", "A", "Y", "y"):
        assert np.array_equal(q[name], p[name]), name


def test_fp8_layer_exactness_case_detects_planted_mistakes(monkeypatch):
    """The same case with a mistake planted in the oracle: W2 cast along its other axis, and the gate weight
    applied before the Y cast instead of after it; either breaks the equality."""
    x, z, W1, W2, k = _exact_fp8_layer_inputs()
    p = O.layer_fwd(x, z, W1, W2, k)

    def wrong_axis(W1_, W2_):
        E, two_f, d = W1_.shape
        f = W2_.shape[2]
        W1h = O.fake_quant_rows(np.float32(W1_).reshape(E * two_f, d)).reshape(E, two_f, d)
        W2t = np.ascontiguousarray(np.transpose(np.float32(W2_), (0, 2, 1)))
        W2h = np.transpose(O.fake_quant_rows(W2t.reshape(E * f, d)).reshape(E, f, d), (0, 2, 1))
        return W1h, W2h

    monkeypatch.setattr(O, "quant_weights", wrong_axis)
    q = O.layer_fwd_fp8(x, z, W1, W2, k)
    assert np.array_equal(q["H"], p["H"]) and not np.array_equal(q["Y"], p["Y"])
    monkeypatch.undo()

    real_combine, real_fq = O.combine, O.fake_quant_rows

    def weight_before_cast(Y_hat, inv_perm, w, T, k_):
        # what a cast of w * Y would give: quantise the weighted rows, then sum without weights
        wrow = np.zeros(Y_hat.shape[0])
        wrow[inv_perm.reshape(-1)] = np.asarray(w, np.float64).reshape(-1)
        return real_combine(real_fq(Y_hat * wrow[:, None]), inv_perm, None, T, k_)

    monkeypatch.setattr(O, "combine", weight_before_cast)
    q = O.layer_fwd_fp8(x, z, W1, W2, k)
    assert not np.array_equal(q["y"], p["y"])


# ---- storage-precision mode: casts decide on what a bf16 pipeline holds ------------------------------------------
def test_bf16_round_matches_torch_and_breaks_ties_to_even():
    """Pin: the oracle's bfloat16 rounding against torch's conversion (an independent routine), on random values
    over many binades and on exact ties, which must go to the even mantissa."""
    rng = np.random.default_rng(5)
    v = (rng.standard_normal(200000) * np.exp2(rng.integers(-40, 40, 200000))).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.bf16_round(v), ref)
    assert O.bf16_round(v.reshape(400, 500)).shape == (400, 500)
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7: goes to 1 (even); 1 + 3 * 2^-8 goes up to 1 + 2^-6 (even)
    ties = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 1 + 2.0 ** -8 + 2.0 ** -20, 0.0, -0.0])
    want = np.array([1.0, 1 + 2.0 ** -6, -1.0, 1 + 2.0 ** -7, 0.0, 0.0])
    assert np.array_equal(O.bf16_round(ties), want)
    # float64 inputs are first rounded to float32, then to bf16, as a float32 producer would have done
    assert O.bf16_round(np.array([1 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0


def test_fp8_layer_in_bf16_storage_mode():
    """store="bf16" changes nothing but where the three handed-over tensors are rounded:
    (a) on the lossless case (all of H, A, Y are small integers times powers of two, exact in bf16) it equals the
        float64 mode, forward and both backwards, bit for bit;
    (b) on random inputs H is bf16-representable and within half a bf16 ulp of the float64 mode's H, the SwiGLU
        output fed to its cast is the bf16 rounding of SwiGLU of that H, and y stays within the distance a few
        flipped e4m3 codes allow;
    (c) the backward on e4m3 operands casts the bf16 rounding of dH: dH itself comes back bf16-representable."""
    x, z, W1, W2, k = _exact_fp8_layer_inputs()
    q0, q1 = O.layer_fwd_fp8(x, z, W1, W2, k), O.layer_fwd_fp8(x, z, W1, W2, k, store="bf16")
    for name in ("H", "A", "Y", "y"):
        assert np.array_equal(q0[name], q1[name]), name
    dy = np.random.default_rng(2).choice([1.0, -2.0, 4.0, 0.5], size=q0["y"].shape)
    g0, g1 = O.layer_bwd_fp8_gemm(x, z, W1, W2, k, dy, q0), O.layer_bwd_fp8_gemm(x, z, W1, W2, k, dy, q1, store=None)
    for name in ("dx", "dW1", "dW2", "dz"):
        assert np.array_equal(g0[name], g1[name]), name

    cfg = MoEConfig("t", T=96, d=64, E=4, k=2, f=48, dtype="bf16", w_std=0.2, wr_std=0.3)
    inp = make_inputs(cfg, seed=21)
    inp["logits"] = O.router_logits(inp["x"], inp["W_r"]).astype(np.float32)
    a = O.layer_fwd_fp8(inp["x"], inp["logits"], inp["W1"], inp["W2"], cfg.k)
    b = O.layer_fwd_fp8(inp["x"], inp["logits"], inp["W1"], inp["W2"], cfg.k, store="bf16")
    assert np.array_equal(O.bf16_round(b["H"]), b["H"])
    assert not np.array_equal(a["H"], b["H"])
    assert np.all(np.abs(a["H"] - b["H"]) <= np.abs(a["H"]) * 2.0 ** -8 + 1e-300)
    f = cfg.f
    pre = O.bf16_round(O.silu(b["H"][:, :f]) * b["H"][:, f:])
    assert np.array_equal(b["A"], O.fake_quant_rows(pre))
    assert np.linalg.norm(a["y"] - b["y"]) / np.linalg.norm(a["y"]) < 5e-2
    with pytest.raises(ValueError):
        O.layer_fwd_fp8(inp["x"], inp["logits"], inp["W1"], inp["W2"], cfg.k, store="fp16")
    g = O.layer_bwd_fp8_gemm(inp["x"], inp["logits"], inp["W1"], inp["W2"], cfg.k, inp["dy"], b, store="bf16")
    assert np.array_equal(O.bf16_round(g["dH"]), g["dH"]) and np.array_equal(O.bf16_round(g["dYp"]), g["dYp"])
    gs = O.layer_bwd_fp8_gemm(inp["x"], inp["logits"], inp["W1"], inp["W2"], cfg.k, inp["dy"], b)
    for name in ("dx", "dW1", "dW2"):
        assert np.linalg.norm(g[name] - gs[name]) / np.linalg.norm(gs[name]) < 5e-2, name
