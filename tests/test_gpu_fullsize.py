"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Routing, offsets and the permutation are compared in full, bit for bit.  Floating-point tensors
are compared on samples the oracle can compute one by one: every output row of 192 random tokens
(forward and backward are row-local given the routing), and for a few experts a 64-column slice of
the expert width, for which the oracle computes the exact weight-gradient slices from all of the
expert's rows (SwiGLU is elementwise in the expert width, so slicing it is exact).
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from synth.moe_inputs import CONFIGS, bf16_bits, make_inputs
from tests.gpu_util import DEV, max_norm_err, to_np

pytestmark = pytest.mark.gpu
TOL = 2e-2


def dev_bf16(a):
    return torch.from_numpy(bf16_bits(a).view(np.int16)).to(DEV).view(torch.bfloat16)


def run_full(cfg, inp):
    from paper_2505_11432_amd.layer import MoELayer
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, dtype=torch.bfloat16, renorm=cfg.renorm)
    x, dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
    w_r = dev_bf16(np.ascontiguousarray(inp["W_r"].T))
    bias = torch.from_numpy(inp["bias"]).to(DEV)
    w1, w2 = dev_bf16(inp["W1"]), dev_bf16(inp["W2"])
    layer.forward(x, w_r, bias, w1, w2)
    layer.backward(x, w_r, w1, w2, dy)
    torch.cuda.synchronize()
    return layer


@pytest.mark.parametrize("name", ["mixtral", "finegrained", "skewed"])
def test_full_size_sampled_parity(name):
    cfg = CONFIGS[name]
    inp = make_inputs(cfg, seed=0)
    layer = run_full(cfg, inp)
    T, k, d, f, E = cfg.T, cfg.k, cfg.d, cfg.f, cfg.E

    # ---- router matmul by tolerance, then routing bit-exact on the GPU's own fp32 logits -------
    z = layer.logits.cpu().numpy()
    assert max_norm_err(z, O.router_logits(inp["x"], inp["W_r"], inp["bias"])) < 1e-4
    r = O.route(z, k, cfg.renorm)
    for nm, got in (("idx", layer.topk_idx), ("counts", layer.counts), ("offsets", layer.offsets),
                    ("perm", layer.perm), ("inv_perm", layer.inv_perm)):
        assert np.array_equal(to_np(got), r[nm]), nm
    assert np.allclose(to_np(layer.topk_w), r["w"], rtol=2e-6, atol=1e-7)
    assert int(r["counts"].sum()) == T * k
    print(f"{name}: rows per expert min {r['counts'].min()} max {r['counts'].max()}")

    # ---- sampled tokens: every row-local tensor ------------------------------------------------
    rng = np.random.default_rng(7)
    toks = np.sort(rng.choice(T, size=192, replace=False))
    a_ids = (toks[:, None] * k + np.arange(k)[None, :]).reshape(-1)          # assignments of the sample
    rows = r["inv_perm"][a_ids].astype(np.int64)                             # their dispatched rows
    e_of = r["idx"].reshape(-1)[a_ids]
    order = np.argsort(e_of, kind="stable")
    rows_s, e_s, a_s = rows[order], e_of[order], a_ids[order]
    offs = np.concatenate([[0], np.cumsum(np.bincount(e_s, minlength=E))]).astype(np.int32)
    xp_s = inp["x"][a_s // k].astype(np.float64)
    H, A, Y = O.expert_ffn_fwd(xp_s, offs, inp["W1"], inp["W2"])
    w_s = r["w"].reshape(-1)[a_s]
    dY_s = inp["dy"][a_s // k].astype(np.float64) * w_s[:, None]
    dxp_s, _, _, dH_s = O.expert_ffn_bwd(xp_s, H, dY_s, offs, inp["W1"], inp["W2"])
    rows_t = torch.from_numpy(rows_s).to(DEV)
    errs = {
        "xp": max_norm_err(to_np(layer.xp[rows_t]), xp_s),
        "H": max_norm_err(to_np(layer.h_save[rows_t]), H),
        "Y": max_norm_err(to_np(layer.yp[rows_t]), Y),
        "dYp": max_norm_err(to_np(layer.d_yp[rows_t]), dY_s),
        "dxp": max_norm_err(to_np(layer.d_xp[rows_t]), dxp_s),
    }
    # token-level results need the sample's rows back in (token, slot) order
    back = np.empty_like(order)
    back[order] = np.arange(order.size)
    Y_ts = Y[back].reshape(len(toks), k, d)
    dxp_ts = dxp_s[back].reshape(len(toks), k, d)
    w_ts = r["w"][toks]
    y_ref = (Y_ts * w_ts[:, :, None]).sum(axis=1)
    dw_ref = np.einsum("td,tkd->tk", inp["dy"][toks].astype(np.float64), Y_ts)
    dz_ref = O.route_bwd(z[toks], r["idx"][toks], w_ts, dw_ref, cfg.renorm)
    dx_ref = dxp_ts.sum(axis=1) + dz_ref @ inp["W_r"].astype(np.float64).T
    tt = torch.from_numpy(toks).to(DEV)
    errs["y"] = max_norm_err(to_np(layer.y[tt]), y_ref)
    errs["dw"] = max_norm_err(to_np(layer.d_topk_w[tt]), dw_ref)
    errs["dz"] = max_norm_err(to_np(layer.d_logits[tt]), dz_ref)
    errs["dx"] = max_norm_err(to_np(layer.dx[tt]), dx_ref)

    # ---- weight-gradient slices for a few experts ------------------------------------------------
    nonempty = np.flatnonzero(r["counts"] > 0)
    pick = {int(nonempty[np.argmax(r["counts"][nonempty])]), int(nonempty[np.argmin(r["counts"][nonempty])]),
            int(rng.choice(nonempty))}
    for e in sorted(pick):
        lo, hi = int(r["offsets"][e]), int(r["offsets"][e + 1])
        j0 = int(rng.integers(0, f // 64)) * 64
        sl = np.r_[j0:j0 + 64, f + j0:f + j0 + 64]
        W1s = inp["W1"][e:e + 1, sl, :]
        W2s = inp["W2"][e:e + 1, :, j0:j0 + 64]
        a_e = r["perm"][lo:hi].astype(np.int64)
        xp_e = inp["x"][a_e // k].astype(np.float64)
        dY_e = inp["dy"][a_e // k].astype(np.float64) * r["w"].reshape(-1)[a_e][:, None]
        off_e = np.array([0, hi - lo], dtype=np.int32)
        H_e, _, _ = O.expert_ffn_fwd(xp_e, off_e, W1s, W2s)
        _, dW1s, dW2s, _ = O.expert_ffn_bwd(xp_e, H_e, dY_e, off_e, W1s, W2s)
        got1 = to_np(layer.d_w1[e][torch.from_numpy(sl).to(DEV)])
        got2 = to_np(layer.d_w2[e][:, j0:j0 + 64])
        errs[f"dW1[{e}] ({hi - lo} rows)"] = max_norm_err(got1, dW1s[0])
        errs[f"dW2[{e}] ({hi - lo} rows)"] = max_norm_err(got2, dW2s[0])
    for e in range(E):
        if r["counts"][e] == 0:
            assert torch.count_nonzero(layer.d_w1[e]) == 0 and torch.count_nonzero(layer.d_w2[e]) == 0

    # router weight gradient in full (cheap)
    dz_full = to_np(layer.d_logits)
    errs["dW_r"] = max_norm_err(to_np(layer.d_w_r), (inp["x"].astype(np.float64).T @ dz_full).T)
    print(name, {k_: f"{v:.2e}" for k_, v in errs.items()})
    bad = {k_: v for k_, v in errs.items() if not v < TOL}
    assert not bad, bad


def test_full_size_is_deterministic():
    cfg = CONFIGS["finegrained"]
    inp = make_inputs(cfg, seed=0)
    a = run_full(cfg, inp)
    ya, dxa, g1a, g2a = a.y.clone(), a.dx.clone(), a.d_w1.clone(), a.d_w2.clone()
    del a
    b = run_full(cfg, inp)
    assert torch.equal(ya, b.y) and torch.equal(dxa, b.dx)
    assert torch.equal(g1a, b.d_w1) and torch.equal(g2a, b.d_w2)


def test_full_size_back_to_back_steps_reproduce():
    """Steps enqueued without a host synchronisation between them (the benchmark's launch pattern: the stores of one
    tile's epilogue, and of one kernel's last tiles, are still in flight when the next loads are issued) give the first
    step's results bit for bit."""
    from paper_2505_11432_amd.layer import MoELayer
    cfg = CONFIGS["mixtral"]
    inp = make_inputs(cfg, seed=0)
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, dtype=torch.bfloat16, renorm=cfg.renorm)
    x, dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
    w_r = dev_bf16(np.ascontiguousarray(inp["W_r"].T))
    bias = torch.from_numpy(inp["bias"]).to(DEV)
    w1, w2 = dev_bf16(inp["W1"]), dev_bf16(inp["W2"])

    def step():
        layer.forward(x, w_r, bias, w1, w2)
        layer.backward(x, w_r, w1, w2, dy)

    step()
    torch.cuda.synchronize()
    names = ("y", "dx", "d_xp", "h_save", "d_w1", "d_w2", "d_w_r", "d_logits")
    first = {n: getattr(layer, n).clone() for n in names}
    for _ in range(4):
        step()
    torch.cuda.synchronize()
    for n in names:
        assert torch.equal(first[n], getattr(layer, n)), n


def test_full_size_fp8_forward_and_fp8_backward_sampled():
    """mixtral_fp8 with all six expert GEMMs on e4m3 operands, at full size.  Stage by stage on samples: casts bit for
    bit against the oracle's quantisers applied to the kernel's own pre-cast rows / column slices, GEMM outputs against
    the oracle's arithmetic on the kernel's codes (sampled rows x sampled columns; weight gradients on slices, summed
    over all rows of the expert)."""
    from paper_2505_11432_amd.layer import MoELayer
    cfg = CONFIGS["mixtral_fp8"]
    inp = make_inputs(cfg, seed=0)
    T, k, d, f, E = cfg.T, cfg.k, cfg.d, cfg.f, cfg.E
    layer = MoELayer(T, d, E, k, f, dtype=torch.bfloat16, renorm=cfg.renorm, fp8=True)
    x, dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
    w_r = dev_bf16(np.ascontiguousarray(inp["W_r"].T))
    w1, w2 = dev_bf16(inp["W1"]), dev_bf16(inp["W2"])
    layer.set_fp8_weights(w1, w2)
    layer.set_fp8_backward_weights(w1, w2)
    layer.forward_fp8(x, w_r, None)
    layer.backward_fp8_gemm(x, w_r, dy)
    torch.cuda.synchronize()
    tol = 6e-2
    offsets = to_np(layer.offsets).astype(np.int64)
    rng = np.random.default_rng(11)
    rows = np.sort(rng.choice(layer.M, size=96, replace=False))
    row_e = np.searchsorted(offsets, rows, side="right") - 1
    cf = np.sort(rng.choice(f, size=48, replace=False))          # columns of the expert width
    cd = np.sort(rng.choice(d, size=48, replace=False))          # columns of the model width
    I = layer.bwd8
    g = lambda t, r=None, c=None: to_np(t if r is None else t[torch.as_tensor(r, device=DEV)] if c is None
                                        else t[torch.as_tensor(r, device=DEV)][:, torch.as_tensor(c, device=DEV)])
    errs = {}

    def wslice(codes, scales, e, rsel):      # dequantised rows rsel of expert e of a [E, R, C] code tensor
        c = g(codes[e], rsel)
        s = g(scales[e], rsel).astype(np.float32)
        return O.dequant_rows(c, s)

    # weight casts (both orientations) on sampled rows: bit-exact
    for e in (0, E - 1):
        for codes, scales, W in ((layer.w1_codes, layer.w1_scale, inp["W1"][e]), (layer.w2_codes, layer.w2_scale, inp["W2"][e]),
                                 (layer.w1t_codes, layer.w1t_scale, inp["W1"][e].T), (layer.w2t_codes, layer.w2t_scale, inp["W2"][e].T)):
            rs = np.sort(rng.choice(W.shape[0], size=8, replace=False))
            c_ref, s_ref = O.quant_rows(np.ascontiguousarray(W[rs]))
            assert np.array_equal(g(codes[e], rs), c_ref) and np.array_equal(g(scales[e], rs).astype(np.float32), s_ref)
    # forward: FC1 on the kernel's xp codes, FC2 on the kernel's A codes
    xp_hat = O.dequant_rows(g(layer.xp, rows), g(layer.xp_scale, rows).astype(np.float32))
    a_hat = O.dequant_rows(g(layer.a_codes, rows), g(layer.a_scale, rows).astype(np.float32))
    H_s = np.zeros((len(rows), 2 * len(cf)))
    Y_s = np.zeros((len(rows), len(cd)))
    hcols = np.concatenate([cf, f + cf])
    for e in np.unique(row_e):
        m = row_e == e
        H_s[m] = xp_hat[m] @ wslice(layer.w1_codes, layer.w1_scale, e, hcols).T
        Y_s[m] = a_hat[m] @ wslice(layer.w2_codes, layer.w2_scale, e, cd).T
    H_gpu = g(layer.h_save, rows, hcols)
    errs["H"] = max_norm_err(H_gpu, H_s)
    cy, sy = g(layer.yp, rows), g(layer.yp_scale, rows).astype(np.float32)
    errs["Y"] = max_norm_err(O.dequant_rows(cy, sy)[:, cd], Y_s)          # includes the per-token cast of Y (<= 2^-4 relative)
    # backward, per-token operands
    dyp = g(layer.d_yp, rows).astype(np.float32)
    c_ref, s_ref = O.quant_rows(dyp)
    assert np.array_equal(g(I["dy_codes"], rows), c_ref) and np.array_equal(g(I["dy_scale"], rows).astype(np.float32), s_ref)
    dY_hat = O.dequant_rows(c_ref, s_ref)
    dA = np.zeros((len(rows), len(cf)))
    for e in np.unique(row_e):
        m = row_e == e
        dA[m] = dY_hat[m] @ wslice(layer.w2t_codes, layer.w2t_scale, e, cf).T
    dG, dU = O.swiglu_bwd(H_gpu[:, :len(cf)], H_gpu[:, len(cf):], dA)
    errs["dH"] = max_norm_err(g(I["dh"], rows, hcols), np.concatenate([dG, dU], axis=1))
    dh_rows = g(I["dh"], rows).astype(np.float32)
    c_ref, s_ref = O.quant_rows(dh_rows)
    assert np.array_equal(g(I["dh_codes"], rows), c_ref) and np.array_equal(g(I["dh_scale"], rows).astype(np.float32), s_ref)
    dH_hat = O.dequant_rows(c_ref, s_ref)
    dxp = np.zeros((len(rows), len(cd)))
    for e in np.unique(row_e):
        m = row_e == e
        dxp[m] = dH_hat[m] @ wslice(layer.w1t_codes, layer.w1t_scale, e, cd).T
    errs["dxp"] = max_norm_err(g(layer.d_xp, rows, cd), dxp)
    # token-group casts on column slices (columns are independent), then the weight gradients of those slices
    po = to_np(I["pad_offsets"]).astype(np.int64)
    assert np.array_equal(po, np.concatenate([[0], np.cumsum((np.diff(offsets) + 127) // 128 * 128)]))
    allr = np.arange(layer.M)

    def tg_slice(src_t, name, cols, row_scale=None):
        src = g(src_t, allr, cols)
        if row_scale is not None:          # e4m3 codes with per-row scales: code * scale, rounded once to fp32
            src = O.e4m3_decode(src).astype(np.float32) * to_np(row_scale).astype(np.float32)[:, None]
        src = src.astype(np.float32)
        c_ref, k_ref = O.quant_tokengroup_pow2(src, offsets)
        ct = g(I[name + "_t"], cols)                                   # [len(cols), ldt]
        e8 = to_np(I[name + "_e8m0"][:, torch.as_tensor(cols, device=DEV)]).astype(np.int64)
        gi = 0
        for e in range(E):
            n = offsets[e + 1] - offsets[e]
            assert np.array_equal(ct[:, po[e]:po[e] + n].T, c_ref[offsets[e]:offsets[e + 1]]), (name, e)
            assert not ct[:, po[e] + n:po[e + 1]].any()
            ng = (n + 127) // 128
            assert np.array_equal(e8[po[e] // 128:po[e] // 128 + ng] - 127, k_ref[gi:gi + ng]), (name, e)
            gi += ng
        return O.dequant_tokengroup_pow2(c_ref, k_ref, offsets)

    dy_g = tg_slice(layer.d_yp, "dy", cd)
    a_g = tg_slice(layer.a_codes, "a", cf, layer.a_scale)
    dh_g = tg_slice(I["dh"], "dh", hcols)
    x_g = tg_slice(layer.xp, "x", cd, layer.xp_scale)
    for e in (0, 3, E - 1):
        lo, hi = offsets[e], offsets[e + 1]
        errs[f"dW2[{e}]"] = max_norm_err(g(layer.d_w2[e], cd, cf), dy_g[lo:hi].T @ a_g[lo:hi])
        errs[f"dW1[{e}]"] = max_norm_err(g(layer.d_w1[e], hcols, cd), dh_g[lo:hi].T @ x_g[lo:hi])
    print("mixtral_fp8 full size:", {k_: f"{v:.2e}" for k_, v in errs.items()})
    bad = {k_: v for k_, v in errs.items() if not v < tol}
    assert not bad, bad


def test_full_size_expert_parallel_share():
    """ep352b_share (4 of 32 experts local, all-gathered tokens) at full size: routing bit-exact, sampled tokens'
    local rows, partial outputs and partial input gradients, and weight-gradient slices of two local experts."""
    cfg = CONFIGS["ep352b_share"]
    inp = make_inputs(cfg, seed=0)
    from paper_2505_11432_amd.layer import MoELayer
    lo_e, hi_e = cfg.expert_range
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, dtype=torch.bfloat16, renorm=cfg.renorm, expert_range=cfg.expert_range)
    x, dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
    w_r = dev_bf16(np.ascontiguousarray(inp["W_r"].T))
    w1, w2 = dev_bf16(inp["W1"]), dev_bf16(inp["W2"])
    layer.forward(x, w_r, None, w1, w2)
    layer.backward(x, w_r, w1, w2, dy, with_router=False)
    torch.cuda.synchronize()
    T, k, d, f = cfg.T, cfg.k, cfg.d, cfg.f
    z = layer.logits.cpu().numpy()
    r = O.route_range(z, k, lo_e, hi_e, cfg.renorm)
    n = int(r["offsets"][-1])
    for nm, got in (("idx", layer.topk_idx), ("counts", layer.counts), ("offsets", layer.offsets), ("inv_perm", layer.inv_perm)):
        assert np.array_equal(to_np(got), r[nm]), nm
    assert np.array_equal(to_np(layer.perm)[:n], r["perm"])
    print(f"ep352b_share: {n} of {T * k} rows local, per local expert {np.diff(r['offsets']).tolist()}")
    rng = np.random.default_rng(9)
    toks = np.sort(rng.choice(T, size=256, replace=False))
    a_ids = (toks[:, None] * k + np.arange(k)[None, :]).reshape(-1)
    rows_all = r["inv_perm"][a_ids].astype(np.int64)
    keep = rows_all >= 0
    a_l, rows_l = a_ids[keep], rows_all[keep]
    e_l = r["idx"].reshape(-1)[a_l] - lo_e
    order = np.argsort(e_l, kind="stable")
    a_s, rows_s, e_s = a_l[order], rows_l[order], e_l[order]
    offs = np.concatenate([[0], np.cumsum(np.bincount(e_s, minlength=hi_e - lo_e))]).astype(np.int32)
    xp_s = inp["x"][a_s // k].astype(np.float64)
    H, A, Y = O.expert_ffn_fwd(xp_s, offs, inp["W1"], inp["W2"])
    w_s = r["w"].reshape(-1)[a_s]
    dY_s = inp["dy"][a_s // k].astype(np.float64) * w_s[:, None]
    dxp_s, _, _, _ = O.expert_ffn_bwd(xp_s, H, dY_s, offs, inp["W1"], inp["W2"])
    rows_t = torch.from_numpy(rows_s).to(DEV)
    errs = {"xp": max_norm_err(to_np(layer.xp[rows_t]), xp_s), "H": max_norm_err(to_np(layer.h_save[rows_t]), H),
            "Y": max_norm_err(to_np(layer.yp[rows_t]), Y), "dxp": max_norm_err(to_np(layer.d_xp[rows_t]), dxp_s)}
    y_ref = np.zeros((T, d)); dx_ref = np.zeros((T, d)); dw_ref = np.zeros((T, k))
    np.add.at(y_ref, a_s // k, Y * w_s[:, None])
    np.add.at(dx_ref, a_s // k, dxp_s)
    dw_ref[a_s // k, a_s % k] = np.einsum("rd,rd->r", inp["dy"][a_s // k].astype(np.float64), Y)
    tt = torch.from_numpy(toks).to(DEV)
    errs["y (partial)"] = max_norm_err(to_np(layer.y[tt]), y_ref[toks])
    errs["dx (partial)"] = max_norm_err(to_np(layer.dx[tt]), dx_ref[toks])
    errs["dw"] = max_norm_err(to_np(layer.d_topk_w[tt]), dw_ref[toks])
    assert np.all(to_np(layer.d_topk_w[tt])[rows_all.reshape(-1, k) < 0] == 0)
    for e in (0, hi_e - lo_e - 1):
        lo, hi = int(r["offsets"][e]), int(r["offsets"][e + 1])
        j0 = int(rng.integers(0, f // 64)) * 64
        sl = np.r_[j0:j0 + 64, f + j0:f + j0 + 64]
        W1s, W2s = inp["W1"][e:e + 1, sl, :], inp["W2"][e:e + 1, :, j0:j0 + 64]
        a_e = r["perm"][lo:hi].astype(np.int64)
        xp_e = inp["x"][a_e // k].astype(np.float64)
        dY_e = inp["dy"][a_e // k].astype(np.float64) * r["w"].reshape(-1)[a_e][:, None]
        off_e = np.array([0, hi - lo], dtype=np.int32)
        H_e, _, _ = O.expert_ffn_fwd(xp_e, off_e, W1s, W2s)
        _, dW1s, dW2s, _ = O.expert_ffn_bwd(xp_e, H_e, dY_e, off_e, W1s, W2s)
        errs[f"dW1[{lo_e + e}]"] = max_norm_err(to_np(layer.d_w1[e][torch.from_numpy(sl).to(DEV)]), dW1s[0])
        errs[f"dW2[{lo_e + e}]"] = max_norm_err(to_np(layer.d_w2[e][:, j0:j0 + 64]), dW2s[0])
    print("ep352b_share", {k_: f"{v:.2e}" for k_, v in errs.items()})
    bad = {k_: v for k_, v in errs.items() if not v < TOL}
    assert not bad, bad


@pytest.mark.parametrize("name", ["mixtral", "skewed"])
def test_full_size_fused_order_sampled(name):
    """The Section 4.1 / 4.2 operator order at the benchmark sizes (bench.py --fused): routing and the row map in
    full and bit-exact, every row-local tensor of 192 sampled tokens and weight-gradient slices against the oracle."""
    from paper_2505_11432_amd.layer import MoELayer
    cfg = CONFIGS[name]
    inp = make_inputs(cfg, seed=0)
    T, k, d, f, E = cfg.T, cfg.k, cfg.d, cfg.f, cfg.E
    layer = MoELayer(T, d, E, k, f, dtype=torch.bfloat16, renorm=cfg.renorm, fused=True)
    x, dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
    w_r = dev_bf16(np.ascontiguousarray(inp["W_r"].T))
    bias = torch.from_numpy(inp["bias"]).to(DEV)
    w1, w2 = dev_bf16(inp["W1"]), dev_bf16(inp["W2"])
    layer.forward(x, w_r, bias, w1, w2)
    layer.backward(x, w_r, w1, w2, dy)
    torch.cuda.synchronize()
    z = layer.logits.cpu().numpy()
    r = O.route(z, k, cfg.renorm)
    for nm, got in (("idx", layer.topk_idx), ("offsets", layer.offsets), ("perm", layer.perm), ("inv_perm", layer.inv_perm)):
        assert np.array_equal(to_np(got), r[nm]), nm
    assert np.array_equal(to_np(layer.row_token), O.row_tokens(r["perm"], k))
    assert np.array_equal(to_np(layer.row_w), to_np(layer.topk_w).reshape(-1)[r["perm"]])

    rng = np.random.default_rng(11)
    toks = np.sort(rng.choice(T, size=192, replace=False))
    a_ids = (toks[:, None] * k + np.arange(k)[None, :]).reshape(-1)
    rows = r["inv_perm"][a_ids].astype(np.int64)
    e_of = r["idx"].reshape(-1)[a_ids]
    order = np.argsort(e_of, kind="stable")
    rows_s, e_s, a_s = rows[order], e_of[order], a_ids[order]
    offs = np.concatenate([[0], np.cumsum(np.bincount(e_s, minlength=E))]).astype(np.int32)
    tok_s, w_s = a_s // k, r["w"].reshape(-1)[a_s]
    H, Aw, Yw = O.expert_ffn_fwd_folded(inp["x"], tok_s, w_s, offs, inp["W1"], inp["W2"])
    dxp_s, _, _, _, drw_s, dxp0_s = O.expert_ffn_bwd_folded(inp["x"], inp["dy"], tok_s, w_s, H, offs, inp["W1"], inp["W2"])
    rows_t = torch.from_numpy(rows_s).to(DEV)
    errs = {"H": max_norm_err(to_np(layer.h_save[rows_t]), H), "Yw": max_norm_err(to_np(layer.yp[rows_t]), Yw),
            "dxp0": max_norm_err(to_np(layer.d_xp[rows_t]), dxp0_s)}
    back = np.empty_like(order)
    back[order] = np.arange(order.size)
    y_ref = Yw[back].reshape(len(toks), k, d).sum(axis=1)
    dw_ref = drw_s[back].reshape(len(toks), k)
    dz_ref = O.route_bwd(z[toks], r["idx"][toks], r["w"][toks], dw_ref, cfg.renorm)
    dx_ref = dxp_s[back].reshape(len(toks), k, d).sum(axis=1) + dz_ref @ inp["W_r"].astype(np.float64).T
    tt = torch.from_numpy(toks).to(DEV)
    errs["y"] = max_norm_err(to_np(layer.y[tt]), y_ref)
    errs["dw"] = max_norm_err(to_np(layer.d_topk_w[tt]), dw_ref)
    errs["dx"] = max_norm_err(to_np(layer.dx[tt]), dx_ref)

    nonempty = np.flatnonzero(r["counts"] > 0)
    pick = {int(nonempty[np.argmax(r["counts"][nonempty])]), int(nonempty[np.argmin(r["counts"][nonempty])])}
    for e in sorted(pick):
        lo, hi = int(r["offsets"][e]), int(r["offsets"][e + 1])
        j0 = int(rng.integers(0, f // 64)) * 64
        sl = np.r_[j0:j0 + 64, f + j0:f + j0 + 64]
        W1s, W2s = inp["W1"][e:e + 1, sl, :], inp["W2"][e:e + 1, :, j0:j0 + 64]
        a_e = r["perm"][lo:hi].astype(np.int64)
        off_e = np.array([0, hi - lo], dtype=np.int32)
        H_e, _, _ = O.expert_ffn_fwd_folded(inp["x"], a_e // k, r["w"].reshape(-1)[a_e], off_e, W1s, W2s)
        _, dW1s, dW2s, _, _, _ = O.expert_ffn_bwd_folded(inp["x"], inp["dy"], a_e // k, r["w"].reshape(-1)[a_e], H_e, off_e, W1s, W2s)
        errs[f"dW1[{e}] ({hi - lo} rows)"] = max_norm_err(to_np(layer.d_w1[e][torch.from_numpy(sl).to(DEV)]), dW1s[0])
        errs[f"dW2[{e}] ({hi - lo} rows)"] = max_norm_err(to_np(layer.d_w2[e][:, j0:j0 + 64]), dW2s[0])
    print(name, "fused", {k_: f"{v:.2e}" for k_, v in errs.items()})
    bad = {k_: v for k_, v in errs.items() if not v < TOL}
    assert not bad, bad


def test_full_size_one_whole_expert_every_output_tile():
    """Mixtral workload at full size: for the largest expert, every element of every output of the six grouped GEMMs
    (H, Y, d_xp for all of its rows; the full dW1[e] and dW2[e]) against the oracle, so that every output tile of one
    expert is covered, the ragged last m-tile and the tiles of workgroups that run several tiles included."""
    cfg = CONFIGS["mixtral"]
    inp = make_inputs(cfg, seed=0)
    layer = run_full(cfg, inp)
    k, E = cfg.k, cfg.E
    z = layer.logits.cpu().numpy()
    r = O.route(z, k, cfg.renorm)
    assert np.array_equal(to_np(layer.perm), r["perm"]) and np.array_equal(to_np(layer.offsets), r["offsets"])
    e = int(np.argmax(r["counts"]))
    lo, hi = int(r["offsets"][e]), int(r["offsets"][e + 1])
    print(f"whole expert {e}: rows {lo}..{hi} ({hi - lo} rows, {(hi - lo + 255) // 256} m-tiles)", flush=True)
    a_e = r["perm"][lo:hi].astype(np.int64)
    xp_e = inp["x"][a_e // k].astype(np.float64)
    dY_e = inp["dy"][a_e // k].astype(np.float64) * r["w"].reshape(-1)[a_e][:, None]
    off_e = np.array([0, hi - lo], dtype=np.int32)
    W1e, W2e = inp["W1"][e:e + 1], inp["W2"][e:e + 1]
    H, _, Y = O.expert_ffn_fwd(xp_e, off_e, W1e, W2e)
    dxp, dW1, dW2, _ = O.expert_ffn_bwd(xp_e, H, dY_e, off_e, W1e, W2e)
    errs = {"H": max_norm_err(to_np(layer.h_save[lo:hi]), H), "Y": max_norm_err(to_np(layer.yp[lo:hi]), Y),
            "dxp": max_norm_err(to_np(layer.d_xp[lo:hi]), dxp)}
    del H, Y, dxp
    errs["dW1"] = max_norm_err(to_np(layer.d_w1[e]), dW1[0])
    errs["dW2"] = max_norm_err(to_np(layer.d_w2[e]), dW2[0])
    print("whole expert:", {k_: f"{v:.2e}" for k_, v in errs.items()})
    bad = {k_: v for k_, v in errs.items() if not v < TOL}
    assert not bad, bad


def _fp8_layer_full(backward):
    from paper_2505_11432_amd.layer import MoELayer
    cfg = CONFIGS["mixtral_fp8"]
    inp = make_inputs(cfg, seed=0)
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, dtype=torch.bfloat16, renorm=cfg.renorm, fp8=True)
    x, dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
    w_r = dev_bf16(np.ascontiguousarray(inp["W_r"].T))
    w1, w2 = dev_bf16(inp["W1"]), dev_bf16(inp["W2"])
    layer.set_fp8_weights(w1, w2)
    layer.forward_fp8(x, w_r, None)
    if backward == "fp8":
        layer.set_fp8_backward_weights(w1, w2)
        layer.backward_fp8_gemm(x, w_r, dy)
    else:
        layer.backward_fp8(x, w_r, w1, w2, dy)
    torch.cuda.synchronize()
    return cfg, inp, layer


def test_full_size_fp8_whole_expert_weight_gradients_on_the_kernels_codes():
    """All-e4m3 step at full size: the full dW1[e] and dW2[e] of the largest expert from the kernel's own transposed
    codes and E8M0 group scales (which the sampled test compares bit for bit with the oracle's quantiser), so every
    output tile of the block-scaled weight-gradient GEMMs of one expert is covered."""
    cfg, inp, layer = _fp8_layer_full("fp8")
    I = layer.bwd8
    offsets = to_np(layer.offsets).astype(np.int64)
    po = to_np(I["pad_offsets"]).astype(np.int64)
    e = int(np.argmax(np.diff(offsets)))
    n = int(offsets[e + 1] - offsets[e])
    off_e = np.array([0, n])
    print(f"whole expert {e}: {n} rows, {(n + 127) // 128} token groups", flush=True)

    def deq(name):
        codes = to_np(I[name + "_t"][:, po[e]:po[e] + n]).T                       # [n, channels]
        ng = (n + 127) // 128
        exps = to_np(I[name + "_e8m0"][po[e] // 128: po[e] // 128 + ng]).astype(np.int64) - 127
        return O.dequant_tokengroup_pow2(np.ascontiguousarray(codes), exps, off_e)

    dy_g, a_g = deq("dy"), deq("a")
    err2 = max_norm_err(to_np(layer.d_w2[e]), dy_g.T @ a_g)
    del dy_g, a_g
    dh_g, x_g = deq("dh"), deq("x")
    err1 = max_norm_err(to_np(layer.d_w1[e]), dh_g.T @ x_g)
    print(f"whole expert e4m3 weight gradients: dW1 {err1:.2e} dW2 {err2:.2e}")
    assert err1 < 6e-2 and err2 < 6e-2


def test_full_size_fp8_forward_with_straight_through_bf16_backward_sampled():
    """mixtral_fp8 in its required form (e4m3 forward, straight-through bf16 backward on the master weights) at full
    size: sampled tokens against the oracle fed the kernel's codes (stage-wise, as in the small cases), and the
    weight-gradient slices of three experts summed over all of their rows."""
    cfg, inp, layer = _fp8_layer_full("bf16")
    T, k, d, f, E = cfg.T, cfg.k, cfg.d, cfg.f, cfg.E
    z = layer.logits.cpu().numpy()
    r = O.route(z, k, cfg.renorm)
    assert np.array_equal(to_np(layer.perm), r["perm"])
    offsets = r["offsets"].astype(np.int64)
    rng = np.random.default_rng(21)
    # dy cast (per channel in 128-token groups, token order): bit-exact on whole groups
    g0 = int(rng.integers(0, T // 128)) * 128
    c_ref, s_ref = O.quant_colgroup128(inp["dy"][g0:g0 + 256])
    assert np.array_equal(to_np(layer.dy_codes[g0:g0 + 256]), c_ref)
    assert np.array_equal(to_np(layer.dy_scale[g0 // 128: g0 // 128 + 2]).astype(np.float32), s_ref)
    dy_hat = to_np(layer.dy_deq)                                                 # [T, d], checked against the codes below
    assert np.array_equal(dy_hat[g0:g0 + 256], O.dequant_colgroup128(c_ref, s_ref).astype(np.float32).astype(np.float64)) or \
        max_norm_err(dy_hat[g0:g0 + 256], O.dequant_colgroup128(c_ref, s_ref)) < 2 ** -8
    # sampled tokens: rows of the backward GEMMs from the kernel's codes (A_hat, xp_hat) and saved H
    toks = np.sort(rng.choice(T, size=96, replace=False))
    a_ids = (toks[:, None] * k + np.arange(k)[None, :]).reshape(-1)
    rows = r["inv_perm"][a_ids].astype(np.int64)
    e_of = r["idx"].reshape(-1)[a_ids]
    order = np.argsort(e_of, kind="stable")
    rows_s, e_s, a_s = rows[order], e_of[order], a_ids[order]
    offs = np.concatenate([[0], np.cumsum(np.bincount(e_s, minlength=E))]).astype(np.int32)
    rt = torch.from_numpy(rows_s).to(DEV)
    xp_hat = O.dequant_rows(to_np(layer.xp[rt]), to_np(layer.xp_scale[rt]).astype(np.float32))
    A_hat = O.dequant_rows(to_np(layer.a_codes[rt]), to_np(layer.a_scale[rt]).astype(np.float32))
    Y_hat = O.dequant_rows(to_np(layer.yp[rt]), to_np(layer.yp_scale[rt]).astype(np.float32))
    H = to_np(layer.h_save[rt])
    w_s = r["w"].reshape(-1)[a_s]
    dY_s = dy_hat[a_s // k] * w_s[:, None]
    dxp_s, _, _, _ = O.expert_ffn_bwd(xp_hat, H, dY_s, offs, inp["W1"], inp["W2"], A=A_hat)
    errs = {"dYp": max_norm_err(to_np(layer.d_yp[rt]), dY_s), "dxp": max_norm_err(to_np(layer.d_xp[rt]), dxp_s)}
    back = np.empty_like(order)
    back[order] = np.arange(order.size)
    dw_ref = np.einsum("td,tkd->tk", dy_hat[toks], Y_hat[back].reshape(len(toks), k, d))
    tt = torch.from_numpy(toks).to(DEV)
    errs["dw"] = max_norm_err(to_np(layer.d_topk_w[tt]), dw_ref)
    dz_ref = O.route_bwd(z[toks], r["idx"][toks], r["w"][toks], dw_ref, cfg.renorm)
    dx_ref = dxp_s[back].reshape(len(toks), k, d).sum(axis=1) + dz_ref @ inp["W_r"].astype(np.float64).T
    errs["dx"] = max_norm_err(to_np(layer.dx[tt]), dx_ref)
    # weight-gradient slices over all rows of three experts, from the kernel's codes
    for e in (0, int(np.argmax(r["counts"])), E - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        j0 = int(rng.integers(0, f // 64)) * 64
        sl = np.r_[j0:j0 + 64, f + j0:f + j0 + 64]
        slt = torch.from_numpy(sl).to(DEV)
        a_e = r["perm"][lo:hi].astype(np.int64)
        dY_e = dy_hat[a_e // k] * r["w"].reshape(-1)[a_e][:, None]
        xp_e = O.dequant_rows(to_np(layer.xp[lo:hi]), to_np(layer.xp_scale[lo:hi]).astype(np.float32))
        A_e = O.dequant_rows(to_np(layer.a_codes[lo:hi, j0:j0 + 64]), to_np(layer.a_scale[lo:hi]).astype(np.float32))
        H_e = to_np(layer.h_save[lo:hi][:, slt])
        off_e = np.array([0, hi - lo], dtype=np.int32)
        _, dW1s, dW2s, _ = O.expert_ffn_bwd(xp_e, H_e, dY_e, off_e, inp["W1"][e:e + 1, sl, :], inp["W2"][e:e + 1, :, j0:j0 + 64], A=A_e)
        errs[f"dW1[{e}]"] = max_norm_err(to_np(layer.d_w1[e][slt]), dW1s[0])
        errs[f"dW2[{e}]"] = max_norm_err(to_np(layer.d_w2[e][:, j0:j0 + 64]), dW2s[0])
    print("mixtral_fp8, bf16 backward, full size:", {k_: f"{v:.2e}" for k_, v in errs.items()})
    bad = {k_: v for k_, v in errs.items() if not v < 6e-2}
    assert not bad, bad
