"""Pins for the oracle's dispatch / expert-FFN / combine and their gradients: special cases that
reduce to plain matmuls, closed forms, adjoint identities, finite differences and an independent
torch-CPU float64 autograd statement of the same layer.  No GPU."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from synth.moe_inputs import CONFIGS, MoEConfig, make_inputs


def small_case(T=24, d=12, E=4, k=2, f=10, seed=0):
    cfg = MoEConfig("t", T=T, d=d, E=E, k=k, f=f, dtype="f32", w_std=0.3, wr_std=0.5)
    inp = make_inputs(cfg, seed=seed)
    z = O.router_logits(inp["x"], inp["W_r"]).astype(np.float32)
    return cfg, inp, z


def dense_swiglu(x, Wg, Wu, Wd):
    g = x @ Wg.T
    u = x @ Wu.T
    return (g / (1 + np.exp(-g)) * u) @ Wd.T


def test_dispatch_combine_identities():
    cfg, inp, z = small_case(T=40, k=4, E=6)
    r = O.route(z, cfg.k)
    x = inp["x"].astype(np.float64)
    xp = O.dispatch(x, r["perm"], cfg.k)
    # every dispatched row is a copy of its token's row
    for row in range(cfg.M):
        assert np.array_equal(xp[row], x[r["perm"][row] // cfg.k])
    # uniform weights 1/k (k a power of two) undo the dispatch exactly; unweighted gives k*x
    w = np.full((cfg.T, cfg.k), 1.0 / cfg.k)
    assert np.array_equal(O.combine(xp, r["inv_perm"], w, cfg.T, cfg.k), x)
    assert np.array_equal(O.combine(xp, r["inv_perm"], None, cfg.T, cfg.k), cfg.k * x)
    # adjointness of dispatch and unweighted combine
    rng = np.random.default_rng(0)
    Y = rng.standard_normal(xp.shape)
    assert np.isclose((xp * Y).sum(), (x * O.combine(Y, r["inv_perm"], None, cfg.T, cfg.k)).sum())
    # row_mul scales row r by the value of its assignment
    mul = rng.standard_normal(cfg.M)
    xs = O.dispatch(x, r["perm"], cfg.k, row_mul=mul.reshape(cfg.T, cfg.k))
    assert np.allclose(xs, xp * mul[r["perm"]][:, None])


def test_combine_brute_force():
    cfg, inp, z = small_case(T=9, k=3, E=5, d=4)
    r = O.route(z, cfg.k)
    rng = np.random.default_rng(1)
    Y = rng.standard_normal((cfg.M, cfg.d))
    y = O.combine(Y, r["inv_perm"], r["w"], cfg.T, cfg.k)
    dy = rng.standard_normal((cfg.T, cfg.d))
    dw = O.gate_grad(dy, Y, r["inv_perm"], cfg.T, cfg.k)
    for t in range(cfg.T):
        acc = np.zeros(cfg.d)
        for j in range(cfg.k):
            row = r["inv_perm"][t * cfg.k + j]
            acc += r["w"][t, j] * Y[row]
            assert np.isclose(dw[t, j], sum(dy[t, c] * Y[row, c] for c in range(cfg.d)))
        assert np.allclose(y[t], acc, rtol=1e-14)


def test_single_expert_is_dense_ffn():
    cfg, inp, _ = small_case(T=16, E=1, k=1)
    z = np.zeros((cfg.T, 1), dtype=np.float32)
    out = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], 1)
    ref = dense_swiglu(inp["x"].astype(np.float64), inp["W1"][0, :cfg.f].astype(np.float64),
                       inp["W1"][0, cfg.f:].astype(np.float64), inp["W2"][0].astype(np.float64))
    assert np.allclose(out["y"], ref, rtol=1e-12, atol=1e-14)
    assert np.allclose(out["w"], 1.0)


def test_shared_weights_equal_dense_ffn_for_any_routing():
    cfg, inp, z = small_case(T=32, E=5, k=3)
    W1 = np.repeat(inp["W1"][:1], cfg.E, axis=0)
    W2 = np.repeat(inp["W2"][:1], cfg.E, axis=0)
    out = O.layer_fwd(inp["x"], z, W1, W2, cfg.k)
    ref = dense_swiglu(inp["x"].astype(np.float64), W1[0, :cfg.f].astype(np.float64),
                       W1[0, cfg.f:].astype(np.float64), W2[0].astype(np.float64))
    assert np.allclose(out["y"], ref, rtol=1e-11, atol=1e-13)
    # and the expert weight gradients add up to the dense layer's gradient
    dy = inp["dy"].astype(np.float64)
    g = O.layer_bwd(inp["x"], z, W1, W2, cfg.k, dy, out)
    xt = torch.tensor(inp["x"], dtype=torch.float64)
    w1t = torch.tensor(W1[0], dtype=torch.float64, requires_grad=True)
    w2t = torch.tensor(W2[0], dtype=torch.float64, requires_grad=True)
    gg = xt @ w1t[:cfg.f].T
    yy = (torch.nn.functional.silu(gg) * (xt @ w1t[cfg.f:].T)) @ w2t.T
    (yy * torch.tensor(dy)).sum().backward()
    assert np.allclose(g["dW1"].sum(axis=0), w1t.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["dW2"].sum(axis=0), w2t.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_zero_down_projection_and_one_hot_rows():
    cfg, inp, z = small_case()
    out = O.layer_fwd(inp["x"], z, inp["W1"], np.zeros_like(inp["W2"]), cfg.k)
    assert np.all(out["y"] == 0.0)
    # one-hot x rows: G and U are single columns of the weights, so y is closed form
    T = cfg.d
    x = np.eye(T, cfg.d, dtype=np.float32) * 2.0
    z = O.router_logits(x, inp["W_r"]).astype(np.float32)
    out = O.layer_fwd(x, z, inp["W1"], inp["W2"], cfg.k)
    W1 = inp["W1"].astype(np.float64)
    W2 = inp["W2"].astype(np.float64)
    for t in range(T):
        acc = np.zeros(cfg.d)
        for j in range(cfg.k):
            e = out["idx"][t, j]
            g = 2.0 * W1[e, :cfg.f, t]
            u = 2.0 * W1[e, cfg.f:, t]
            acc += out["w"][t, j] * (W2[e] @ (g / (1 + np.exp(-g)) * u))
        assert np.allclose(out["y"][t], acc, rtol=1e-12, atol=1e-14)


def test_h_layout_gate_first_then_up():
    cfg, inp, z = small_case()
    out = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k)
    row = 3
    e = int(np.searchsorted(out["offsets"], row, side="right") - 1)
    xr = out["xp"][row]
    assert np.allclose(out["H"][row, :cfg.f], inp["W1"][e, :cfg.f].astype(np.float64) @ xr)
    assert np.allclose(out["H"][row, cfg.f:], inp["W1"][e, cfg.f:].astype(np.float64) @ xr)
    assert np.allclose(out["A"][row], O.silu(out["H"][row, :cfg.f]) * out["H"][row, cfg.f:])


@pytest.mark.parametrize("renorm", [1, 0])
def test_backward_finite_differences(renorm):
    cfg, inp, z = small_case(T=12, d=8, E=4, k=2, f=6, seed=3)
    x = inp["x"].astype(np.float64)
    W1 = inp["W1"].astype(np.float64)
    W2 = inp["W2"].astype(np.float64)
    dy = inp["dy"].astype(np.float64)
    fwd = O.layer_fwd(x, z, W1, W2, cfg.k, renorm)
    g = O.layer_bwd(x, z, W1, W2, cfg.k, dy, fwd, renorm)
    rng = np.random.default_rng(5)
    eps = 1e-6

    def frozen_loss(xv, zv, w1, w2):
        # same selection as fwd (no re-routing), weights recomputed from zv
        w = O.gate_weights(zv, fwd["idx"], renorm)
        xp = O.dispatch(xv, fwd["perm"], cfg.k)
        _, _, Y = O.expert_ffn_fwd(xp, fwd["offsets"], w1, w2)
        return float((O.combine(Y, fwd["inv_perm"], w, cfg.T, cfg.k) * dy).sum())

    z64 = z.astype(np.float64)
    for name, base, grad in (("x", x, g["dx"]), ("W1", W1, g["dW1"]), ("W2", W2, g["dW2"]), ("z", z64, g["dz"])):
        for _ in range(3):
            v = rng.standard_normal(base.shape)
            args_p = dict(xv=x, zv=z64, w1=W1, w2=W2)
            args_m = dict(args_p)
            key = {"x": "xv", "W1": "w1", "W2": "w2", "z": "zv"}[name]
            args_p[key] = base + eps * v
            args_m[key] = base - eps * v
            num = (frozen_loss(**args_p) - frozen_loss(**args_m)) / (2 * eps)
            ana = float((grad * v).sum())
            assert np.isclose(num, ana, rtol=2e-6, atol=1e-8), (name, num, ana)


def torch_layer(x, z, W1, W2, idx, k, renorm):
    """The same layer stated with torch ops and no permutation at all (loop over tokens' slots)."""
    T = x.shape[0]
    f = W1.shape[1] // 2
    sel = torch.gather(z, 1, idx)
    if renorm:
        w = torch.softmax(sel, dim=1)
    else:
        w = torch.gather(torch.softmax(z, dim=1), 1, idx)
    y = torch.zeros_like(x)
    for j in range(k):
        We1 = W1[idx[:, j]]            # [T, 2f, d]
        We2 = W2[idx[:, j]]            # [T, d, f]
        h = torch.einsum("tnd,td->tn", We1, x)
        a = torch.nn.functional.silu(h[:, :f]) * h[:, f:]
        y = y + w[:, j:j + 1] * torch.einsum("tdf,tf->td", We2, a)
    return y


@pytest.mark.parametrize("renorm", [1, 0])
def test_backward_against_torch_autograd(renorm):
    cfg, inp, z = small_case(T=20, d=8, E=5, k=3, f=6, seed=8)
    fwd = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k, renorm)
    g = O.layer_bwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], fwd, renorm, W_r=None)
    tx = torch.tensor(inp["x"], dtype=torch.float64, requires_grad=True)
    tz = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    tw1 = torch.tensor(inp["W1"], dtype=torch.float64, requires_grad=True)
    tw2 = torch.tensor(inp["W2"], dtype=torch.float64, requires_grad=True)
    ty = torch_layer(tx, tz, tw1, tw2, torch.tensor(fwd["idx"], dtype=torch.int64), cfg.k, renorm)
    assert np.allclose(ty.detach().numpy(), fwd["y"], rtol=1e-11, atol=1e-13)
    (ty * torch.tensor(inp["dy"], dtype=torch.float64)).sum().backward()
    assert np.allclose(g["dx"], tx.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(g["dz"], tz.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(g["dW1"], tw1.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(g["dW2"], tw2.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_router_gradients_included_when_requested():
    cfg, inp, z = small_case(T=10, d=8, E=4, k=2, f=6, seed=2)
    fwd = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k)
    g0 = O.layer_bwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], fwd)
    g1 = O.layer_bwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], fwd, W_r=inp["W_r"])
    assert np.allclose(g1["dx"] - g0["dx"], g0["dz"] @ inp["W_r"].astype(np.float64).T)
    assert np.allclose(g1["dW_r"], inp["x"].astype(np.float64).T @ g0["dz"])


def test_empty_expert_gets_zero_gradients():
    cfg, inp, z = small_case(T=30, E=5, k=2)
    z[:, 1] = -1e4
    fwd = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k)
    assert fwd["counts"][1] == 0
    g = O.layer_bwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], fwd)
    assert np.all(g["dW1"][1] == 0.0) and np.all(g["dW2"][1] == 0.0)
    assert np.any(g["dW1"][0] != 0.0)


def test_synthetic_shapes_follow_table2():
    rows = {}
    with open(__file__.rsplit("/", 1)[0] + "/golden/table2_model_shapes.txt") as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows[p[0]] = dict(h=int(p[2]), hffn=int(p[5]), E=int(p[6]), k=int(p[7]))
    mx = CONFIGS["mixtral"]
    assert (mx.d, mx.f, mx.E, mx.k) == (rows["Mixtral-8x7B"]["h"], rows["Mixtral-8x7B"]["hffn"],
                                        rows["Mixtral-8x7B"]["E"], rows["Mixtral-8x7B"]["k"])
    fg = CONFIGS["finegrained"]
    assert (fg.d, fg.f, fg.E) == (rows["DeepSeekMoE"]["h"], rows["DeepSeekMoE"]["hffn"], rows["DeepSeekMoE"]["E"])
    sk = CONFIGS["skewed"]
    assert sk.d == rows["Internal-352B"]["h"] and sk.E == rows["Internal-352B"]["E"]


# ---- Section 4.1 operator order (row select inside FC1, gate weight after SwiGLU) -------------------------

@pytest.mark.parametrize("variant", ["full", "range", "capacity"])
def test_folded_order_equals_the_plain_layer(variant):
    # The reordered layer is the same function: pinned against layer_fwd / layer_bwd (themselves pinned by
    # finite differences and autograd above), on a full route, an expert-parallel share and a route with drops.
    rng = np.random.default_rng(31)
    T, d, E, k, f = 37, 16, 6, 3, 8
    x = rng.standard_normal((T, d))
    dy = rng.standard_normal((T, d))
    logits = rng.standard_normal((T, E)).astype(np.float32)
    W1 = rng.standard_normal((E, 2 * f, d)) * 0.3
    W2 = rng.standard_normal((E, d, f)) * 0.3
    if variant == "full":
        r = O.route(logits, k)
        W1l, W2l = W1, W2
    elif variant == "range":
        r = O.route_range(logits, k, 2, 5)
        W1l, W2l = W1[2:5], W2[2:5]
    else:
        r = O.route_capacity(logits, k, 3, 25)
        W1l, W2l = W1, W2
        assert (r["inv_perm"] < 0).any()
    plain = O.layer_fwd_routed(x, r, W1l, W2l, k)
    fold = O.layer_fwd_folded(x, r, W1l, W2l, k)
    M = int(r["offsets"][-1])
    np.testing.assert_allclose(fold["y"], plain["y"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(fold["H"][:M], plain["H"][:M], rtol=0, atol=1e-12)
    np.testing.assert_allclose(fold["Yw"][:M], plain["Y"][:M] * fold["row_w"][:, None], rtol=0, atol=1e-12)
    pb = O.layer_bwd_routed(x, W1l, W2l, k, dy, plain)
    fb = O.layer_bwd_folded(x, W1l, W2l, k, dy, fold)
    for key in ("dw", "dx", "dW1", "dW2"):
        np.testing.assert_allclose(fb[key], pb[key], rtol=0, atol=1e-11, err_msg=key)
    np.testing.assert_allclose(fb["dxp"][:M], pb["dxp"][:M], rtol=0, atol=1e-11)
    np.testing.assert_allclose(fb["dH0"][:M] * fold["row_w"][:, None], pb["dH"][:M], rtol=0, atol=1e-11)
    np.testing.assert_allclose(fb["dxp0"][:M] * fold["row_w"][:, None], pb["dxp"][:M], rtol=0, atol=1e-11)


def test_folded_gate_gradient_by_finite_differences():
    # d_row_w is the derivative of <dy, y> w.r.t. each row's gate weight with the rest held fixed
    rng = np.random.default_rng(32)
    T, d, E, k, f = 9, 8, 3, 2, 4
    x = rng.standard_normal((T, d))
    dy = rng.standard_normal((T, d))
    logits = rng.standard_normal((T, E)).astype(np.float32)
    W1 = rng.standard_normal((E, 2 * f, d)) * 0.4
    W2 = rng.standard_normal((E, d, f)) * 0.4
    r = O.route(logits, k)
    fwd = O.layer_fwd_folded(x, r, W1, W2, k)
    g = O.layer_bwd_folded(x, W1, W2, k, dy, fwd)["d_row_w"]
    eps = 1e-6
    for row in range(0, T * k, 5):
        vals = []
        for sgn in (+1, -1):
            rw = fwd["row_w"].copy()
            rw[row] += sgn * eps
            _, _, Yw = O.expert_ffn_fwd_folded(x, fwd["tok"], rw, r["offsets"], W1, W2)
            vals.append(float((dy * O.combine(Yw, r["inv_perm"], None, T, k)).sum()))
        assert abs((vals[0] - vals[1]) / (2 * eps) - g[row]) < 1e-6
