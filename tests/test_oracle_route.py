"""Pins for the oracle's routing functions: brute force on tiny inputs, constructed ties,
closed forms and library routines.  No GPU."""
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import moe_oracle as O
from synth.moe_inputs import MoEConfig, make_inputs, random_logits


def brute_topk(z_row, k):
    """Full ordering of one token's experts by (logit descending, id ascending), pure Python."""
    order = sorted(range(len(z_row)), key=lambda e: (-float(z_row[e]), e))
    return order[:k]


def brute_row_map(idx, E):
    """Definition of the row map with explicit loops: row(a) = offset[e(a)] + #{a' < a : e(a') = e(a)}."""
    e_of_a = [int(v) for v in idx.reshape(-1)]
    M = len(e_of_a)
    counts = [0] * E
    for e in e_of_a:
        counts[e] += 1
    offsets = [0] * (E + 1)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    perm = [None] * M
    inv = [None] * M
    for a in range(M):
        earlier = sum(1 for b in range(a) if e_of_a[b] == e_of_a[a])
        r = offsets[e_of_a[a]] + earlier
        perm[r] = a
        inv[a] = r
    return counts, offsets, perm, inv


@pytest.mark.parametrize("T,E,k,quantum", [(37, 8, 2, None), (64, 8, 2, 0.5), (50, 5, 5, 1.0),
                                           (33, 16, 1, 0.25), (20, 64, 8, 0.5), (9, 3, 2, 2.0)])
def test_topk_matches_brute_force(T, E, k, quantum):
    z = random_logits(T, E, seed=T + E, quantum=quantum)
    idx = O.topk_select(z, k)
    for t in range(T):
        assert list(idx[t]) == brute_topk(z[t], k)


def test_constructed_ties():
    # all equal: experts 0..k-1, weights 1/k
    z = np.full((3, 6), 1.25, dtype=np.float32)
    r = O.route(z, 3)
    assert np.array_equal(r["idx"], np.tile(np.arange(3, dtype=np.int32), (3, 1)))
    assert np.allclose(r["w"], 1.0 / 3.0, atol=1e-15)
    # -0.0 and +0.0 are the same logit: lower id wins
    z = np.array([[-0.0, 0.0, -1.0, 0.0]], dtype=np.float32)
    assert list(O.topk_select(z, 2)[0]) == [0, 1]
    z = np.array([[0.0, -0.0, -1.0, 0.0]], dtype=np.float32)
    assert list(O.topk_select(z, 3)[0]) == [0, 1, 3]
    # duplicates straddling the k-th place: the lower ids among the equals get in
    z = np.array([[1.0, 5.0, 1.0, 1.0, 7.0]], dtype=np.float32)
    assert list(O.topk_select(z, 3)[0]) == [4, 1, 0]
    assert list(O.topk_select(z, 4)[0]) == [4, 1, 0, 2]
    # pairs equal: order inside the pair is by id
    z = np.array([[2.0, 3.0, 3.0, 2.0]], dtype=np.float32)
    assert list(O.topk_select(z, 4)[0]) == [1, 2, 0, 3]
    # k = 1 is argmax with the first occurrence
    z = random_logits(100, 7, seed=3, quantum=1.0)
    assert np.array_equal(O.topk_select(z, 1)[:, 0], np.argmax(z, axis=1))
    # E = k selects everything
    z = random_logits(10, 4, seed=5)
    assert np.array_equal(np.sort(O.topk_select(z, 4), axis=1), np.tile(np.arange(4), (10, 1)))


def test_slot_order_is_descending_logit():
    z = random_logits(200, 16, seed=9)
    idx = O.topk_select(z, 5)
    sel = np.take_along_axis(z, idx.astype(np.int64), axis=1)
    assert np.all(np.diff(sel, axis=1) <= 0)


def test_gate_weights_closed_forms():
    z = random_logits(128, 8, seed=1)
    for k in (1, 2, 8):
        idx = O.topk_select(z, k)
        w = O.gate_weights(z, idx, renorm=1)
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-12)
        assert np.all(w > 0)
    # k = E with renormalisation is the full softmax (library routine), in the selected order
    idx = O.topk_select(z, 8)
    w = O.gate_weights(z, idx, renorm=1)
    p = scipy_softmax(z.astype(np.float64), axis=1)
    assert np.allclose(w, np.take_along_axis(p, idx.astype(np.int64), axis=1), rtol=1e-12, atol=1e-15)
    # renorm = 0: softmax over all experts read at the selected ones
    idx = O.topk_select(z, 2)
    w0 = O.gate_weights(z, idx, renorm=0)
    assert np.allclose(w0, np.take_along_axis(p, idx.astype(np.int64), axis=1), rtol=1e-12, atol=1e-15)
    # renormalising the selected entries of the full softmax gives the renorm=1 weights
    w1 = O.gate_weights(z, idx, renorm=1)
    assert np.allclose(w0 / w0.sum(axis=1, keepdims=True), w1, rtol=1e-12)
    # two experts: weight of the top one is the logistic of the logit gap
    sel = np.take_along_axis(z.astype(np.float64), idx.astype(np.int64), axis=1)
    assert np.allclose(w1[:, 0], 1.0 / (1.0 + np.exp(-(sel[:, 0] - sel[:, 1]))), rtol=1e-12)


def test_gate_weights_shift_invariance_and_large_logits():
    z = (random_logits(16, 8, seed=2) * 30).astype(np.float32)
    idx = O.topk_select(z, 3)
    w = O.gate_weights(z, idx)
    w_shift = O.gate_weights(z.astype(np.float64) + 1000.0, idx)
    assert np.all(np.isfinite(w)) and np.allclose(w, w_shift, rtol=1e-9)


@pytest.mark.parametrize("T,E,k,quantum", [(23, 4, 2, None), (40, 8, 3, 1.0), (16, 6, 6, None), (31, 9, 1, 0.5)])
def test_row_map_matches_brute_force(T, E, k, quantum):
    z = random_logits(T, E, seed=7 * T + k, quantum=quantum)
    r = O.route(z, k)
    counts, offsets, perm, inv = brute_row_map(r["idx"], E)
    assert list(r["counts"]) == counts
    assert list(r["offsets"]) == offsets
    assert list(r["perm"]) == perm
    assert list(r["inv_perm"]) == inv


def test_row_map_invariants_and_library_routines():
    T, E, k = 3000, 64, 8
    z = random_logits(T, E, seed=11)
    z[:, 5] -= 100.0          # expert 5 is never chosen
    r = O.route(z, k)
    M = T * k
    e_of_a = r["idx"].reshape(-1)
    assert r["counts"].sum() == M and r["counts"][5] == 0
    assert np.array_equal(r["counts"], np.bincount(e_of_a, minlength=E))
    assert np.array_equal(r["offsets"], np.concatenate([[0], np.cumsum(r["counts"])]))
    assert r["offsets"][E] == M and np.all(np.diff(r["offsets"]) >= 0)
    assert np.array_equal(np.sort(r["perm"]), np.arange(M))
    assert np.array_equal(r["inv_perm"][r["perm"]], np.arange(M))
    e_sorted = e_of_a[r["perm"]]
    assert np.all(np.diff(e_sorted) >= 0)
    for e in range(E):
        seg = r["perm"][r["offsets"][e]:r["offsets"][e + 1]]
        assert np.all(np.diff(seg) > 0)
        assert np.all(e_of_a[seg] == e)
    # each token's k experts are distinct
    assert all(len(set(row)) == k for row in r["idx"][:200])


def test_all_tokens_one_expert():
    z = np.zeros((17, 4), dtype=np.float32)
    z[:, 2] = 5.0
    r = O.route(z, 1)
    assert list(r["counts"]) == [0, 0, 17, 0]
    assert list(r["offsets"]) == [0, 0, 0, 17, 17]
    assert np.array_equal(r["perm"], np.arange(17))


def _num_jac_w(z64, idx, renorm, eps=1e-6):
    T, E = z64.shape
    k = idx.shape[1]
    J = np.zeros((T, k, E))
    for e in range(E):
        zp, zm = z64.copy(), z64.copy()
        zp[:, e] += eps
        zm[:, e] -= eps
        J[:, :, e] = (O.gate_weights(zp, idx, renorm) - O.gate_weights(zm, idx, renorm)) / (2 * eps)
    return J


@pytest.mark.parametrize("renorm", [1, 0])
def test_route_bwd_finite_differences(renorm):
    T, E, k = 6, 7, 3
    z = random_logits(T, E, seed=4)
    idx = O.topk_select(z, k)
    w = O.gate_weights(z, idx, renorm)
    rng = np.random.default_rng(0)
    dw = rng.standard_normal((T, k))
    dz = O.route_bwd(z, idx, w, dw, renorm)
    J = _num_jac_w(z.astype(np.float64), idx, renorm)
    dz_num = np.einsum("tk,tke->te", dw, J)
    assert np.allclose(dz, dz_num, rtol=1e-6, atol=1e-8)
    if renorm:
        # softmax Jacobian has the all-ones vector in its null space; unselected entries are zero
        assert np.allclose(dz.sum(axis=1), 0.0, atol=1e-12)
        mask = np.ones((T, E), bool)
        np.put_along_axis(mask, idx.astype(np.int64), False, axis=1)
        assert np.all(dz[mask] == 0.0)


def test_router_matmul_and_bwd():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 4))
    W = rng.standard_normal((4, 3))
    b = rng.standard_normal(3)
    z = O.router_logits(x, W, b)
    for t in range(5):
        for e in range(3):
            assert abs(z[t, e] - (sum(x[t, i] * W[i, e] for i in range(4)) + b[e])) < 1e-12
    dz = rng.standard_normal((5, 3))
    dW, dx = O.router_bwd(x, W, dz)
    # adjoint identities: <dz, x dW'> = <dW, dW'> for any dW', likewise for x
    Wp = rng.standard_normal((4, 3))
    xp = rng.standard_normal((5, 4))
    assert np.isclose((dz * (x @ Wp)).sum(), (dW * Wp).sum())
    assert np.isclose((dz * (xp @ W)).sum(), (dx * xp).sum())


# ---- expert-parallel share (Section 3.2: local scatter after the all-gather) -------------------------------
def test_route_range_is_the_filtered_full_route():
    z = random_logits(257, 12, seed=5, quantum=0.5)
    full = O.route(z, 3)
    for lo, hi in ((0, 12), (0, 4), (4, 9), (9, 12), (5, 5)):
        r = O.route_range(z, 3, lo, hi)
        assert np.array_equal(r["idx"], full["idx"]) and np.array_equal(r["w"], full["w"])
        assert np.array_equal(r["counts"], full["counts"])
        keep = full["perm"][full["offsets"][lo]:full["offsets"][hi]]          # the full map's rows of the local experts
        assert np.array_equal(r["perm"], keep)
        assert np.array_equal(r["offsets"], full["offsets"][lo:hi + 1] - full["offsets"][lo])
        e_of_a = full["idx"].reshape(-1)
        local = (e_of_a >= lo) & (e_of_a < hi)
        assert np.all(r["inv_perm"][~local] == -1)
        assert np.array_equal(r["inv_perm"][local], full["inv_perm"][local] - full["offsets"][lo])


def test_expert_parallel_shares_add_up_to_the_full_layer():
    """Partition invariance: partial outputs and partial input gradients of disjoint expert ranges sum to the
    full layer's; expert gradients and gate-weight gradients are those of the full layer, range by range."""
    cfg = MoEConfig("t", T=96, d=24, E=6, k=3, f=16, dtype="f32", w_std=0.3, wr_std=0.8)
    inp = make_inputs(cfg, seed=4)
    z = O.router_logits(inp["x"], inp["W_r"]).astype(np.float32)
    full = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k)
    gfull = O.layer_bwd(inp["x"], z, inp["W1"], inp["W2"], cfg.k, inp["dy"], full)
    y = np.zeros_like(full["y"]); dx = np.zeros_like(gfull["dx"]); dw = np.zeros_like(gfull["dw"])
    for lo, hi in ((0, 2), (2, 3), (3, 6)):
        f = O.layer_fwd_range(inp["x"], z, inp["W1"][lo:hi], inp["W2"][lo:hi], cfg.k, lo, hi)
        g = O.layer_bwd_range(inp["x"], z, inp["W1"][lo:hi], inp["W2"][lo:hi], cfg.k, inp["dy"], f)
        y += f["y"]; dx += g["dx"]; dw += g["dw"]
        assert np.allclose(g["dW1"], gfull["dW1"][lo:hi], rtol=1e-12, atol=1e-12)
        assert np.allclose(g["dW2"], gfull["dW2"][lo:hi], rtol=1e-12, atol=1e-12)
        e_of = full["idx"]
        assert np.all(g["dw"][(e_of < lo) | (e_of >= hi)] == 0)
    assert np.allclose(y, full["y"], rtol=1e-12, atol=1e-12)
    assert np.allclose(dx, gfull["dx"], rtol=1e-12, atol=1e-12)
    assert np.allclose(dw, gfull["dw"], rtol=1e-12, atol=1e-12)


# ---- load balance (Section 3.2: auxiliary loss and token dropping per device) ------------------------------------
def test_balance_loss_closed_forms_and_gradient():
    T, E, k, G = 64, 8, 2, 4
    # uniform logits: s = 1/E, P'_g = per/E; f'_g depends on the selection only; sum_g f'_g = G * (E/(kT)) * kT / E / ... = G
    z = np.zeros((T, E), dtype=np.float32)
    idx = O.topk_select(z, k)                              # ties -> experts 0 and 1 for every token
    loss, fg, Pg = O.balance_loss(z, idx, G, alpha=0.5)
    assert np.allclose(Pg, 2 / 8) and np.allclose(fg, [E / (k * T) * T * 2 / 2, 0, 0, 0])     # all assignments on device 0
    assert np.isclose(loss, 0.5 * fg[0] * 0.25)
    # perfectly balanced selection and uniform affinities give alpha (the textbook minimum of this loss)
    idx_bal = np.stack([np.arange(T) % E, (np.arange(T) + 4) % E], axis=1)
    loss_bal, fg_bal, _ = O.balance_loss(z, idx_bal, G, alpha=1.0)
    assert np.allclose(fg_bal, 1.0) and np.isclose(loss_bal, 1.0)
    # gradient against central differences (f held fixed, as the analytic form assumes)
    rng = np.random.default_rng(2)
    z = rng.standard_normal((12, E))
    idx = O.topk_select(z.astype(np.float32), k)
    g = O.balance_loss_bwd(z, idx, G, alpha=0.7)
    num = np.zeros_like(z)
    for t in range(12):
        for c in range(E):
            zp, zm = z.copy(), z.copy()
            zp[t, c] += 1e-6; zm[t, c] -= 1e-6
            num[t, c] = (O.balance_loss(zp, idx, G, 0.7)[0] - O.balance_loss(zm, idx, G, 0.7)[0]) / 2e-6
    assert np.allclose(g, num, rtol=1e-5, atol=1e-9)
    assert np.allclose(g.sum(axis=1), 0, atol=1e-15)          # softmax gradients sum to zero per token


def test_capacity_keep_drops_the_lowest_affinities_per_device():
    rng = np.random.default_rng(8)
    T, E, k, G, cap = 50, 6, 2, 3, 20
    z = rng.standard_normal((T, E)).astype(np.float32)
    z[:, 0] += 1.5                                          # device 0 is overloaded
    idx = O.topk_select(z, k)
    score = O.affinity_scores(z, idx)
    assert np.allclose(score, np.take_along_axis(scipy_softmax(z.astype(np.float64), axis=1), idx.astype(np.int64), axis=1), rtol=1e-6)
    keep = O.capacity_keep(score, idx, E, G, cap)
    grp = idx // (E // G)
    for g in range(G):
        m = grp == g
        assert keep[m].sum() == min(cap, m.sum())
        if m.sum() > cap:                                   # every kept score >= every dropped score of the device
            assert score[m & keep].min() >= score[m & ~keep].max()
    # brute force on a tiny case with ties: equal affinities -> the lower assignment id stays
    z2 = np.zeros((4, 2), dtype=np.float32)
    i2 = O.topk_select(z2, 1)
    keep2 = O.capacity_keep(O.affinity_scores(z2, i2), i2, 2, 1, 2)
    assert keep2.reshape(-1).tolist() == [True, True, False, False]
    assert O.capacity_keep(score, idx, E, G, T * k).all()   # capacity never reached: nothing dropped


def test_route_capacity_row_map():
    z = random_logits(200, 8, seed=3)
    z[:, 1] += 2.0
    full = O.route(z, 2)
    r = O.route_capacity(z, 2, n_groups=4, capacity=60)
    assert np.array_equal(r["idx"], full["idx"]) and np.array_equal(r["w"], full["w"])
    kf = r["keep"].reshape(-1)
    assert np.all(r["inv_perm"][~kf] == -1)
    assert np.array_equal(np.sort(r["perm"]), np.flatnonzero(kf))
    e_rows = full["idx"].reshape(-1)[r["perm"]]
    assert np.all(np.diff(e_rows) >= 0)                       # grouped by expert
    for e in range(8):
        seg = r["perm"][r["offsets"][e]:r["offsets"][e + 1]]
        assert np.all(np.diff(seg) > 0) and r["counts"][e] == seg.size
    assert r["counts"].reshape(4, 2).sum(axis=1).max() <= 60
    big = O.route_capacity(z, 2, n_groups=4, capacity=10 ** 6)
    for nm in ("counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(big[nm], full[nm]), nm
