"""CPU oracle for one GPU's share of an MoE FFN layer, forward and backward.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
layer computes, in float64 numpy.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does, and it
shares no code, tables or helpers with the HIP kernels.

What the paper fixes and what is read into it
---------------------------------------------
The paper treats the layer's mathematics as background (Section 2.1: a trainable
gate routes each token to its top-k experts, Fig. 2) and describes the operators
and their order (Section 3.2 "Efficient operators": a row map computed from the
routing result drives scatter and gather; Section 4.1: FC1 GroupedGEMM -> SwiGLU
-> weighted sum -> FC2 GroupedGEMM, and which tensors the FC2 backward needs;
Section 4.2: tokens ordered by expert, then by source rank, which on one rank is
plain token order; Section 5 and Section 7 "FP8 training": E4M3 everywhere,
per-token quantisation forward, per-channel quantisation in 128-token groups
backward, gate weight applied after FC2 in the FP8 variant).  The method reaches
exactly the plain layer result, so every function below is the plain definition
written out.  Readings where the paper is silent (softmax gate over the selected
logits, ties toward the lower expert id, slot order by descending logit, stable
order inside an expert's segment, dropless, scale = amax/448; for the FP8 backward
GEMMs: a second quantisation of the weights along their other axis, and power-of-two
group scales for the operands whose contraction index is the token) are stated where
they are used.  The FP8 functions take an optional store="bf16": intermediate tensors are
then rounded to bfloat16 where one step hands them to the next (Section 5's BF16
mixed-precision training keeps activations in that type), so that a cast decides on the
values a bf16 pipeline holds; the default keeps float64 between the casts.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
brute force, closed forms, finite differences or an independent library routine.
Nothing in this file is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Routing: Section 2.1 (top-k gate), Section 3.2 (row map), Section 4.2 (order)
# --------------------------------------------------------------------------

def topk_select(logits: np.ndarray, k: int) -> np.ndarray:
    """Experts chosen per token, as int32 [T, k].

    Reading: the k largest *logits* win; equal logits go to the lower expert id
    (so -0.0 and +0.0 tie); slot j holds the (j+1)-th largest.
    """
    z = np.asarray(logits)
    assert z.dtype == np.float32 and z.ndim == 2
    assert np.all(np.isfinite(z)), "routing is defined for finite logits only"
    T, E = z.shape
    assert 1 <= k <= E
    # A stable ascending sort of -z keeps equal logits in ascending expert id.
    order = np.argsort(-z.astype(F64), axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def gate_weights(logits: np.ndarray, idx: np.ndarray, renorm: int = 1) -> np.ndarray:
    """Gate weights float64 [T, k].

    renorm=1: softmax over the k selected logits (equals softmax over all experts
    followed by renormalising the selected ones).  renorm=0: softmax over all E
    experts, read at the selected ones.
    """
    z = np.asarray(logits).astype(F64)
    sel = np.take_along_axis(z, idx.astype(np.int64), axis=1)
    m = z.max(axis=1, keepdims=True)          # the row maximum is always selected
    if renorm:
        e = np.exp(sel - m)
        return e / e.sum(axis=1, keepdims=True)
    den = np.exp(z - m).sum(axis=1, keepdims=True)
    return np.exp(sel - m) / den


def row_map(idx: np.ndarray, E: int):
    """counts [E], offsets [E+1], perm [M], inv_perm [M] (all int32).

    Assignment id a = t*k + j.  Expert e owns rows offsets[e] .. offsets[e+1]-1 and
    inside that segment assignments keep ascending id (Section 4.2: by expert, then
    by source; one source here, so by token, then slot).  perm[row] = a,
    inv_perm[a] = row.  Dropless and unpadded: offsets is the plain prefix sum.
    """
    e_of_a = np.asarray(idx).reshape(-1).astype(np.int64)
    M = e_of_a.size
    counts = np.zeros(E, dtype=np.int64)
    for e in range(E):
        counts[e] = int(np.count_nonzero(e_of_a == e))
    offsets = np.zeros(E + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(counts)
    perm = np.argsort(e_of_a, kind="stable")
    inv_perm = np.empty(M, dtype=np.int64)
    inv_perm[perm] = np.arange(M)
    return (counts.astype(np.int32), offsets.astype(np.int32),
            perm.astype(np.int32), inv_perm.astype(np.int32))


def route(logits: np.ndarray, k: int, renorm: int = 1) -> dict:
    idx = topk_select(logits, k)
    w = gate_weights(logits, idx, renorm)
    counts, offsets, perm, inv_perm = row_map(idx, logits.shape[1])
    return dict(idx=idx, w=w, counts=counts, offsets=offsets, perm=perm, inv_perm=inv_perm)


def route_range(logits: np.ndarray, k: int, e_lo: int, e_hi: int, renorm: int = 1) -> dict:
    """One GPU's expert-parallel share (Section 3.2: after the all-gather a local scatter keeps only the
    tokens routed to local experts).  The gate runs over all E experts as in route(); only assignments
    whose expert lies in [e_lo, e_hi) get a row.  counts [E] stays global; offsets [e_hi-e_lo+1] and
    perm [M_local] cover the local experts (same order: by expert, then ascending assignment id);
    inv_perm [T*k] is -1 for assignments that were dropped."""
    idx = topk_select(logits, k)
    w = gate_weights(logits, idx, renorm)
    E = logits.shape[1]
    e_of_a = idx.reshape(-1).astype(np.int64)
    counts = np.array([np.count_nonzero(e_of_a == e) for e in range(E)], dtype=np.int32)
    offsets = np.zeros(e_hi - e_lo + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(counts[e_lo:e_hi])
    perm = np.concatenate([np.flatnonzero(e_of_a == e) for e in range(e_lo, e_hi)] + [np.zeros(0, np.int64)])
    inv_perm = np.full(e_of_a.size, -1, dtype=np.int64)
    inv_perm[perm] = np.arange(perm.size)
    return dict(idx=idx, w=w, counts=counts, offsets=offsets.astype(np.int32), perm=perm.astype(np.int32),
                inv_perm=inv_perm.astype(np.int32))


def layer_fwd_range(x, logits, W1_local, W2_local, k: int, e_lo: int, e_hi: int, renorm: int = 1) -> dict:
    """Forward of one expert-parallel share: W1_local / W2_local hold experts e_lo..e_hi-1; y is the partial
    sum over the local experts (what a reduce-scatter would add up across the ranks)."""
    return layer_fwd_routed(x, route_range(logits, k, e_lo, e_hi, renorm), W1_local, W2_local, k)


def layer_fwd_routed(x, r: dict, W1, W2, k: int) -> dict:
    """Forward from a routing result r (route_range or route_capacity): assignments without a row contribute
    nothing; W1 / W2 hold the experts that r's offsets cover."""
    T = x.shape[0]
    r = dict(r)
    xp = dispatch(x, r["perm"], k)
    H, A, Y = expert_ffn_fwd(xp, r["offsets"], W1, W2)
    y = combine(Y, r["inv_perm"], r["w"], T, k)
    r.update(xp=xp, H=H, A=A, Y=Y, y=y)
    return r


def layer_bwd_range(x, logits, W1_local, W2_local, k: int, dy, fwd: dict) -> dict:
    return layer_bwd_routed(x, W1_local, W2_local, k, dy, fwd)


def layer_bwd_routed(x, W1_local, W2_local, k: int, dy, fwd: dict) -> dict:
    """Backward of layer_fwd_range: gradients of the local experts, the local part of dx and of the gate-weight
    gradient (zero for dropped assignments); the gate's own backward needs the sum of dw over all shares."""
    T = x.shape[0]
    dYp = dispatch(dy, fwd["perm"], k, row_mul=fwd["w"])
    dw = gate_grad(dy, fwd["Y"], fwd["inv_perm"], T, k)
    dxp, dW1, dW2, dH = expert_ffn_bwd(fwd["xp"], fwd["H"], dYp, fwd["offsets"], W1_local, W2_local)
    dx = combine(dxp, fwd["inv_perm"], None, T, k)
    return dict(dYp=dYp, dw=dw, dxp=dxp, dW1=dW1, dW2=dW2, dH=dH, dx=dx)


def route_bwd(logits, idx, w, dw, renorm: int = 1) -> np.ndarray:
    """d(loss)/d(logits) float64 [T, E] given d(loss)/d(w); the selection is constant."""
    T, E = np.asarray(logits).shape
    idx64 = idx.astype(np.int64)
    w = np.asarray(w, F64)
    dw = np.asarray(dw, F64)
    dz = np.zeros((T, E), dtype=F64)
    if renorm:
        inner = (w * dw).sum(axis=1, keepdims=True)
        np.put_along_axis(dz, idx64, w * (dw - inner), axis=1)
        return dz
    z = np.asarray(logits).astype(F64)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    inner = (w * dw).sum(axis=1, keepdims=True)      # w_j = p[e_j]
    dz = -p * inner
    sel = np.take_along_axis(dz, idx64, axis=1) + w * dw
    np.put_along_axis(dz, idx64, sel, axis=1)
    return dz


# --------------------------------------------------------------------------
# Router matmul (the "routing scores" operator of Section 7)
# --------------------------------------------------------------------------

def router_logits(x, W_r, bias=None) -> np.ndarray:
    """z = x W_r (+ b) in float64; x [T,d], W_r [d,E]."""
    z = np.asarray(x, F64) @ np.asarray(W_r, F64)
    if bias is not None:
        z = z + np.asarray(bias, F64)[None, :]
    return z


def router_bwd(x, W_r, dz):
    """dW_r = x^T dz,  dx_r = dz W_r^T."""
    x = np.asarray(x, F64)
    dz = np.asarray(dz, F64)
    return x.T @ dz, dz @ np.asarray(W_r, F64).T


# --------------------------------------------------------------------------
# Dispatch / combine: Section 3.2 (scatter and gather by a precomputed row map)
# --------------------------------------------------------------------------

def dispatch(x, perm, k: int, row_mul=None) -> np.ndarray:
    """xp[r,:] = x[perm[r] div k, :]  (times row_mul[perm[r]] when given)."""
    x = np.asarray(x, F64)
    a = perm.astype(np.int64)
    xp = x[a // k, :]
    if row_mul is not None:
        xp = xp * np.asarray(row_mul, F64).reshape(-1)[a][:, None]
    return xp


def combine(Y, inv_perm, w, T: int, k: int) -> np.ndarray:
    """y[t,:] = sum_j w[t,j] * Y[inv_perm[t*k+j], :], slots in ascending j.  w=None: unweighted.
    An assignment without a row (inv_perm < 0: its expert is not local, see route_range) adds nothing."""
    Y = np.asarray(Y, F64)
    rows = inv_perm.astype(np.int64).reshape(T, k)
    y = np.zeros((T, Y.shape[1]), dtype=F64)
    for j in range(k):
        has = rows[:, j] >= 0
        term = np.zeros_like(y)
        term[has] = Y[rows[has, j], :]
        if w is not None:
            term = term * np.asarray(w, F64)[:, j][:, None]
        y += term
    return y


def gate_grad(dy, Y, inv_perm, T: int, k: int) -> np.ndarray:
    """dw[t,j] = <dy[t,:], Y[inv_perm[t*k+j], :]>  (derivative of combine w.r.t. the gate weight)."""
    dy = np.asarray(dy, F64)
    Y = np.asarray(Y, F64)
    rows = inv_perm.astype(np.int64).reshape(T, k)
    dw = np.zeros((T, k), dtype=F64)
    for j in range(k):
        has = rows[:, j] >= 0                      # assignments without a local row get no gradient here
        dw[has, j] = np.einsum("td,td->t", dy[has], Y[rows[has, j], :])
    return dw


# --------------------------------------------------------------------------
# Expert FFN: Section 4.1 (FC1 GroupedGEMM -> SwiGLU -> FC2 GroupedGEMM)
# --------------------------------------------------------------------------

def silu(g):
    return g / (1.0 + np.exp(-g))


def expert_ffn_fwd(xp, offsets, W1, W2):
    """Per expert e over its rows: G = X Wg^T, U = X Wu^T, A = silu(G)*U, Y = A Wd^T.

    W1 [E, 2f, d] holds the gate projection in rows 0..f-1 and the up projection in
    rows f..2f-1; W2 [E, d, f] is the down projection.  Returns H=[G|U], A, Y.
    """
    xp = np.asarray(xp, F64)
    E, two_f, d = W1.shape
    f = two_f // 2
    M = xp.shape[0]
    H = np.zeros((M, two_f), dtype=F64)
    A = np.zeros((M, f), dtype=F64)
    Y = np.zeros((M, d), dtype=F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        X = xp[lo:hi]
        G = X @ np.asarray(W1[e, :f, :], F64).T
        U = X @ np.asarray(W1[e, f:, :], F64).T
        H[lo:hi, :f] = G
        H[lo:hi, f:] = U
        A[lo:hi] = silu(G) * U
        Y[lo:hi] = A[lo:hi] @ np.asarray(W2[e], F64).T
    return H, A, Y


def swiglu_bwd(G, U, dA):
    """dG = dA*U*s*(1+G*(1-s)), dU = dA*G*s with s = sigmoid(G)."""
    s = 1.0 / (1.0 + np.exp(-G))
    return dA * U * s * (1.0 + G * (1.0 - s)), dA * G * s


def expert_ffn_bwd(xp, H, dY, offsets, W1, W2, A=None):
    """Gradients of expert_ffn_fwd: returns dxp [M,d], dW1 [E,2f,d], dW2 [E,d,f], dH [M,2f].

    A (the FC2 input) is recomputed from the saved H unless given (the fp8 path
    passes the quantised-dequantised A that FC2 actually consumed).  Experts with
    no rows get exactly-zero weight gradients.
    """
    xp = np.asarray(xp, F64)
    H = np.asarray(H, F64)
    dY = np.asarray(dY, F64)
    E, two_f, d = W1.shape
    f = two_f // 2
    M = xp.shape[0]
    dxp = np.zeros((M, d), dtype=F64)
    dH = np.zeros((M, two_f), dtype=F64)
    dW1 = np.zeros((E, two_f, d), dtype=F64)
    dW2 = np.zeros((E, d, f), dtype=F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        G, U = H[lo:hi, :f], H[lo:hi, f:]
        Ae = silu(G) * U if A is None else np.asarray(A[lo:hi], F64)
        dYe = dY[lo:hi]
        dA = dYe @ np.asarray(W2[e], F64)
        dW2[e] = dYe.T @ Ae
        dG, dU = swiglu_bwd(G, U, dA)
        dH[lo:hi, :f] = dG
        dH[lo:hi, f:] = dU
        dW1[e] = dH[lo:hi].T @ xp[lo:hi]
        dxp[lo:hi] = dH[lo:hi] @ np.asarray(W1[e], F64)
    return dxp, dW1, dW2, dH


# --------------------------------------------------------------------------
# Section 4.1 / 4.2 operator order: rows selected by the index map inside FC1 (no
# dispatched copy of the input), the gate weight multiplied right after SwiGLU so
# that the FC2 output need not be kept, the gate-weight gradient taken where the
# recomputed FC2 input is at hand.  Same layer, other association: pinned equal to
# layer_fwd / layer_bwd.
# --------------------------------------------------------------------------

def row_tokens(perm, k: int) -> np.ndarray:
    """Token whose copy dispatched row r is: perm[r] div k."""
    return np.asarray(perm, np.int64) // k


def row_gate_weights(w, perm) -> np.ndarray:
    """Gate weight of the assignment behind dispatched row r: w.flat[perm[r]]."""
    return np.asarray(w, F64).reshape(-1)[np.asarray(perm, np.int64)]


def expert_ffn_fwd_folded(x, tok, row_w, offsets, W1, W2):
    """[G|U] = x[tok[r]] W1^T,  A' = w_r * silu(G) * U,  Y' = A' W2^T  (Y' = w_r * Y).  Returns H, A', Y'."""
    x = np.asarray(x, F64)
    row_w = np.asarray(row_w, F64)
    E, two_f, d = W1.shape
    f = two_f // 2
    M = len(tok)
    H = np.zeros((M, two_f), dtype=F64)
    Aw = np.zeros((M, f), dtype=F64)
    Yw = np.zeros((M, d), dtype=F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        X = x[tok[lo:hi], :]
        G = X @ np.asarray(W1[e, :f, :], F64).T
        U = X @ np.asarray(W1[e, f:, :], F64).T
        H[lo:hi, :f] = G
        H[lo:hi, f:] = U
        Aw[lo:hi] = row_w[lo:hi, None] * silu(G) * U
        Yw[lo:hi] = Aw[lo:hi] @ np.asarray(W2[e], F64).T
    return H, Aw, Yw


def expert_ffn_bwd_folded(x, dy, tok, row_w, H, offsets, W1, W2):
    """Backward of expert_ffn_fwd_folded followed by an unweighted combine.

    dY'[r] = dy[tok[r]];  dA' = dY' W2 (gradient w.r.t. A' = w_r A);  d_row_w[r] = <dA'[r], A[r]> with A
    recomputed from H;  dW2 = dY'^T A'.  Everything downstream of dA' is linear in it, so the weight is applied
    once per row: dH0 = SwiGLU'(G, U, dA'), dxp0 = dH0 W1 (both WITHOUT the weight), the true input-row gradient
    is dxp = w_r dxp0, and dW1 = dH0^T (w_r x[tok[r]]).  Returns dxp, dW1, dW2, dH0, d_row_w, dxp0.
    """
    x = np.asarray(x, F64)
    dy = np.asarray(dy, F64)
    H = np.asarray(H, F64)
    row_w = np.asarray(row_w, F64)
    E, two_f, d = W1.shape
    f = two_f // 2
    M = H.shape[0]
    dxp0 = np.zeros((M, d), dtype=F64)
    dH0 = np.zeros((M, two_f), dtype=F64)
    dW1 = np.zeros((E, two_f, d), dtype=F64)
    dW2 = np.zeros((E, d, f), dtype=F64)
    d_row_w = np.zeros(M, dtype=F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        G, U = H[lo:hi, :f], H[lo:hi, f:]
        A = silu(G) * U
        dYw = dy[tok[lo:hi], :]
        dAw = dYw @ np.asarray(W2[e], F64)
        d_row_w[lo:hi] = np.einsum("rf,rf->r", dAw, A)
        dW2[e] = dYw.T @ (A * row_w[lo:hi, None])
        dG, dU = swiglu_bwd(G, U, dAw)
        dH0[lo:hi, :f] = dG
        dH0[lo:hi, f:] = dU
        dW1[e] = dH0[lo:hi].T @ (row_w[lo:hi, None] * x[tok[lo:hi], :])
        dxp0[lo:hi] = dH0[lo:hi] @ np.asarray(W1[e], F64)
    return dxp0 * row_w[:, None], dW1, dW2, dH0, d_row_w, dxp0


def layer_fwd_folded(x, r: dict, W1, W2, k: int) -> dict:
    """Forward from a routing result r in the Section 4.1 order.  Rows at or past offsets[E] do not exist."""
    T = x.shape[0]
    r = dict(r)
    M = int(r["offsets"][-1])
    tok = row_tokens(r["perm"][:M], k)
    rw = row_gate_weights(r["w"], r["perm"][:M])
    H, Aw, Yw = expert_ffn_fwd_folded(x, tok, rw, r["offsets"], W1, W2)
    y = combine(Yw, r["inv_perm"], None, T, k)
    r.update(tok=tok, row_w=rw, H=H, Aw=Aw, Yw=Yw, y=y)
    return r


def layer_bwd_folded(x, W1, W2, k: int, dy, fwd: dict) -> dict:
    """Backward of layer_fwd_folded up to the gate-weight gradient dw [T,k] (zero where an assignment has no row)."""
    T = x.shape[0]
    M = int(fwd["offsets"][-1])
    dxp, dW1, dW2, dH0, d_row_w, dxp0 = expert_ffn_bwd_folded(x, dy, fwd["tok"], fwd["row_w"], fwd["H"], fwd["offsets"], W1, W2)
    dw = np.zeros(T * k, dtype=F64)
    dw[np.asarray(fwd["perm"][:M], np.int64)] = d_row_w
    dx = combine(dxp0, fwd["inv_perm"], fwd["w"], T, k)          # the weight, once per row
    return dict(dw=dw.reshape(T, k), dxp=dxp, dxp0=dxp0, dW1=dW1, dW2=dW2, dH0=dH0, dx=dx, d_row_w=d_row_w)


# --------------------------------------------------------------------------
# Whole layer
# --------------------------------------------------------------------------

def layer_fwd(x, logits, W1, W2, k: int, renorm: int = 1) -> dict:
    """Forward of the whole path from fp32 logits: route, dispatch, expert FFN, combine."""
    T = x.shape[0]
    r = route(logits, k, renorm)
    xp = dispatch(x, r["perm"], k)
    H, A, Y = expert_ffn_fwd(xp, r["offsets"], W1, W2)
    y = combine(Y, r["inv_perm"], r["w"], T, k)
    r.update(xp=xp, H=H, A=A, Y=Y, y=y)
    return r


def layer_bwd(x, logits, W1, W2, k: int, dy, fwd: dict, renorm: int = 1, W_r=None) -> dict:
    """Backward of the whole path.  The top-k selection is treated as a constant.

    dY[r] = w[a]*dy[t];  dw = <dy, Y>;  expert-FFN gradients;  dx[t] = sum_j dxp[row(t,j)];
    dz from the gate; with W_r given the router matmul's gradients are added too.
    """
    T = x.shape[0]
    dYp = dispatch(dy, fwd["perm"], k, row_mul=fwd["w"])
    dw = gate_grad(dy, fwd["Y"], fwd["inv_perm"], T, k)
    dxp, dW1, dW2, dH = expert_ffn_bwd(fwd["xp"], fwd["H"], dYp, fwd["offsets"], W1, W2)
    dx = combine(dxp, fwd["inv_perm"], None, T, k)
    dz = route_bwd(logits, fwd["idx"], fwd["w"], dw, renorm)
    out = dict(dYp=dYp, dw=dw, dxp=dxp, dW1=dW1, dW2=dW2, dH=dH, dx=dx, dz=dz)
    if W_r is not None:
        dWr, dx_r = router_bwd(x, W_r, dz)
        out["dW_r"] = dWr
        out["dx"] = dx + dx_r
    return out


# --------------------------------------------------------------------------
# FP8 E4M3 cast (Section 5 "Communication compression for FP8 training", Section 7)
# --------------------------------------------------------------------------
# Reading: OCP e4m3fn -- 1 sign, 4 exponent (bias 7), 3 mantissa bits, subnormals
# down to 2^-9, largest finite 448, no infinity, NaN = S.1111.111.

E4M3_MAX = 448.0


def e4m3_decode(codes) -> np.ndarray:
    """Value of each 8-bit code as float64."""
    c = np.asarray(codes).astype(np.int64)
    s = np.where((c >> 7) & 1, -1.0, 1.0)
    e = (c >> 3) & 15
    m = (c & 7).astype(F64)
    sub = m / 8.0 * 2.0 ** -6
    nor = (1.0 + m / 8.0) * np.exp2((e - 7).astype(F64))
    v = s * np.where(e == 0, sub, nor)
    return np.where((e == 15) & ((c & 7) == 7), np.nan, v)


def e4m3_encode(v) -> np.ndarray:
    """Nearest code (ties to even mantissa), magnitudes above 448 saturate to 448; uint8."""
    v = np.asarray(v, F64)
    sign = np.signbit(v)
    a = np.minimum(np.abs(np.where(np.isnan(v), 0.0, v)), E4M3_MAX)
    # subnormal range and the first binade share the spacing 2^-9
    _, ex = np.frexp(np.where(a > 0, a, 1.0))       # a = mant * 2^ex, mant in [0.5, 1)
    e = np.maximum(ex - 1, -6)                       # unbiased exponent, clamped at the subnormal scale
    q = np.rint(a / np.exp2((e - 3).astype(F64)))    # multiples of 2^(e-3); rint = ties to even
    # q in [0, 16]: q < 8 subnormal (mantissa q), 8..15 normal, 16 carries into the next binade
    carry = q >= 16
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 8.0, q)
    code = np.where(q < 8, q, ((e + 7) * 8 + (q - 8))).astype(np.int64)
    code = np.where(np.isnan(v), 0x7F, code)
    return (code | (sign.astype(np.int64) << 7)).astype(np.uint8)


def _f32(a):
    return np.asarray(a, dtype=np.float32)


def _scale_and_codes(v32: np.ndarray, amax32: np.ndarray):
    """Reading: amax = 0 gives scale 1; inv = 448/amax and scale = amax/448 are single fp32
    divisions; the product v*inv is rounded to fp32, clamped to +-448, then encoded."""
    safe = np.where(amax32 > 0, amax32, np.float32(1.0)).astype(np.float32)
    inv = np.where(amax32 > 0, np.float32(E4M3_MAX) / safe, np.float32(1.0)).astype(np.float32)
    scale = np.where(amax32 > 0, safe / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
    p = (v32 * inv).astype(np.float32)
    p = np.clip(p, np.float32(-E4M3_MAX), np.float32(E4M3_MAX))
    return e4m3_encode(p), scale


def quant_rows(v):
    """Per-token (1 x cols) quantisation: codes uint8 [rows, cols], scales float32 [rows]."""
    v32 = _f32(v)
    amax = np.abs(v32).max(axis=1, keepdims=True) if v32.shape[1] else np.zeros((v32.shape[0], 1), np.float32)
    codes, scale = _scale_and_codes(v32, amax.astype(np.float32))
    return codes, scale.reshape(-1)


def quant_colgroup128(v, group: int = 128):
    """Per-channel quantisation inside groups of 128 consecutive rows (tokens):
    codes uint8 [rows, cols], scales float32 [ceil(rows/128), cols]."""
    v32 = _f32(v)
    rows, cols = v32.shape
    ng = (rows + group - 1) // group
    codes = np.zeros((rows, cols), dtype=np.uint8)
    scales = np.ones((ng, cols), dtype=np.float32)
    for g in range(ng):
        blk = v32[g * group:(g + 1) * group]
        amax = np.abs(blk).max(axis=0, keepdims=True).astype(np.float32)
        c, s = _scale_and_codes(blk, amax)
        codes[g * group:(g + 1) * group] = c
        scales[g] = s.reshape(-1)
    return codes, scales


def dequant_rows(codes, scales) -> np.ndarray:
    return e4m3_decode(codes) * np.asarray(scales, F64).reshape(-1, 1)


def dequant_colgroup128(codes, scales, group: int = 128) -> np.ndarray:
    rows = codes.shape[0]
    s = np.repeat(np.asarray(scales, F64), group, axis=0)[:rows]
    return e4m3_decode(codes) * s


def fake_quant_rows(v) -> np.ndarray:
    return dequant_rows(*quant_rows(v))


def bf16_round(v) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), returned as float64.  Finite inputs only."""
    b = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return b.astype(np.uint32).view(np.float32).astype(F64).reshape(np.shape(v))


def _stored(v, store):
    """The value of an intermediate tensor as later steps see it: itself (store None: float64 throughout), or its
    bfloat16 rounding (store "bf16": the tensor is kept in bf16 between two steps, and a cast that follows it takes
    its decisions on the kept values)."""
    if store is None:
        return v
    if store == "bf16":
        return bf16_round(v)
    raise ValueError(f"unknown storage type {store!r}")


def quant_weights(W1, W2):
    """Per-output-channel weight quantisation: each row of W1[e] (2f rows of length d) and of
    W2[e] (d rows of length f) gets one scale.  Returns (W1_hat, W2_hat) dequantised, float64."""
    E, two_f, d = W1.shape
    f = W2.shape[2]
    W1h = fake_quant_rows(_f32(W1).reshape(E * two_f, d)).reshape(E, two_f, d)
    W2h = fake_quant_rows(_f32(W2).reshape(E * d, f)).reshape(E, d, f)
    return W1h, W2h


def layer_fwd_fp8(x, logits, W1, W2, k: int, renorm: int = 1, store=None) -> dict:
    """Forward with the FP8 casts as part of the function (float64 in between).

    Quantisation points: x per token before dispatch; W1, W2 per output channel; the
    SwiGLU output A per token; the FC2 output Y per token; the gate weight is applied
    after FC2 on the dequantised Y (Section 7's placement for FP8).

    store = "bf16": the three tensors a step hands to the next one (the FC1 output H, the SwiGLU output before
    its cast, the FC2 output before its cast) are rounded to bfloat16 where they are handed over, the type the
    paper's BF16 mixed-precision training keeps activations in (Section 5); each cast then decides on the values a
    bf16 pipeline really holds.  The sums and SwiGLU themselves stay float64.
    """
    T = x.shape[0]
    r = route(logits, k, renorm)
    x_hat = fake_quant_rows(x)
    xp = dispatch(x_hat, r["perm"], k)
    W1h, W2h = quant_weights(W1, W2)
    E, two_f, d = W1.shape
    f = two_f // 2
    M = xp.shape[0]
    H = np.zeros((M, two_f), F64)
    A_hat = np.zeros((M, f), F64)
    Y = np.zeros((M, d), F64)
    for e in range(E):
        lo, hi = int(r["offsets"][e]), int(r["offsets"][e + 1])
        if hi == lo:
            continue
        G = _stored(xp[lo:hi] @ W1h[e, :f].T, store)
        U = _stored(xp[lo:hi] @ W1h[e, f:].T, store)
        H[lo:hi, :f], H[lo:hi, f:] = G, U
        A_hat[lo:hi] = fake_quant_rows(_stored(silu(G) * U, store))
        Y[lo:hi] = _stored(A_hat[lo:hi] @ W2h[e].T, store)
    Y_hat = fake_quant_rows(Y)
    y = combine(Y_hat, r["inv_perm"], r["w"], T, k)
    r.update(x_hat=x_hat, xp=xp, H=H, A=A_hat, Y=Y_hat, y=y)
    return r


def layer_bwd_fp8(x, logits, W1, W2, k: int, dy, fwd: dict, renorm: int = 1) -> dict:
    """Backward of layer_fwd_fp8, straight-through (each cast has derivative 1).

    Reading: dy is quantised per channel in 128-token groups in token order, and its
    dequantised value is what every later step sees.  The four backward GEMMs use the
    unquantised master weights, the saved H, the quantised-dequantised A and xp that
    the forward GEMMs consumed.
    """
    T = x.shape[0]
    dy_hat = dequant_colgroup128(*quant_colgroup128(dy))
    dYp = dispatch(dy_hat, fwd["perm"], k, row_mul=fwd["w"])
    dw = gate_grad(dy_hat, fwd["Y"], fwd["inv_perm"], T, k)
    dxp, dW1, dW2, dH = expert_ffn_bwd(fwd["xp"], fwd["H"], dYp, fwd["offsets"], W1, W2, A=fwd["A"])
    dx = combine(dxp, fwd["inv_perm"], None, T, k)
    dz = route_bwd(logits, fwd["idx"], fwd["w"], dw, renorm)
    return dict(dy_hat=dy_hat, dYp=dYp, dw=dw, dxp=dxp, dW1=dW1, dW2=dW2, dH=dH, dx=dx, dz=dz)


# --------------------------------------------------------------------------
# FP8 backward GEMMs: Section 7 "FP8 training" (per-token quantisation in the forward
# orientation, per-channel quantisation within 128-token groups in the backward one)
# --------------------------------------------------------------------------
def pow2_exponent(amax) -> np.ndarray:
    """Reading: a backward group scale is a power of two, 2^k with k the smallest integer for
    which amax * 2^-k <= 448 (k = 0 for amax = 0), clamped to -126 <= k <= 127.  Such scales
    are what block-scaled matrix hardware applies inside the contraction."""
    a = np.asarray(amax, F64)
    k = np.zeros(a.shape, dtype=np.int64)
    pos = a > 0
    if pos.any():
        mant, ex = np.frexp(a[pos] / E4M3_MAX)        # a/448 = mant * 2^ex, mant in [0.5, 1)
        k[pos] = np.where(mant == 0.5, ex - 1, ex)      # smallest k with a/448 <= 2^k
    return np.clip(k, -126, 127)


def token_groups(offsets, group: int = 128):
    """Groups of `group` consecutive rows inside each expert's segment (a group never spans two
    experts; the last group of a segment may be short).  Returns a list of (expert, lo, hi)."""
    out = []
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        for g0 in range(lo, hi, group):
            out.append((e, g0, min(g0 + group, hi)))
    return out


def quant_tokengroup_pow2(v, offsets, group: int = 128):
    """Per-channel quantisation within 128-token groups of the dispatched (expert-ordered) rows,
    power-of-two scales: codes uint8 [rows, cols] and exponents int64 [n_groups, cols]; the value
    of an element is decode(code) * 2^k of its (group, column).  The product v * 2^-k is exact in
    fp32, is clamped to +-448 and rounded to the nearest code (ties to even)."""
    v32 = _f32(v)
    rows, cols = v32.shape
    groups = token_groups(offsets, group)
    codes = np.zeros((rows, cols), dtype=np.uint8)
    exps = np.zeros((len(groups), cols), dtype=np.int64)
    for gi, (_, lo, hi) in enumerate(groups):
        blk = v32[lo:hi].astype(F64)
        k = pow2_exponent(np.abs(blk).max(axis=0))
        exps[gi] = k
        codes[lo:hi] = e4m3_encode(np.clip(blk * np.exp2(-k.astype(F64)), -E4M3_MAX, E4M3_MAX))
    return codes, exps


def dequant_tokengroup_pow2(codes, exps, offsets, group: int = 128) -> np.ndarray:
    out = np.zeros(codes.shape, F64)
    for gi, (_, lo, hi) in enumerate(token_groups(offsets, group)):
        out[lo:hi] = e4m3_decode(codes[lo:hi]) * np.exp2(exps[gi].astype(F64))
    return out


def quant_weights_transposed(W1, W2):
    """Second, transposed-orientation quantisation of the weights for the dgrad GEMMs: the
    contraction of dA = dY * W2 runs over W2's output channels, so the scale must be constant
    along them: one scale per input channel, i.e. per row of W2[e]^T ([f, d]); likewise per row
    of W1[e]^T ([d, 2f]).  Returns the dequantised transposes, float64."""
    E, two_f, d = W1.shape
    f = W2.shape[2]
    W1t = np.ascontiguousarray(np.transpose(_f32(W1), (0, 2, 1)))      # [E, d, 2f]
    W2t = np.ascontiguousarray(np.transpose(_f32(W2), (0, 2, 1)))      # [E, f, d]
    W1th = fake_quant_rows(W1t.reshape(E * d, two_f)).reshape(E, d, two_f)
    W2th = fake_quant_rows(W2t.reshape(E * f, d)).reshape(E, f, d)
    return W1th, W2th


def expert_ffn_bwd_fp8(xp_hat, H, dYp, A_hat, offsets, W1, W2, store=None):
    """The four backward GEMMs on E4M3 operands (float64 in between), straight-through casts.

        dA  = Qrow(dY) * Q(W2^T)^T          per-token dY, per-input-channel W2
        dH  = SwiGLU'(H, dA)                 on the saved pre-activations
        dxp = Qrow(dH) * Q(W1^T)^T          per-token dH, per-input-channel W1
        dW2[e] = Qg(dY_e)^T * Qg(A_e)        both per channel within 128-token groups (power-of-two
        dW1[e] = Qg(dH_e)^T * Qg(xp_e)       scales), A and xp being what the forward GEMMs consumed

    store = "bf16": dH is rounded to bfloat16 where it is handed to its two casts (see layer_fwd_fp8); dA is
    never kept, SwiGLU' reads it as summed.
    """
    E, two_f, d = W1.shape
    f = two_f // 2
    M = dYp.shape[0]
    W1th, W2th = quant_weights_transposed(W1, W2)
    dYr = fake_quant_rows(dYp)
    dA = np.zeros((M, f), F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        dA[lo:hi] = dYr[lo:hi] @ W2th[e].T
    dG, dU = swiglu_bwd(H[:, :f], H[:, f:], dA)
    dH = _stored(np.concatenate([dG, dU], axis=1), store)
    dHr = fake_quant_rows(dH)
    dxp = np.zeros((M, d), F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        dxp[lo:hi] = dHr[lo:hi] @ W1th[e].T
    dYg = dequant_tokengroup_pow2(*quant_tokengroup_pow2(dYp, offsets), offsets)
    dHg = dequant_tokengroup_pow2(*quant_tokengroup_pow2(dH, offsets), offsets)
    Ag = dequant_tokengroup_pow2(*quant_tokengroup_pow2(A_hat, offsets), offsets)
    Xg = dequant_tokengroup_pow2(*quant_tokengroup_pow2(xp_hat, offsets), offsets)
    dW1 = np.zeros((E, two_f, d), F64)
    dW2 = np.zeros((E, d, f), F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        dW2[e] = dYg[lo:hi].T @ Ag[lo:hi]
        dW1[e] = dHg[lo:hi].T @ Xg[lo:hi]
    return dict(dA=dA, dH=dH, dxp=dxp, dW1=dW1, dW2=dW2)


def layer_bwd_fp8_gemm(x, logits, W1, W2, k: int, dy, fwd: dict, renorm: int = 1, store=None) -> dict:
    """Backward of layer_fwd_fp8 with the backward GEMMs on E4M3 operands (expert_ffn_bwd_fp8);
    everything outside the expert FFN is as in layer_bwd_fp8.  store = "bf16" (to be paired with a forward
    made with the same setting): the weighted, dispatched dY and dH are rounded to bfloat16 before their casts."""
    T = x.shape[0]
    dy_hat = dequant_colgroup128(*quant_colgroup128(dy))
    dYp = _stored(dispatch(dy_hat, fwd["perm"], k, row_mul=fwd["w"]), store)
    dw = gate_grad(dy_hat, fwd["Y"], fwd["inv_perm"], T, k)
    g = expert_ffn_bwd_fp8(fwd["xp"], fwd["H"], dYp, fwd["A"], fwd["offsets"], W1, W2, store=store)
    dx = combine(g["dxp"], fwd["inv_perm"], None, T, k)
    dz = route_bwd(logits, fwd["idx"], fwd["w"], dw, renorm)
    return dict(dy_hat=dy_hat, dYp=dYp, dw=dw, dxp=g["dxp"], dW1=g["dW1"], dW2=g["dW2"], dH=g["dH"], dx=dx, dz=dz)


# --------------------------------------------------------------------------
# Load balance: Section 3.2 "Load balance" (auxiliary loss and token dropping, both per device:
# the experts placed on one GPU form a group, as in DeepSeek-V2)
# --------------------------------------------------------------------------
def softmax_all(logits) -> np.ndarray:
    """Affinity s[t,e]: softmax of a token's logits over all E experts."""
    z = np.asarray(logits, F64)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    return p / p.sum(axis=1, keepdims=True)


def balance_loss(logits, idx, n_groups: int, alpha: float):
    """Device-level balance loss.  Reading (the paper names DeepSeek-V2's scheme and gives no formula):
    with f_e = E/(k*T) * #{assignments to e}, P_e = mean_t s[t,e], experts e of group g = the E/n_groups
    consecutive experts on device g:  f'_g = mean_{e in g} f_e,  P'_g = sum_{e in g} P_e,
    loss = alpha * sum_g f'_g * P'_g.  Returns (loss, f' [n_groups], P' [n_groups])."""
    T, E = logits.shape
    k = idx.shape[1]
    per = E // n_groups
    counts = np.bincount(np.asarray(idx).reshape(-1), minlength=E).astype(F64)
    f = counts * E / (k * T)
    P = softmax_all(logits).mean(axis=0)
    fg = f.reshape(n_groups, per).mean(axis=1)
    Pg = P.reshape(n_groups, per).sum(axis=1)
    return float(alpha * np.sum(fg * Pg)), fg, Pg


def balance_loss_bwd(logits, idx, n_groups: int, alpha: float) -> np.ndarray:
    """d loss / d logits with the selection counts f treated as constants (they are piecewise constant):
    dz[t,c] = alpha/T * s[t,c] * (F_c - sum_e s[t,e] F_e),  F_e = f' of e's group."""
    T, E = logits.shape
    _, fg, _ = balance_loss(logits, idx, n_groups, 1.0)
    F = np.repeat(fg, E // n_groups)
    s = softmax_all(logits)
    return alpha / T * s * (F[None, :] - (s * F[None, :]).sum(axis=1, keepdims=True))


def affinity_scores(logits, idx) -> np.ndarray:
    """s[t, idx[t,j]] as float32 [T,k]: the precision in which the drop decision is taken."""
    s32 = softmax_all(logits).astype(np.float32)
    return np.take_along_axis(s32, np.asarray(idx, np.int64), axis=1)


def capacity_keep(score, idx, E: int, n_groups: int, capacity: int) -> np.ndarray:
    """Device-level token dropping.  Reading (after DeepSeek-V2, which the paper follows): each device keeps at
    most `capacity` assignments; when more arrive, those with the lowest affinity score[t,j] (float32) are
    dropped; among equal affinities the higher assignment id goes first.  Returns keep [T,k] bool."""
    T, k = idx.shape
    per = E // n_groups
    score = np.asarray(score, np.float32).reshape(-1)
    grp = (np.asarray(idx).reshape(-1) // per)
    keep = np.zeros(T * k, dtype=bool)
    for g in range(n_groups):
        a = np.flatnonzero(grp == g)
        order = np.lexsort((a, -score[a].astype(F64)))          # best first: score descending, id ascending
        keep[a[order[:capacity]]] = True
    return keep.reshape(T, k)


def route_capacity(logits, k: int, n_groups: int, capacity: int, renorm: int = 1, score=None) -> dict:
    """route() with device-level token dropping: a dropped assignment keeps its slot in idx / w (the weights are
    not renormalised) but gets no row (inv_perm = -1); counts, offsets and perm cover the kept assignments.
    `score` overrides the affinities the decision is taken from (a parity test passes the kernel's own)."""
    idx = topk_select(logits, k)
    w = gate_weights(logits, idx, renorm)
    E = logits.shape[1]
    if score is None:
        score = affinity_scores(logits, idx)
    keep = capacity_keep(score, idx, E, n_groups, capacity)
    e_of_a = idx.reshape(-1).astype(np.int64)
    kf = keep.reshape(-1)
    counts = np.array([np.count_nonzero((e_of_a == e) & kf) for e in range(E)], dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(counts)
    perm = np.concatenate([np.flatnonzero((e_of_a == e) & kf) for e in range(E)] + [np.zeros(0, np.int64)])
    inv_perm = np.full(e_of_a.size, -1, dtype=np.int64)
    inv_perm[perm] = np.arange(perm.size)
    return dict(idx=idx, w=w, keep=keep, score=np.asarray(score, np.float32).reshape(idx.shape), counts=counts, offsets=offsets.astype(np.int32), perm=perm.astype(np.int32),
                inv_perm=inv_perm.astype(np.int32))
