"""Randomised sweep of small layer shapes on the GPU (hypothesis, derandomised so every run draws the same cases):
routing compared bit for bit and every tensor of the bf16 layer element-wise with the oracle.  The strategy reaches the
corners by construction: one expert, k = E, experts that get no token, every token on one expert, tied logits."""
import numpy as np
import pytest
import torch
from hypothesis import HealthCheck, Phase, given, settings
from hypothesis import strategies as st

from oracle import moe_oracle as O
from synth.moe_inputs import MoEConfig, make_inputs, random_logits
from tests.gpu_util import DEV, max_norm_err, to_dev, to_np

pytestmark = pytest.mark.gpu


@st.composite
def layer_cases(draw):
    E = draw(st.sampled_from([1, 2, 3, 5, 8, 12, 33, 64]))
    k = draw(st.sampled_from(sorted({1, min(2, E), min(3, E), min(8, E), min(E, 16)})))
    T = draw(st.integers(min_value=1, max_value=700))
    d = 16 * draw(st.integers(min_value=1, max_value=20))
    f = 16 * draw(st.integers(min_value=1, max_value=24))
    logit_kind = draw(st.sampled_from(["normal", "coarse", "tied", "one_expert", "empty_experts"]))
    renorm = draw(st.sampled_from([1, 1, 0]))
    fused = draw(st.booleans())
    seed = draw(st.integers(min_value=0, max_value=10 ** 6))
    return dict(T=T, d=d, E=E, k=k, f=f, logit_kind=logit_kind, renorm=renorm, fused=fused, seed=seed)


def make_logits(c):
    T, E = c["T"], c["E"]
    kind = c["logit_kind"]
    if kind == "normal":
        return random_logits(T, E, seed=c["seed"])
    if kind == "coarse":
        return random_logits(T, E, seed=c["seed"], quantum=0.5)
    if kind == "tied":
        return np.full((T, E), 0.25, dtype=np.float32)                    # every row all-equal: lowest ids win
    z = random_logits(T, E, seed=c["seed"], quantum=0.25)
    if kind == "one_expert":
        z[:, E // 2] += 50.0                                              # slot 0 of every token is the same expert
    else:
        z[:, ::2] -= 1e4                                                  # even experts get tokens only when k forces it
    return z


@settings(max_examples=120, deadline=None, derandomize=True, phases=[Phase.generate],
          suppress_health_check=list(HealthCheck))
@given(layer_cases())
def test_random_small_layers_match_the_oracle(c):
    from paper_2505_11432_amd import binding as B
    from paper_2505_11432_amd.layer import MoELayer
    print("case", c, flush=True)
    T, d, E, k, f = c["T"], c["d"], c["E"], c["k"], c["f"]
    cfg = MoEConfig("prop", T=T, d=d, E=E, k=k, f=f, dtype="bf16", w_std=1.0 / np.sqrt(d), wr_std=0.3, renorm=c["renorm"])
    inp = make_inputs(cfg, seed=c["seed"] % 1000)
    z = make_logits(c)
    td = torch.bfloat16
    layer = MoELayer(T, d, E, k, f, dtype=td, renorm=c["renorm"], fused=c["fused"])
    x, dy, wr = to_dev(inp["x"], td), to_dev(inp["dy"], td), to_dev(inp["W_r"].T, td)
    w1, w2 = to_dev(inp["W1"], td), to_dev(inp["W2"], td)
    layer.forward(x, wr, None, w1, w2, logits=to_dev(z))
    layer.backward(x, wr, w1, w2, dy, with_router=False)
    torch.cuda.synchronize()
    fwd = O.layer_fwd(inp["x"], z, inp["W1"], inp["W2"], k, c["renorm"])
    bwd = O.layer_bwd(inp["x"], z, inp["W1"], inp["W2"], k, inp["dy"], fwd, c["renorm"])
    for name, got in (("idx", layer.topk_idx), ("counts", layer.counts), ("offsets", layer.offsets),
                      ("perm", layer.perm), ("inv_perm", layer.inv_perm)):
        assert np.array_equal(to_np(got), fwd[name]), (name, c)
    assert int(fwd["counts"].sum()) == T * k
    assert np.allclose(to_np(layer.topk_w), fwd["w"], rtol=2e-6, atol=1e-7)
    # The gate-weight gradient is a dot product <dy[t], Y[r]> that can cancel to almost nothing, and in the smallest
    # shapes the whole tensor is one such number: its error (and that of d_logits, which is linear in it) is measured
    # against the natural scale of the dot products, max ||dy[t]|| * ||Y[r]||, not against the cancelled result.
    dot_scale = max(np.linalg.norm(inp["dy"], axis=1).max() * np.linalg.norm(fwd["Y"], axis=1).max(), 1e-30)
    errs = {"H": max_norm_err(to_np(layer.h_save), fwd["H"]), "y": max_norm_err(to_np(layer.y), fwd["y"]),
            "dw": float(np.abs(to_np(layer.d_topk_w) - bwd["dw"]).max() / max(np.abs(bwd["dw"]).max(), dot_scale)),
            "dx": max_norm_err(to_np(layer.dx), bwd["dx"]),
            "dz": float(np.abs(to_np(layer.d_logits) - bwd["dz"]).max() / max(np.abs(bwd["dz"]).max(), dot_scale))}
    dW1, dW2 = to_np(layer.d_w1), to_np(layer.d_w2)
    for e in range(E):
        if fwd["counts"][e] == 0:
            assert np.all(dW1[e] == 0) and np.all(dW2[e] == 0), (e, c)
    errs["dW1"] = max_norm_err(dW1, bwd["dW1"])
    errs["dW2"] = max_norm_err(dW2, bwd["dW2"])
    bad = {n: v for n, v in errs.items() if not v < 2e-2}
    assert not bad, (bad, c)
