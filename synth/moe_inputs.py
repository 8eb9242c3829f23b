"""Seeded synthetic inputs for one MoE FFN layer (shapes after the paper's Table 2).

This module only draws random tensors and rounds them to their storage type.  It
holds none of the layer's arithmetic: no gating, no permutation, no matmul of the
expert path.  Both the CPU oracle's tests and the HIP path's tests/bench feed on
the arrays made here, so the two sides always see the same bytes.

Recipe (one PCG64 stream per tensor, keyed by (seed, tensor_id); the expert weights use one
stream per expert, keyed by (seed, tensor_id, expert), so they can be drawn in parallel):
  tensor_id: x=0, W_r=1, W_g=2, W_u=3, W_d=4, dy=5, router-bias permutation=6
  draw float32 standard normals, multiply by the std, round once to the storage
  type (bf16 round-to-nearest-even, or keep fp32).
Weights are laid out "out, in":  W1 = [W_g ; W_u] as [E, 2f, d],  W2 = W_d as [E, d, f].
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

TENSOR_IDS = {"x": 0, "W_r": 1, "W_g": 2, "W_u": 3, "W_d": 4, "dy": 5, "bias_perm": 6}


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int            # tokens
    d: int            # d_model (the paper's h)
    E: int            # experts
    k: int            # experts per token
    f: int            # d_ff (the paper's h_ffn)
    dtype: str        # "f32" | "bf16" | "fp8"  (storage of activations/weights)
    w_std: float      # std of expert weights
    wr_std: float     # std of router weight
    bias: str = "none"    # "none" | "linear" | "zipf"
    bias_gamma: float = 0.0
    renorm: int = 1
    expert_range: tuple | None = None     # (e_lo, e_hi): one GPU's expert-parallel share; weights only for these experts

    @property
    def M(self) -> int:
        return self.T * self.k

    @property
    def local_experts(self) -> range:
        return range(self.E) if self.expert_range is None else range(*self.expert_range)

    def with_tokens(self, T: int) -> "MoEConfig":
        return replace(self, T=T)


CONFIGS = {
    # Tiny fp32 correctness config.
    "tiny": MoEConfig("tiny", T=256, d=128, E=8, k=2, f=256, dtype="f32",
                      w_std=1.0 / math.sqrt(128), wr_std=0.02),
    # Mixtral-8x7B layer shape (Table 2: h=4096, h_ffn=14336, 8 experts, top-2).
    "mixtral": MoEConfig("mixtral", T=8192, d=4096, E=8, k=2, f=14336, dtype="bf16",
                         w_std=0.02, wr_std=0.02),
    # DeepSeekMoE-like fine-grained experts (Table 2: h=2048, h_ffn=1408, 64 experts).
    "finegrained": MoEConfig("finegrained", T=16384, d=2048, E=64, k=8, f=1408, dtype="bf16",
                             w_std=0.02, wr_std=1.0 / math.sqrt(2048), bias="linear",
                             bias_gamma=0.17),
    # Skewed routing stress: Zipf-ranked expert bias.
    "skewed": MoEConfig("skewed", T=16384, d=4096, E=32, k=4, f=2048, dtype="bf16",
                        w_std=0.02, wr_std=1.0 / math.sqrt(4096), bias="zipf",
                        bias_gamma=1.2),
    # One GPU's expert-parallel share of the paper's Internal-352B layer (Table 2: h=4096, h_ffn=14336, 32 experts,
    # top-3; SP8+EP8 inside a node): the 8 x 1024 all-gathered tokens of one 8192-token sequence, 4 of the 32 experts local.
    "ep352b_share": MoEConfig("ep352b_share", T=8192, d=4096, E=32, k=3, f=14336, dtype="bf16",
                              w_std=0.02, wr_std=1.0 / math.sqrt(4096), expert_range=(8, 12)),
    # Mixtral shapes with fp8 (e4m3) dispatched activations / returned outputs.
    "mixtral_fp8": MoEConfig("mixtral_fp8", T=8192, d=4096, E=8, k=2, f=14336, dtype="fp8",
                             w_std=0.02, wr_std=0.02),
}


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(key, shape, std: float, storage: str, out=None) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(list(key)))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if storage != "f32":
        a = bf16_round(a)
    if out is not None:
        out[...] = a
        return out
    return a


def router_bias(cfg: MoEConfig, seed: int = 0) -> np.ndarray:
    """Fixed per-expert logit bias that shapes the load histogram (float32 [E])."""
    if cfg.bias == "none":
        return np.zeros(cfg.E, dtype=np.float32)
    rng = np.random.Generator(np.random.PCG64([seed, TENSOR_IDS["bias_perm"]]))
    pi = rng.permutation(cfg.E)
    if cfg.bias == "linear":
        u = np.linspace(1.0, -1.0, cfg.E)
        return (cfg.bias_gamma * u[pi]).astype(np.float32)
    if cfg.bias == "zipf":
        rank = 1.0 + pi
        return (-cfg.bias_gamma * np.log(rank)).astype(np.float32)
    raise ValueError(cfg.bias)


def make_inputs(cfg: MoEConfig, seed: int = 0, with_weights: bool = True) -> dict:
    """All tensors of one layer as float32 numpy arrays holding storage-rounded values."""
    st = "f32" if cfg.dtype == "f32" else "bf16"
    out = {
        "x": _normal((seed, TENSOR_IDS["x"]), (cfg.T, cfg.d), 1.0, st),
        "dy": _normal((seed, TENSOR_IDS["dy"]), (cfg.T, cfg.d), 1.0, st),
        "W_r": _normal((seed, TENSOR_IDS["W_r"]), (cfg.d, cfg.E), cfg.wr_std, st),
        "bias": router_bias(cfg, seed),
    }
    if with_weights:
        # with an expert range, W1 / W2 hold the local experts only (index 0 = expert e_lo), drawn from the same
        # per-expert streams as in the full layer
        local = cfg.local_experts
        w1 = np.empty((len(local), 2 * cfg.f, cfg.d), dtype=np.float32)
        w2 = np.empty((len(local), cfg.d, cfg.f), dtype=np.float32)
        jobs = []
        for i, e in enumerate(local):
            jobs.append(((seed, TENSOR_IDS["W_g"], e), (cfg.f, cfg.d), w1[i, :cfg.f, :]))
            jobs.append(((seed, TENSOR_IDS["W_u"], e), (cfg.f, cfg.d), w1[i, cfg.f:, :]))
            jobs.append(((seed, TENSOR_IDS["W_d"], e), (cfg.d, cfg.f), w2[i]))
        with ThreadPoolExecutor(max_workers=8) as pool:
            list(pool.map(lambda j: _normal(j[0], j[1], cfg.w_std, st, out=j[2]), jobs))
        out["W1"], out["W2"] = w1, w2
    return out


def random_logits(T: int, E: int, seed: int = 0, quantum: float | None = None) -> np.ndarray:
    """Float32 logits for routing tests; `quantum` snaps them to a coarse grid so ties abound."""
    rng = np.random.Generator(np.random.PCG64([seed, 101]))
    z = rng.standard_normal(size=(T, E), dtype=np.float32)
    if quantum is not None:
        z = (np.round(z / quantum) * quantum).astype(np.float32)
    return z
