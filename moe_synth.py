"""Seeded synthetic inputs for the MoE-layer hot path.

This module only draws numbers and packs them into the storage formats both the
CPU oracle and the HIP library read (fp32, or bf16 bit patterns).  It holds none
of the method's arithmetic: no gating, no ordering, no expert math.

The five workloads follow the layer shapes the paper sweeps (Table 4: B, L, M,
H/M, f, ffn-type in {simple, Mixtral}) and its two real models (GPT-2 style
two-layer experts, Mixtral style three-matrix experts; Sec. 3.1 "Expert").
All values are synthetic: x ~ N(0, sx^2), every weight ~ N(0, 0.02^2)
(0.02 is a standard deviation), dy ~ N(0, sx^2).

Random numbers come from numpy's Philox counter-based bit generator; each
tensor has its own (seed, tensor-id) stream so any tensor (or any one expert's
slice of a weight) can be drawn without drawing the others.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np

# activation / dtype codes: same integers as the C header's enums (interface constants)
ACT_RELU, ACT_GELU_TANH, ACT_SWIGLU, ACT_GELU_ERF = 0, 1, 2, 3
DT_F32, DT_BF16 = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    N: int            # tokens = B*L
    M: int            # d_model
    E: int            # experts
    H: int            # expert hidden size
    k: int            # top-k
    f: float | None   # capacity factor; None = the paper's f=* (no dropping)
    act: int
    dtype: int
    renormalize: int  # 1: softmax over the kept top-k; 0: softmax over all E
    add_residual: int
    x_std: float
    bias: str         # "none" | "normal" | "zipf"
    seed: int

    @property
    def gated(self) -> bool:
        return self.act == ACT_SWIGLU


WORKLOADS = {
    # Tiny fp32 layer: 256 tokens, 4 two-layer ReLU experts, top-1, f=1.25, seed 0
    "tiny": Workload("tiny", 256, 64, 4, 128, 1, 1.25, ACT_RELU, DT_F32, 0, 0, 0.02, "none", 0),
    # GPT-2-small style: 8x1024 tokens, 16 two-layer GELU experts, top-2, f=1.2
    "gpt2": Workload("gpt2", 8192, 768, 16, 3072, 2, 1.2, ACT_GELU_TANH, DT_BF16, 0, 0, 1.0, "none", 2),
    # Mixtral style: 4x4096 tokens, 8 SwiGLU experts, top-2 renormalised, f=* (no drop)
    "mixtral": Workload("mixtral", 16384, 4096, 8, 14336, 2, None, ACT_SWIGLU, DT_BF16, 1, 0, 1.0, "none", 3),
    # Fine-grained: 64 small SwiGLU experts, top-6, f=1.5, N(0,1) gate bias (imbalanced loads)
    "finegrained": Workload("finegrained", 32768, 2048, 64, 1408, 6, 1.5, ACT_SWIGLU, DT_BF16, 0, 0, 1.0, "normal", 4),
    # Switch style: top-1, f=1.0, overflow dropped with residual passthrough, Zipf(1.1) gate bias
    "switch": Workload("switch", 65536, 2048, 32, 8192, 1, 1.0, ACT_GELU_TANH, DT_BF16, 0, 1, 1.0, "zipf", 5),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some sizes replaced (for small parity cases)."""
    return replace(w, **kw)


# ----------------------------------------------------------------------------- storage formats

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor (fp32 array, or uint16 bf16 bits) to fp64."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------- draws

_TENSOR_IDS = {"x": 1, "w_gate": 2, "b_gate": 3, "w1": 4, "w3": 5, "w2": 6, "dy": 7, "perm": 8, "sample": 9,
               "w_noise": 10, "noise": 11, "dtopk_w": 12, "w_proj": 13, "w_embed": 14}


def _rng(seed: int, tensor: str, part: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | _TENSOR_IDS[tensor], part]))


def _normal(seed: int, tensor: str, shape, std: float, part: int = 0) -> np.ndarray:
    g = _rng(seed, tensor, part)
    a = g.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    return a


def _store(a: np.ndarray, dtype: int) -> np.ndarray:
    return f32_to_bf16_bits(a) if dtype == DT_BF16 else a


def draw_x(w: Workload) -> np.ndarray:
    return _store(_normal(w.seed, "x", (w.N, w.M), w.x_std), w.dtype)


def draw_dy(w: Workload) -> np.ndarray:
    return _store(_normal(w.seed, "dy", (w.N, w.M), w.x_std), w.dtype)


def draw_w_gate(w: Workload) -> np.ndarray:
    return _store(_normal(w.seed, "w_gate", (w.M, w.E), 0.02), w.dtype)


def draw_w_noise(w: Workload) -> np.ndarray:
    """W_noise of the noisy gate, like W_g."""
    return _store(_normal(w.seed, "w_noise", (w.M, w.E), 0.02), w.dtype)


def draw_w_proj(w: Workload, d_proj: int) -> np.ndarray:
    """W_proj of the X-MoE gate, [M, d_proj], initialised like W_g."""
    return _store(_normal(w.seed, "w_proj", (w.M, d_proj), 0.02), w.dtype)


def draw_w_embed(w: Workload, d_proj: int) -> np.ndarray:
    """Expert embeddings of the X-MoE gate, [d_proj, E] (one per column)."""
    return _store(_normal(w.seed, "w_embed", (d_proj, w.E), 0.5), w.dtype)


def draw_noise(w: Workload) -> np.ndarray:
    """The standard-normal draws of the noisy gate, fp32 [N,E] (an input of the path)."""
    return _normal(w.seed, "noise", (w.N, w.E), 1.0)


def draw_dtopk_w(w: Workload) -> np.ndarray:
    """An upstream gradient for the gate weights, fp32 [N,k] (for gate-only backward checks)."""
    return _normal(w.seed, "dtopk_w", (w.N, w.k), 1.0)


def draw_b_gate(w: Workload):
    """Gate bias, always fp32 [E]; None when the workload has no skew."""
    if w.bias == "none":
        return None
    if w.bias == "normal":
        return _normal(w.seed, "b_gate", (w.E,), 1.0)
    if w.bias == "zipf":
        rank = _rng(w.seed, "perm").permutation(w.E) + 1
        return (-1.1 * np.log(rank.astype(np.float64))).astype(np.float32)
    raise ValueError(w.bias)


def draw_expert_weight(w: Workload, which: str, e: int) -> np.ndarray:
    """One expert's matrix: w1, w3 are [M, H]; w2 is [H, M] (the paper's shapes, Sec. 2.1)."""
    shape = (w.M, w.H) if which in ("w1", "w3") else (w.H, w.M)
    return _store(_normal(w.seed, which, shape, 0.02, part=e), w.dtype)


def draw_expert_weights(w: Workload, which: str) -> np.ndarray:
    """All experts' matrices stacked: [E, M, H] or [E, H, M]."""
    first = draw_expert_weight(w, which, 0)
    out = np.empty((w.E,) + first.shape, dtype=first.dtype)
    out[0] = first
    for e in range(1, w.E):
        out[e] = draw_expert_weight(w, which, e)
    return out


def draw_all(w: Workload) -> dict:
    d = {
        "x": draw_x(w), "w_gate": draw_w_gate(w), "b_gate": draw_b_gate(w),
        "w1": draw_expert_weights(w, "w1"), "w2": draw_expert_weights(w, "w2"),
        "w3": draw_expert_weights(w, "w3") if w.gated else None, "dy": draw_dy(w),
    }
    return d


def sample_indices(w: Workload, n: int, upper: int, part: int = 0) -> np.ndarray:
    """A seeded sorted sample of n distinct indices below `upper` (for sampled parity checks)."""
    n = min(n, upper)
    return np.sort(_rng(w.seed, "sample", part).choice(upper, size=n, replace=False))


def capacity_factor_text(w: Workload) -> str:
    return "*" if w.f is None else repr(w.f)
