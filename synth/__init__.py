"""Seeded synthetic inputs for one MoHGE layer call.

This module serves both the CPU oracle and the HIP library with byte-identical
inputs.  It holds no arithmetic of the method itself: it only names workloads
(shapes in the paper's notation: T tokens, hidden d, N_g groups of N experts,
per-group SwiGLU width d_ff, K_g groups and K_e experts per token) and draws
random tensors for them.

The tensors stand in for the activations and weights of a trained model, which
the paper's experiments use and which are not available here; only the shapes
of a layer call are taken over.

Draw order (fixed, one numpy Generator per workload, seeded with `seed`):
    x, W_G, W_E, then for each group g: W_gate[g], W_up[g], W_down[g],
    then (skewed workloads) one rank permutation per group, then (training) dy.
All draws are float32 standard normals; weights are scaled by 0.02 (a standard
deviation).  For bf16 workloads x, dy and the expert weights are rounded to
bf16 (round to nearest even) before either side sees them; the router weights
stay float32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

SELECT_GLOBAL = 0      # keep the K_e best experts over all selected groups (Eq. 5)
SELECT_PER_GROUP = 1   # keep K_e / K_g experts inside every selected group


@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    d: int
    n_groups: int
    experts_per_group: int
    d_ff: Tuple[int, ...]
    k_groups: int
    k_experts: int
    select_mode: int = SELECT_PER_GROUP
    dtype: str = "bf16"            # "bf16" or "f32": storage type of x and expert weights
    seed: int = 0
    skew_beta: float = 0.0         # > 0: Zipf(1.1)-shaped per-expert logit bias
    training: bool = False         # also draw the upstream gradient dy
    alpha_g: float = 1e-4          # coefficient ablation, appendix
    alpha_e: float = 2.5e-3
    eps: float = 1e-9

    @property
    def n_experts(self) -> int:
        return self.n_groups * self.experts_per_group

    @property
    def n_pairs(self) -> int:
        return self.T * self.k_experts

    def replace(self, **kw) -> "Workload":
        import dataclasses
        return dataclasses.replace(self, **kw)


# The five named configurations, then the paper's own layer shapes (appendix,
# architecture table: d=1024, N_g=8, K_g=3, K_e=6 chosen globally).
WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("tiny_f32", T=64, d=128, n_groups=3, experts_per_group=4,
                 d_ff=(64, 128, 256), k_groups=2, k_experts=2, dtype="f32", seed=0),
        Workload("mid_prefill", T=4096, d=2048, n_groups=3, experts_per_group=8,
                 d_ff=(512, 1024, 1536), k_groups=2, k_experts=4, seed=1),
        Workload("decode", T=32, d=4096, n_groups=4, experts_per_group=16,
                 d_ff=(768, 1024, 1536, 2048), k_groups=2, k_experts=4, seed=2),
        Workload("large_prefill_skewed", T=16384, d=4096, n_groups=4, experts_per_group=16,
                 d_ff=(768, 1024, 1536, 2048), k_groups=2, k_experts=4, seed=3,
                 skew_beta=2.0),
        Workload("training", T=8192, d=2048, n_groups=3, experts_per_group=8,
                 d_ff=(512, 1024, 1536), k_groups=2, k_experts=4, seed=4, training=True),
        Workload("paper_1b", T=4096, d=1024, n_groups=8, experts_per_group=4,
                 d_ff=(256, 320, 384, 512, 640, 768, 832, 896), k_groups=3, k_experts=6,
                 select_mode=SELECT_GLOBAL, seed=11),
        Workload("paper_3b", T=4096, d=1024, n_groups=8, experts_per_group=8,
                 d_ff=(384, 512, 640, 768, 896, 1024, 1152, 1280), k_groups=3, k_experts=6,
                 select_mode=SELECT_GLOBAL, seed=12),
        Workload("paper_14b", T=4096, d=1024, n_groups=8, experts_per_group=16,
                 d_ff=(640, 768, 896, 1024, 1152, 1280, 1408, 1536), k_groups=3, k_experts=6,
                 select_mode=SELECT_GLOBAL, seed=13),
    ]
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the 16-bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).reshape(-1)
    out = np.empty(bits.shape, dtype=np.uint16)
    step = 1 << 20                      # chunks that stay in cache: the large workloads have 10^9 weights
    for i in range(0, bits.size, step):
        b = bits[i:i + step]
        r = (b >> np.uint32(16)) & np.uint32(1)
        r += np.uint32(0x7FFF)
        r += b
        r >>= np.uint32(16)
        out[i:i + step] = r
    return out.reshape(a.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


class Tensor:
    """One generated tensor: float32 values, and the bf16 bit patterns when the
    workload stores it in bf16 (then `f32` holds exactly the widened values, made on first use:
    the device side only needs the bit patterns)."""

    def __init__(self, f32: Optional[np.ndarray] = None, bits: Optional[np.ndarray] = None):
        self._f32 = f32
        self.bits = bits

    @property
    def f32(self) -> np.ndarray:
        if self._f32 is None:
            self._f32 = bf16_bits_to_f32(self.bits)
        return self._f32

    @f32.setter
    def f32(self, value: np.ndarray) -> None:
        self._f32 = value


@dataclass
class LayerInputs:
    workload: Workload
    x: Tensor                       # [T, d]
    w_group: np.ndarray             # [N_g, d] float32
    w_expert: np.ndarray            # [N_e, d] float32, expert e = g*N + i
    w_gate: List[Tensor] = field(default_factory=list)   # per group [N, F_g, d]
    w_up: List[Tensor] = field(default_factory=list)     # per group [N, F_g, d]
    w_down: List[Tensor] = field(default_factory=list)   # per group [N, d, F_g]
    expert_logit_bias: Optional[np.ndarray] = None       # [N_e] float32 or None
    dy: Optional[Tensor] = None     # [T, d]


def _draw(rng: np.random.Generator, shape, scale: float, as_bf16: bool) -> Tensor:
    a = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    if as_bf16:
        return Tensor(None, f32_to_bf16_bits(a))
    return Tensor(a, None)


def generate(w: Workload) -> LayerInputs:
    """Draw every tensor of one layer call for workload `w` (see module docstring)."""
    rng = np.random.default_rng(w.seed)
    lowp = w.dtype == "bf16"
    N, d = w.experts_per_group, w.d
    x = _draw(rng, (w.T, d), 1.0, lowp)
    w_group = _draw(rng, (w.n_groups, d), 0.02, False).f32
    w_expert = _draw(rng, (w.n_experts, d), 0.02, False).f32
    out = LayerInputs(w, x, w_group, w_expert)
    for g in range(w.n_groups):
        F = w.d_ff[g]
        out.w_gate.append(_draw(rng, (N, F, d), 0.02, lowp))
        out.w_up.append(_draw(rng, (N, F, d), 0.02, lowp))
        out.w_down.append(_draw(rng, (N, d, F), 0.02, lowp))
    if w.skew_beta > 0.0:
        # Inside every group a random ranking rho in 1..N; the bias is beta times
        # the log of a Zipf(s = 1.1) mass function, log rho^-1.1.
        bias = np.empty((w.n_groups, N), dtype=np.float32)
        for g in range(w.n_groups):
            rho = rng.permutation(N).astype(np.float64) + 1.0
            bias[g] = (-w.skew_beta * 1.1 * np.log(rho)).astype(np.float32)
        out.expert_logit_bias = bias.reshape(-1)
    if w.training:
        out.dy = _draw(rng, (w.T, d), 1.0, lowp)
    return out
