"""Seeded synthetic inputs for the branched SwiGLU MLP (MLPMoE, Sec. 3.1).

This module only draws random numbers and converts storage formats.  It holds
none of the method's arithmetic (no slicing rule, no alpha rule, no forward),
so that both the CPU oracle's tests and the HIP path's tests can share it.

The arrays stand in for the MLP weights of the two models of Sec. 5
(Qwen2.5-0.5B-Instruct, DeepSeek-R1-Distill-Llama-8B): only their layer shapes
are used, values are N(0, 0.02^2) weights and N(0, 1) activations.

Layouts (row-major):
    x       [T, d_model]
    W_gate  [d_inter, d_model]     one row per intermediate neuron
    W_up    [d_inter, d_model]
    W_down  [d_model, d_inter]     one column per intermediate neuron
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


# --------------------------------------------------------------------------
# storage-format helpers (bf16 is kept as its uint16 bit pattern)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns.

    Inputs here are finite, so no NaN handling is needed.
    """
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# workload table: the five layer configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    d_model: int
    d_inter: int
    B: int
    dtype: str                      # "f32" or "bf16" (storage of x and W)
    alpha_range: Optional[tuple]    # None -> all ones
    n_inactive: int = 0             # branches switched off (seeded choice)
    fade: bool = False              # per-branch neuron removal, keep 1-0.4*b/(B-1)
    T_list: tuple = ()


WORKLOADS = {
    # tiny fp32 identity case: branched sum must equal the dense MLP
    "tiny_f32": Workload("tiny_f32", 64, 256, 4, "f32", None, T_list=(32,)),
    # Qwen2.5-0.5B-shaped layer, 8 equal branches of 608
    "qwen05b": Workload("qwen05b", 896, 4864, 8, "bf16", (0.9, 1.1), T_list=(2048, 1)),
    # same shape, 2 of 8 branches pruned, survivors rescaled
    "qwen05b_pruned": Workload("qwen05b_pruned", 896, 4864, 8, "bf16", (1.0, 1.2),
                               n_inactive=2, T_list=(2048, 1, 8, 16)),
    # Llama-8B-shaped layer, 16 equal branches of 896
    "llama8b": Workload("llama8b", 4096, 14336, 16, "bf16", (0.9, 1.1), T_list=(1, 16, 512, 4096)),
    # same shape with differential per-branch neuron sparsity
    "llama8b_fade": Workload("llama8b_fade", 4096, 14336, 16, "bf16", (0.9, 1.2),
                             fade=True, T_list=(1, 4096)),
}


@dataclass
class LayerInputs:
    """One synthetic layer.  bf16 arrays are uint16 bit patterns."""
    workload: Workload
    T: int
    x: np.ndarray
    W_gate: np.ndarray
    W_up: np.ndarray
    W_down: np.ndarray
    alpha_draw: np.ndarray          # [B] fp32, the per-branch scalar gates
    inactive: np.ndarray            # sorted indices of switched-off branches
    neuron_keep: Optional[np.ndarray] = None   # [d_inter] uint8, None if no neuron removal
    seed: int = 0
    extra: dict = field(default_factory=dict)

    def as_f32(self, name: str) -> np.ndarray:
        a = getattr(self, name)
        return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


def fade_keep_counts(d_b: int, B: int) -> list:
    """Kept-neuron count per branch for the fade workload: round(d_b*(1-0.4*b/(B-1)))."""
    return [int(np.floor(d_b * (1.0 - 0.4 * b / (B - 1)) + 0.5)) for b in range(B)]


def make_layer(workload: str | Workload, T: int, seed: int = 0, *,
               d_model: int | None = None, d_inter: int | None = None, B: int | None = None,
               dtype: str | None = None) -> LayerInputs:
    """Draw one layer.  Shape overrides let tests shrink a workload but keep its recipe."""
    w = WORKLOADS[workload] if isinstance(workload, str) else workload
    if d_model or d_inter or B or dtype:
        w = Workload(w.name, d_model or w.d_model, d_inter or w.d_inter, B or w.B,
                     dtype or w.dtype, w.alpha_range, w.n_inactive, w.fade, w.T_list)
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((T, w.d_model), dtype=np.float32)
    Wg = rng.standard_normal((w.d_inter, w.d_model), dtype=np.float32) * np.float32(0.02)
    Wu = rng.standard_normal((w.d_inter, w.d_model), dtype=np.float32) * np.float32(0.02)
    Wd = rng.standard_normal((w.d_model, w.d_inter), dtype=np.float32) * np.float32(0.02)
    if w.alpha_range is None:
        alpha = np.ones(w.B, dtype=np.float32)
    else:
        alpha = rng.uniform(w.alpha_range[0], w.alpha_range[1], size=w.B).astype(np.float32)
    inactive = np.sort(rng.choice(w.B, size=w.n_inactive, replace=False)).astype(np.int64)
    keep = None
    if w.fade:
        # equal contiguous branch ranges before removal; uniform choice of kept neurons
        assert w.d_inter % w.B == 0
        d_b = w.d_inter // w.B
        keep = np.zeros(w.d_inter, dtype=np.uint8)
        for b, k in enumerate(fade_keep_counts(d_b, w.B)):
            idx = rng.choice(d_b, size=k, replace=False)
            keep[b * d_b + idx] = 1
    if w.dtype == "bf16":
        x, Wg, Wu, Wd = (f32_to_bf16_bits(a) for a in (x, Wg, Wu, Wd))
    return LayerInputs(w, T, x, Wg, Wu, Wd, alpha, inactive, keep, seed)


def random_layer(rng: np.random.Generator, T: int, d_model: int, d_inter: int, dtype: str = "f32",
                 w_scale: float = 0.02):
    """Free-form small layer for unit tests: returns (x, W_gate, W_up, W_down)."""
    x = rng.standard_normal((T, d_model), dtype=np.float32)
    Wg = rng.standard_normal((d_inter, d_model), dtype=np.float32) * np.float32(w_scale)
    Wu = rng.standard_normal((d_inter, d_model), dtype=np.float32) * np.float32(w_scale)
    Wd = rng.standard_normal((d_model, d_inter), dtype=np.float32) * np.float32(w_scale)
    if dtype == "bf16":
        return tuple(f32_to_bf16_bits(a) for a in (x, Wg, Wu, Wd))
    return x, Wg, Wu, Wd
