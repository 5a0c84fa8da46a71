"""Oracle for Fractal Fade weight preparation (Sec. 3.2) -- test infrastructure only.

The operation, restated from Sec. 3.2 and the description of its implementation in Sec. 4:
for every branch i > 0 of a layer with B branches, with sparsity ratio s_i = 0.9 i / B, and
separately for the branch's block of W_gate and of W_up (W_down is left alone), take the
quantile of the absolute values of the block at fraction s_i (the linear-interpolation quantile:
position p = s (n - 1) in the ascending order statistics, value interpolated between the two
neighbours) and zero every entry whose absolute value is not strictly greater than it.

This file is that definition written out with numpy in double precision; nothing here is shared
with the GPU library.  Readings taken where the text is silent:
  * a branch whose sparsity is 0 (branch 0, or any branch given s = 0) is not touched at all;
  * an entry is "zeroed" by multiplying it by 0, so it keeps its sign (-0.0 stays negative);
  * bf16 storage: absolute values are taken on the stored values (exact in double).
"""
from __future__ import annotations

import numpy as np


def _to_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:                      # bf16 bit patterns
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def linear_quantile(values: np.ndarray, s: float) -> float:
    """Linear-interpolation quantile of a 1-D array at fraction s in [0, 1]."""
    v = np.sort(np.asarray(values, dtype=np.float64).ravel())
    p = s * (v.size - 1)
    lo = int(np.floor(p))
    hi = min(lo + 1, v.size - 1)
    return float(v[lo] + (p - lo) * (v[hi] - v[lo]))


def fade_block(block: np.ndarray, s: float):
    """One projection block of one branch.  Returns (new block in the input's storage, threshold, kept count)."""
    if s <= 0.0 or block.size == 0:
        return block.copy(), None, int(block.size)
    a = np.abs(_to_f64(block))
    thr = linear_quantile(a, s)
    keep = a > thr
    out = block.copy()
    if block.dtype == np.uint16:
        out[~keep] &= np.uint16(0x8000)           # +-0: the product of the stored value and 0
    else:
        out[~keep] = out[~keep] * block.dtype.type(0)
    return out, thr, int(keep.sum())


def fractal_fade(W_gate: np.ndarray, W_up: np.ndarray, branch_offsets, sparsity=None):
    """Fades W_gate and W_up ([d_inter, d_model], a branch = a block of rows) branch by branch.

    sparsity: one ratio per branch; None = the schedule of Sec. 3.2, s_i = 0.9 i / B.
    Returns (W_gate', W_up', thresholds[B][2] (None where untouched), kept[B][2]).
    """
    off = [int(o) for o in branch_offsets]
    B = len(off) - 1
    if sparsity is None:
        sparsity = [0.9 * i / B for i in range(B)]
    Wg, Wu = W_gate.copy(), W_up.copy()
    thr, kept = [], []
    for b in range(B):
        r0, r1 = off[b], off[b + 1]
        g, tg, kg = fade_block(W_gate[r0:r1], float(sparsity[b]))
        u, tu, ku = fade_block(W_up[r0:r1], float(sparsity[b]))
        Wg[r0:r1], Wu[r0:r1] = g, u
        thr.append((tg, tu))
        kept.append((kg, ku))
    return Wg, Wu, thr, kept


def neuron_scores(W_gate: np.ndarray, W_up: np.ndarray) -> np.ndarray:
    """Score of every intermediate neuron for the structured form of the fade: the squared Euclidean
    norm of its W_gate row and its W_up row together, in double precision."""
    g = _to_f64(W_gate)
    u = _to_f64(W_up)
    return (g * g).sum(axis=1) + (u * u).sum(axis=1)


def fade_neurons(W_gate: np.ndarray, W_up: np.ndarray, branch_offsets, keep_count):
    """Structured form of the differential sparsity of Sec. 3.2: instead of zeroing single weights,
    branch b keeps keep_count[b] whole neurons and drops the rest (the benchmark layer with
    variable branch widths is of this kind; the paper itself only defines the element-wise form, so
    the ranking rule is a reading: largest score first, equal scores by lower index).

    Returns (neuron_keep [d_inter] uint8, scores [d_inter] float64).  Written as the definition:
    per branch, a stable sort of the scores in descending order, the first keep_count[b] survive."""
    off = np.asarray(branch_offsets, dtype=np.int64)
    scores = neuron_scores(W_gate, W_up)
    keep = np.zeros(scores.shape[0], dtype=np.uint8)
    for b in range(off.size - 1):
        lo, hi = int(off[b]), int(off[b + 1])
        k = int(keep_count[b])
        if not 0 <= k <= hi - lo:
            raise ValueError("keep_count[%d] outside [0, d_b]" % b)
        order = np.argsort(-scores[lo:hi], kind="stable")      # descending, ties by lower index
        keep[lo + order[:k]] = 1
    return keep, scores
