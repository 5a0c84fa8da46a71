"""Oracle for the host-side transforms around the forward (test infrastructure).

Plain numpy / Python restatements of:
  * the contiguous partition of the intermediate dimension (Sec. 3.1),
  * the scalar gates alpha_b, initialised to 1 (Sec. 3.1),
  * Compensated Branch Pruning, alpha_b = sqrt(B/K) for b < K else 0 (Sec. 3.3),
  * the Fractal Fade sparsity schedule s_i = 0.9 i / B (Sec. 3.2),
  * neuron removal with compaction (structured reading of Sec. 3.2): dropping
    neuron j deletes row j of W_gate and W_up and column j of W_down.
Nothing here is imported by the GPU library or its binding.
"""
from __future__ import annotations

import math

import numpy as np


def split_sizes(d_inter: int, B: int) -> list:
    """Widths d_b of B contiguous slices with sum d_b = d_inter (Sec. 3.1).

    The paper leaves the remainder rule open; reading taken: the first
    d_inter mod B branches are one neuron wider.
    """
    base, rem = divmod(d_inter, B)
    return [base + (1 if b < rem else 0) for b in range(B)]


def compensated_alpha(B: int, K: int) -> list:
    """alpha_b of Sec. 3.3: sqrt(B/K) for the first K branches, 0 for the rest."""
    return [math.sqrt(B / K) if b < K else 0.0 for b in range(B)]


def fade_sparsity(i: int, B: int) -> float:
    """Sparsity ratio of branch i (0-based, branch 0 dense): s_i = 0.9 i / B  (Sec. 3.2)."""
    return 0.9 * i / B


def slice_plan(d_inter, B, K_keep=0, neuron_keep=None, pad_to=1, pad_rows_to=1):
    """Reference for the library's slicing calls.

    Returns (offsets[B+1], alpha[B], mask[B], gather) where gather lists, for
    every row of the compacted layer, the source neuron index or -1 for a
    zero padding row that rounds a branch up to a multiple of pad_to; the row
    count of the whole layer is then rounded up to a multiple of pad_rows_to
    with more zero rows at the end of the last branch.  (Padding is a storage
    convenience of this implementation, not part of the method: a zero gate/up
    row with a zero down column adds exactly nothing to the sum of Sec. 3.1.)
    """
    sizes = split_sizes(d_inter, B)
    if K_keep and 0 < K_keep < B:
        alpha = compensated_alpha(B, K_keep)
        mask = [1 if b < K_keep else 0 for b in range(B)]
    else:
        alpha = [1.0] * B
        mask = [1] * B
    offsets = [0]
    gather = []
    start = 0
    for b in range(B):
        idx = list(range(start, start + sizes[b]))
        if neuron_keep is not None:
            idx = [j for j in idx if neuron_keep[j]]
        n = len(idx)
        padded = (n + pad_to - 1) // pad_to * pad_to
        gather.extend(idx + [-1] * (padded - n))
        offsets.append(offsets[-1] + padded)
        start += sizes[b]
    extra = (-offsets[-1]) % pad_rows_to
    gather.extend([-1] * extra)
    offsets[-1] += extra
    return (np.asarray(offsets, dtype=np.int32), np.asarray(alpha, dtype=np.float32),
            np.asarray(mask, dtype=np.uint8), np.asarray(gather, dtype=np.int32))


def compact_layer(W_gate, W_up, W_down, gather):
    """Apply a gather list: rows of W_gate/W_up and columns of W_down; -1 gives zeros."""
    gather = np.asarray(gather)
    safe = np.where(gather >= 0, gather, 0)
    Wg = np.ascontiguousarray(W_gate[safe])
    Wu = np.ascontiguousarray(W_up[safe])
    Wd = np.ascontiguousarray(W_down[:, safe])
    pad = gather < 0
    Wg[pad] = 0
    Wu[pad] = 0
    Wd[:, pad] = 0
    return Wg, Wu, Wd
