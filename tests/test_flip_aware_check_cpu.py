"""The flip-aware bf16 parity check (tests/gpu_util.py) exercised on the CPU: it must accept a faithful fp32
evaluation of the bf16 pipeline (numpy float32, a different summation order than the oracle's) at any number
of active neurons, and reject planted mistakes.  The stand-in for the GPU here is numpy, never the HIP path."""
import numpy as np
import pytest

import oracle
from gpu_util import check_bf16_flip_aware, widen
from paper_2511_21089_amd import synth


def fp32_pipeline(x, Wg, Wu, Wd, off, alpha, mask):
    """alpha * SiLU(g) * u in float32 from float32 sums, one rounding to bf16, float32 down projection."""
    xw, Wgw, Wuw, Wdw = (widen(a) for a in (x, Wg, Wu, Wd))
    g = xw @ Wgw.T
    u = xw @ Wuw.T
    a = np.zeros(int(off[-1]), np.float32)
    act = np.zeros(int(off[-1]), bool)
    for b in range(len(alpha)):
        a[off[b]:off[b + 1]] = alpha[b]
        act[off[b]:off[b + 1]] = bool(mask[b])
    h = a * ((g / (np.float32(1) + np.exp(-g))) * u)
    Hb = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(h.astype(np.float32)))
    Hb = np.where(act, Hb, np.float32(np.nan))                   # inactive columns: never written
    out = np.where(act, Hb, np.float32(0)).astype(np.float32) @ Wdw.T
    return out, Hb.astype(np.float64)


def case(seed, T, d_model, widths, mask):
    rng = np.random.default_rng(seed)
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    x, Wg, Wu, Wd = synth.random_layer(rng, T, d_model, int(off[-1]), dtype="bf16", w_scale=0.08)
    alpha = rng.uniform(0.9, 1.2, size=len(widths)).astype(np.float32)
    return x, Wg, Wu, Wd, off, alpha, np.array(mask, np.uint8)


@pytest.mark.parametrize("widths,mask", [((8,), (1,)), ((40, 24), (1, 1)), ((64, 128, 192), (1, 0, 1)),
                                         ((512, 512, 512), (1, 1, 1))])
def test_accepts_a_faithful_fp32_evaluation(widths, mask):
    args = case(sum(widths), 96, 256, widths, mask)
    out, H = fp32_pipeline(*args)
    e_c, e_e, frac = check_bf16_flip_aware(out, H, *args, label=str(widths))
    assert frac < 0.02


def test_rejects_planted_mistakes():
    args = case(5, 64, 128, (64, 64), (1, 1))
    out, H = fp32_pipeline(*args)
    check_bf16_flip_aware(out, H, *args)
    # a stored h one bf16 unit off where the value is nowhere near a rounding boundary
    H2 = H.copy()
    t, j = np.unravel_index(np.argmax(np.abs(H)), H.shape)
    H2[t, j] *= 1.0 + 2.0 ** -7
    with pytest.raises(AssertionError, match="outside"):
        check_bf16_flip_aware(out, H2, *args)
    # an unwritten h (poison left in the workspace)
    H3 = H.copy()
    H3[3, 5] = np.nan
    with pytest.raises(AssertionError):
        check_bf16_flip_aware(out, H3, *args)
    # a neuron dropped from the down projection
    x, Wg, Wu, Wd, off, alpha, mask = args
    Hz = np.nan_to_num(H).astype(np.float32)
    Hz[:, 17] = 0
    with pytest.raises(AssertionError, match="down projection"):
        check_bf16_flip_aware(Hz @ widen(Wd).T, H, *args)
    # alpha applied twice
    with pytest.raises(AssertionError):
        check_bf16_flip_aware(out * alpha[0], H, *args)
    # W_down read transposed (square case so that shapes still match)
    sq = case(6, 32, 128, (128,), (1,))
    o2, H4 = fp32_pipeline(*sq)
    check_bf16_flip_aware(o2, H4, *sq)
    bad = np.nan_to_num(H4).astype(np.float32) @ widen(sq[3])
    with pytest.raises(AssertionError):
        check_bf16_flip_aware(bad, H4, *sq)


def test_routed_entries_are_masked():
    args = case(7, 48, 128, (32, 32, 64), (1, 1, 1))
    x, Wg, Wu, Wd, off, alpha, mask = args
    rng = np.random.default_rng(0)
    route = (rng.uniform(size=(48, 3)) < 0.6).astype(np.uint8)
    route[4] = 0
    _, H = fp32_pipeline(*args)
    take = np.zeros(H.shape, bool)
    for b in range(3):
        take[:, off[b]:off[b + 1]] = route[:, b:b + 1] != 0
    out = np.where(take, H, 0).astype(np.float32) @ widen(Wd).T
    Hp = np.where(take, H, np.nan)                                # whatever a token does not take may hold anything
    check_bf16_flip_aware(out, Hp, *args, route=route)
    assert not np.any(out[4])
