"""Pins for oracle.round_to_bf16 (the rounding of the forward's result when it is stored as bf16):
hand-placed values and ties, the format's limits, and PyTorch's float32 -> bfloat16 conversion as an
independent library routine."""
import numpy as np

import oracle


def test_representable_values_and_hand_placed_ties():
    r = oracle.round_to_bf16
    for v in (0.0, 1.0, -1.0, 1.0 + 2.0 ** -7, 255.0, 2.0 ** -126, 3.0 * 2.0 ** -133, -2.0 ** 127 * 1.9921875):
        assert r(v) == v
    # halfway between 1 (fraction 0, even) and 1 + 2^-7 (fraction 1, odd): down to even
    assert r(1.0 + 2.0 ** -8) == 1.0
    # halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even): up to even
    assert r(1.0 + 3.0 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    # just above / below a tie
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -30) == 1.0 + 2.0 ** -7
    assert r(1.0 + 3.0 * 2.0 ** -8 - 2.0 ** -30) == 1.0 + 2.0 ** -7
    # carry into the next binade: 1.99609375 = 2 - 2^-8 is halfway between 2 - 2^-7 (odd) and 2 (even)
    assert r(2.0 - 2.0 ** -8) == 2.0
    assert r(-(2.0 - 2.0 ** -8)) == -2.0
    # sign of zero, infinities, overflow, subnormals
    assert np.signbit(r(-0.0)) and r(-0.0) == 0.0
    assert r(np.inf) == np.inf and r(-np.inf) == -np.inf and np.isnan(r(np.nan))
    big = 2.0 ** 127 * (2.0 - 2.0 ** -7)                 # largest bf16
    assert r(big) == big and r(big * (1 + 2.0 ** -10)) == big and r(2.0 ** 128 * 0.9999) == np.inf
    assert r(2.0 ** -134) == 0.0                          # half of the smallest subnormal: tie to even (0)
    assert r(1.5 * 2.0 ** -133) == 2.0 ** -132            # tie between 1 and 2 units: even


def test_spacing_and_error_bound():
    rng = np.random.default_rng(0)
    v = rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))
    q = oracle.round_to_bf16(v)
    assert np.all(np.abs(q - v) <= np.abs(v) * 2.0 ** -8)          # half a unit in the last place at most
    assert np.all(oracle.round_to_bf16(q) == q)                      # idempotent
    m, _ = np.frexp(np.abs(q))
    assert np.all(m * 256 == np.rint(m * 256))                       # 8 significant bits


def test_against_torch_conversion():
    import torch
    rng = np.random.default_rng(1)
    v = (rng.standard_normal(300000) * np.exp(rng.uniform(-30, 30, 300000))).astype(np.float32)
    bits = rng.integers(0, 2 ** 32, size=300000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    bits = bits[np.isfinite(bits)]
    for a in (v, bits):
        want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
        got = oracle.round_to_bf16(a.astype(np.float64))
        assert np.array_equal(got, want)
