"""Pins for the Fractal Fade oracle (Sec. 3.2): brute force with exact rationals, closed forms on
distinct values, a library quantile, ties, sign handling, and the zero counts the paper's
tables imply."""
import math
import os
from fractions import Fraction

import numpy as np

import oracle
from paper_2511_21089_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_tables.txt")


def brute_quantile(values, s: Fraction) -> Fraction:
    """The linear-interpolation quantile in exact rational arithmetic."""
    v = sorted(Fraction(x) for x in values)
    p = s * (len(v) - 1)
    lo = p.numerator // p.denominator
    hi = min(lo + 1, len(v) - 1)
    return v[lo] + (p - lo) * (v[hi] - v[lo])


def test_quantile_and_mask_against_exact_rationals():
    rng = np.random.default_rng(0)
    for n, s in ((7, Fraction(1, 4)), (10, Fraction(3, 8)), (33, Fraction(27, 32)), (18, Fraction(9, 16)), (5, Fraction(1, 1))):   # s exact in binary
        w = rng.integers(-50, 50, size=n).astype(np.float32) / 8       # exact in float, with ties
        thr = brute_quantile([abs(float(x)) for x in w], s)
        assert Fraction(oracle.linear_quantile(np.abs(w), float(s))) == thr
        out, t, kept = oracle.fade_block(w, float(s))
        expect = [x if abs(Fraction(float(x))) > thr else 0.0 for x in w]
        assert np.array_equal(out, np.array(expect, np.float32))
        assert kept == sum(1 for x in w if abs(Fraction(float(x))) > thr)


def test_matches_library_quantile():
    rng = np.random.default_rng(1)
    a = np.abs(rng.standard_normal(1001))
    for s in (0.05625, 0.45, 0.84375, 0.9 * 7 / 8):
        assert math.isclose(oracle.linear_quantile(a, s), float(np.quantile(a, s, method="linear")), rel_tol=1e-14)


def test_kept_count_closed_form_on_distinct_values():
    rng = np.random.default_rng(2)
    w = rng.standard_normal((37, 41))                                  # distinct with probability 1
    n = w.size
    for i in range(1, 8):
        s = 0.9 * i / 8
        _, thr, kept = oracle.fade_block(w, s)
        assert kept == n - 1 - math.floor(s * (n - 1))
        assert (np.abs(w) > thr).sum() == kept


def test_ties_are_zeroed_by_the_strict_comparison():
    w = np.array([1.0, -2.0, 2.0, 2.0, 3.0], np.float32)
    out, thr, kept = oracle.fade_block(w, 0.25)                        # p = 1 -> threshold 2
    assert thr == 2.0 and kept == 1
    assert np.array_equal(out, np.array([0.0, -0.0, 0.0, 0.0, 3.0], np.float32))
    assert np.signbit(out[1]) and not np.signbit(out[2])               # multiplied by 0: sign kept


def test_schedule_untouched_parts_and_scale_invariance():
    L = synth.make_layer("qwen05b", 1, seed=3, d_model=64, d_inter=8 * 24)
    off = np.arange(9) * 24
    Wg, Wu, thr, kept = oracle.fractal_fade(L.W_gate, L.W_up, off)
    assert np.array_equal(Wg[:24], L.W_gate[:24]) and np.array_equal(Wu[:24], L.W_up[:24])   # branch 0 dense
    assert thr[0] == (None, None) and kept[0] == (24 * 64, 24 * 64)
    for b in range(1, 8):
        assert thr[b][0] is not None and thr[b][0] != thr[b][1]       # one threshold per projection
        frac = 1 - kept[b][0] / (24 * 64)
        assert 0.9 * b / 8 <= frac <= 0.9 * b / 8 + 0.02               # ties only add zeros
        # survivors are untouched, the rest are +-0
        blk, new = L.W_gate[b * 24:(b + 1) * 24], Wg[b * 24:(b + 1) * 24]
        assert np.all((new == blk) | ((new & 0x7FFF) == 0))
        assert np.all((new & 0x8000) == (blk & 0x8000))
    # scaling every weight by 4 (exact in bf16) scales the thresholds and keeps the pattern
    f = synth.bf16_bits_to_f32(L.W_gate) * 4
    Wg4, _, thr4, kept4 = oracle.fractal_fade(synth.f32_to_bf16_bits(f), L.W_up, off)
    assert [k[0] for k in kept4] == [k[0] for k in kept]
    assert all(math.isclose(t4[0], 4 * t[0]) for t4, t in zip(thr4[1:], thr[1:]))
    assert np.array_equal((Wg4 & 0x7FFF) == 0, (Wg & 0x7FFF) == 0)
    # explicit sparsity list: s = 0 leaves a branch alone, s = 1 clears it
    sp = [0, 1.0, 0, 0.5, 0, 0, 0, 0]
    Wg2, _, _, kept2 = oracle.fractal_fade(L.W_gate, L.W_up, off, sp)
    assert kept2[1][0] == 0 and np.all((Wg2[24:48] & 0x7FFF) == 0)
    assert np.array_equal(Wg2[48:72], L.W_gate[48:72])


def test_zero_counts_implied_by_the_papers_tables():
    """Tables 1-2 (MLPMoE-DiffSparsity, 16 branches per layer): zeros = total - nonzero.  On distinct
    values the operation zeroes floor(s (n - 1)) + 1 entries per block; ties at the threshold (the
    strict comparison) can only add to that.  Printed counts sit 0.2 % above the closed form."""
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        model, variant, total, nz = line.split()
        rows[(model, variant)] = (int(total), int(nz))
    for model, layers, dm, di in (("qwen05b", 24, 896, 4864), ("llama8b", 32, 4096, 14336)):
        total, nz = rows[(model, "MLPMoE-DiffSparsity")]
        n = (di // 16) * dm
        predicted = layers * sum(2 * (math.floor(oracle.fade_sparsity(i, 16) * (n - 1)) + 1) for i in range(1, 16))
        assert predicted <= total - nz <= predicted * 1.005
