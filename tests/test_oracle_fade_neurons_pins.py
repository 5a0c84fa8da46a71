"""Pins for oracle.fade_neurons (structured form of the fade: whole neurons ranked by the squared norm of
their gate and up rows): hand-made cases, brute force by pairwise comparison, invariants, and the
equivalence with removing the dropped neurons from the forward."""
import math

import numpy as np

import oracle
from paper_2511_21089_amd import synth


def test_hand_made_case_with_ties():
    # scores: gate row squared + up row squared
    Wg = np.array([[3, 0], [0, 1], [1, 1], [2, 0], [0, 0], [1, 0]], np.float32)
    Wu = np.array([[0, 4], [1, 0], [1, 1], [0, 1], [0, 0], [0, 2]], np.float32)
    off = np.array([0, 4, 6], np.int32)
    keep, sc = oracle.fade_neurons(Wg, Wu, off, [2, 1])
    assert list(sc) == [25.0, 2.0, 4.0, 5.0, 0.0, 5.0]
    assert list(keep) == [1, 0, 0, 1, 0, 1]                  # branch 0: 25 and 5; branch 1: 5
    # equal scores: the lower index wins
    Wg = np.array([[1, 2], [2, 1], [1, 2], [0, 0]], np.float32)
    Wu = np.zeros((4, 2), np.float32)
    for k, want in ((0, [0, 0, 0, 0]), (1, [1, 0, 0, 0]), (2, [1, 1, 0, 0]), (3, [1, 1, 1, 0]), (4, [1, 1, 1, 1])):
        keep, _ = oracle.fade_neurons(Wg, Wu, np.array([0, 4], np.int32), [k])
        assert list(keep) == want


def test_scores_in_closed_form_and_with_fsum():
    rng = np.random.default_rng(0)
    Wg = rng.standard_normal((7, 33)).astype(np.float32)
    Wu = rng.standard_normal((7, 33)).astype(np.float32)
    sc = oracle.neuron_scores(Wg, Wu)
    for j in range(7):
        want = math.fsum(float(v) ** 2 for v in Wg[j]) + math.fsum(float(v) ** 2 for v in Wu[j])
        assert abs(sc[j] - want) <= 1e-12 * want
    # bf16 storage is widened exactly: 1.5 and -0.25 are representable
    bits = np.array([[0x3FC0, 0xBE80]], np.uint16)
    assert oracle.neuron_scores(bits, bits)[0] == 2 * (1.5 ** 2 + 0.25 ** 2)


def test_brute_force_ranking_and_invariants():
    rng = np.random.default_rng(1)
    d_model, widths = 16, [5, 0, 9, 1, 12]
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    Wg = rng.integers(-3, 4, size=(off[-1], d_model)).astype(np.float32)      # small integers: many exact ties
    Wu = rng.integers(-3, 4, size=(off[-1], d_model)).astype(np.float32)
    counts = [3, 0, 4, 1, 7]
    keep, sc = oracle.fade_neurons(Wg, Wu, off, counts)
    for b, k in enumerate(counts):
        lo, hi = off[b], off[b + 1]
        assert keep[lo:hi].sum() == k
        for j in range(lo, hi):
            # rank by pairwise comparison: how many neurons of the branch come before j
            rank = sum(1 for i in range(lo, hi) if sc[i] > sc[j] or (sc[i] == sc[j] and i < j))
            assert keep[j] == (1 if rank < k else 0)
    # permuting the columns (the model dimension) changes nothing
    perm = rng.permutation(d_model)
    keep2, _ = oracle.fade_neurons(Wg[:, perm], Wu[:, perm], off, counts)
    assert np.array_equal(keep, keep2)
    # keeping everything / nothing
    assert oracle.fade_neurons(Wg, Wu, off, widths)[0].all()
    assert not oracle.fade_neurons(Wg, Wu, off, [0] * 5)[0].any()


def test_kept_set_feeds_the_slicing_and_the_forward():
    """neuron_keep -> slice_plan -> compact_layer gives the same output as zeroing the dropped neurons' up rows."""
    L = synth.make_layer("tiny_f32", 9, seed=5)
    off = np.array([0, 64, 128, 192, 256], np.int32)
    keep, _ = oracle.fade_neurons(L.W_gate, L.W_up, off, [64, 40, 17, 0])
    offc, alpha, mask, gather = oracle.slice_plan(256, 4, 0, keep, 1)
    assert list(np.diff(offc)) == [64, 40, 17, 0]
    Wg, Wu, Wd = oracle.compact_layer(L.W_gate, L.W_up, L.W_down, gather)
    got = oracle.mlpmoe_forward(L.x, Wg, Wu, Wd, offc, alpha, mask)
    Wu0 = L.W_up.copy()
    Wu0[keep == 0] = 0
    ref = oracle.mlpmoe_forward(L.x, L.W_gate, Wu0, L.W_down, off, np.ones(4, np.float32), np.ones(4, np.uint8))
    assert oracle.rel_max_err(got, ref) <= 1e-12
