"""Pins for the oracle's per-token routing: reductions to the unrouted forward, linearity over
branches, token independence, and a pure-Python brute force."""
import math

import numpy as np

import oracle


def layer(seed, T, dm, off):
    rng = np.random.default_rng(seed)
    di = off[-1]
    x = rng.standard_normal((T, dm)).astype(np.float32)
    Wg = (rng.standard_normal((di, dm)) * 0.2).astype(np.float32)
    Wu = (rng.standard_normal((di, dm)) * 0.2).astype(np.float32)
    Wd = (rng.standard_normal((dm, di)) * 0.2).astype(np.float32)
    alpha = rng.uniform(0.5, 1.5, size=len(off) - 1).astype(np.float32)
    return x, Wg, Wu, Wd, np.array(off, np.int32), alpha


def test_all_routed_and_none_routed():
    x, Wg, Wu, Wd, off, alpha = layer(0, 9, 12, [0, 5, 5, 11, 20])
    mask = np.array([1, 1, 0, 1], np.uint8)
    full = oracle.mlpmoe_forward(x, Wg, Wu, Wd, off, alpha, mask)
    ones = np.ones((9, 4), np.uint8)
    assert np.array_equal(oracle.mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, mask, ones), full)
    assert np.all(oracle.mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, mask, 0 * ones) == 0)
    # a route bit cannot switch a pruned branch back on
    only2 = np.zeros((9, 4), np.uint8)
    only2[:, 2] = 1
    assert np.all(oracle.mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, mask, only2) == 0)


def test_token_rows_follow_their_own_branch_sets():
    """Row t of the routed result == row t of the unrouted forward run with mask = route[t]."""
    x, Wg, Wu, Wd, off, alpha = layer(1, 7, 10, [0, 4, 9, 15])
    mask = np.ones(3, np.uint8)
    rng = np.random.default_rng(5)
    route = rng.integers(0, 2, size=(7, 3)).astype(np.uint8)
    route[3] = 0
    got = oracle.mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, mask, route, mode="contract")
    for t in range(7):
        ref = oracle.mlpmoe_forward(x[t:t + 1], Wg, Wu, Wd, off, alpha, route[t], mode="contract")
        assert np.array_equal(got[t], ref[0])
    assert np.all(got[3] == 0)


def test_sum_over_single_branch_routes():
    """The routed forward is additive over branches: route = sum of one-hot routes."""
    x, Wg, Wu, Wd, off, alpha = layer(2, 6, 8, [0, 3, 8, 10, 16])
    mask = np.ones(4, np.uint8)
    route = np.random.default_rng(9).integers(0, 2, size=(6, 4)).astype(np.uint8)
    total = oracle.mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, mask, route)
    parts = np.zeros_like(total)
    for b in range(4):
        r = np.zeros_like(route)
        r[:, b] = route[:, b]
        parts += oracle.mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, mask, r)
    assert np.allclose(total, parts, rtol=1e-13, atol=1e-15)


def test_brute_force_tiny():
    x, Wg, Wu, Wd, off, alpha = layer(3, 3, 4, [0, 2, 5])
    route = np.array([[1, 0], [0, 1], [1, 1]], np.uint8)
    got = oracle.mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, np.ones(2, np.uint8), route)
    for t in range(3):
        for m in range(4):
            terms = []
            for b in range(2):
                if not route[t, b]:
                    continue
                for j in range(off[b], off[b + 1]):
                    g = math.fsum(float(Wg[j, k]) * float(x[t, k]) for k in range(4))
                    u = math.fsum(float(Wu[j, k]) * float(x[t, k]) for k in range(4))
                    terms.append(float(alpha[b]) * float(Wd[m, j]) * (g / (1.0 + math.exp(-g))) * u)
            assert math.isclose(got[t, m], math.fsum(terms), rel_tol=1e-12, abs_tol=1e-15)
