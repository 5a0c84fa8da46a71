"""Pins of the oracle's gated-intermediate function and of the parity metric itself (CPU only)."""
import math

import numpy as np

import oracle
from paper_2511_21089_amd import synth


def small_layer(seed, T=6, d_model=24, widths=(8, 0, 16, 5)):
    rng = np.random.default_rng(seed)
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    x, Wg, Wu, Wd = synth.random_layer(rng, T, d_model, int(off[-1]), w_scale=0.3)
    alpha = rng.uniform(0.5, 1.5, size=len(widths)).astype(np.float32)
    return x, Wg, Wu, Wd, off, alpha


def test_rel_max_err_hand_computed():
    """max|got - ref| / rms(ref) on a 2 x 2 case worked by hand: ref = [[3, 4], [0, 0]] has
    rms = sqrt((9 + 16) / 4) = 2.5; got differs by 0.5 and by 1 -> 1 / 2.5 = 0.4."""
    ref = np.array([[3.0, 4.0], [0.0, 0.0]])
    got = np.array([[3.5, 4.0], [0.0, -1.0]])
    assert oracle.rel_max_err(got, ref) == 0.4
    assert oracle.rel_max_err(ref, ref) == 0.0
    # the denominator is the rms of the REFERENCE (not of got, not the max, not the sum)
    assert oracle.rel_max_err(10 * ref, ref) == (9 * 4.0) / 2.5
    # a zero reference: 0 if equal, inf otherwise
    z = np.zeros((2, 2))
    assert oracle.rel_max_err(z, z) == 0.0 and oracle.rel_max_err(z + 1, z) == float("inf")
    assert oracle.rel_max_err(np.zeros((0, 3)), np.zeros((0, 3))) == 0.0


def test_hidden_times_down_is_the_forward():
    """Sec. 3.1: MLPMoE(x) = sum_b alpha_b W_down^(b) h^(b): the forward is the library fp64 product of the
    gated intermediate with W_down^T, in both modes (bit for bit in contract mode up to summation order)."""
    x, Wg, Wu, Wd, off, alpha = small_layer(1)
    for mask in ([1, 1, 1, 1], [1, 1, 0, 1], [0, 0, 1, 0]):
        mask = np.array(mask, np.uint8)
        for mode in ("exact", "contract"):
            h = oracle.mlpmoe_hidden(x, Wg, Wu, off, alpha, mask, mode)
            ref = oracle.mlpmoe_forward(x, Wg, Wu, Wd, off, alpha, mask, mode)
            assert np.allclose(h @ Wd.astype(np.float64).T, ref, rtol=1e-13, atol=1e-15)
            # neurons of inactive branches contribute nothing
            for b in range(4):
                if not mask[b]:
                    assert not np.any(h[:, off[b]:off[b + 1]])


def test_hidden_brute_force_and_details():
    """Pure-Python evaluation of alpha_b * SiLU(<Wg_j, x>) * <Wu_j, x> with math.fsum, and the detail outputs."""
    x, Wg, Wu, Wd, off, alpha = small_layer(2, T=3, d_model=10, widths=(3, 4))
    mask = np.array([1, 1], np.uint8)
    h, g, u, ag, au = oracle.mlpmoe_hidden(x, Wg, Wu, off, alpha, mask, "exact", details=True)
    for t in range(3):
        for j in range(7):
            b = 0 if j < 3 else 1
            gg = math.fsum(float(x[t, k]) * float(Wg[j, k]) for k in range(10))
            uu = math.fsum(float(x[t, k]) * float(Wu[j, k]) for k in range(10))
            want = float(alpha[b]) * (gg / (1.0 + math.exp(-gg))) * uu
            assert math.isclose(h[t, j], want, rel_tol=1e-13, abs_tol=1e-300)
            assert math.isclose(g[t, j], gg, rel_tol=1e-13, abs_tol=1e-15)
            assert math.isclose(u[t, j], uu, rel_tol=1e-13, abs_tol=1e-15)
            assert math.isclose(ag[t, j], math.fsum(abs(float(x[t, k]) * float(Wg[j, k])) for k in range(10)), rel_tol=1e-13)
            assert math.isclose(au[t, j], math.fsum(abs(float(x[t, k]) * float(Wu[j, k])) for k in range(10)), rel_tol=1e-13)
    assert np.all(ag >= np.abs(g)) and np.all(au >= np.abs(u))


def test_hidden_contract_values_are_bf16_and_within_half_a_unit():
    x, Wg, Wu, Wd, off, alpha = small_layer(3, T=40)
    mask = np.ones(4, np.uint8)
    hc = oracle.mlpmoe_hidden(x, Wg, Wu, off, alpha, mask, "contract")
    he = oracle.mlpmoe_hidden(x, Wg, Wu, off, alpha, mask, "exact")
    assert np.array_equal(oracle.round_to_bf16(hc), hc)          # representable in bf16
    _, e = np.frexp(np.abs(he))
    half_unit = np.ldexp(1.0, e - 9)                              # bf16 keeps 8 significant bits
    assert np.all(np.abs(hc - he) <= half_unit * (1 + 1e-3))
    # and it is the NEAREST one for all but values sitting on a boundary to within float precision
    assert np.mean(hc == oracle.round_to_bf16(he)) > 0.99
