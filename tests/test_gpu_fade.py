"""GPU parity for Fractal Fade weight preparation (Sec. 3.2): bit-exact against the oracle."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, oracle_out, to_dev
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


def bits(t):
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def fade_and_compare(mm, L, off, sparsity=None):
    Wg_d, Wu_d = to_dev(L.W_gate), to_dev(L.W_up)
    thr, kept = mm.mlpmoe_fade(Wg_d, Wu_d, off, sparsity)
    rWg, rWu, rthr, rkept = oracle.fractal_fade(L.W_gate, L.W_up, off, sparsity)
    assert np.array_equal(bits(Wg_d), rWg) and np.array_equal(bits(Wu_d), rWu)
    for b in range(len(off) - 1):
        for m in range(2):
            assert int(kept[b, m]) == rkept[b][m], (b, m)
            if rthr[b][m] is None:
                assert np.isnan(thr[b, m])
            else:
                assert abs(float(thr[b, m]) - rthr[b][m]) <= 1e-6 * abs(rthr[b][m]) + 1e-30
    return Wg_d, Wu_d, rWg, rWu


@pytest.fixture(scope="module")
def mm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2511_21089_amd import binding
    return binding


def test_fade_schedule_small(mm):
    """B = 8 with uneven, empty and tiny branches; the schedule of Sec. 3.2."""
    L = synth.make_layer("qwen05b", 1, seed=5, d_model=72, d_inter=1000)
    off = np.array([0, 130, 130, 131, 400, 520, 777, 999, 1000], np.int32)
    fade_and_compare(mm, L, off)


def test_fade_explicit_sparsity_and_ties(mm):
    L = synth.make_layer("qwen05b", 1, seed=6, d_model=64, d_inter=512)
    # heavy ties: quantise the weights to a handful of magnitudes
    f = np.round(synth.bf16_bits_to_f32(L.W_gate) * 200) / 200
    L.W_gate[:] = synth.f32_to_bf16_bits(f.astype(np.float32))
    off = np.arange(5, dtype=np.int32) * 128
    fade_and_compare(mm, L, off, [0.0, 1.0, 0.37, 1e-9])


def test_fade_full_size_then_forward(mm):
    """The 0.5B-shaped layer with 16 branches (the paper's configuration): bit-exact fade, then
    the forward on the faded weights against the oracle forward on the oracle's faded weights."""
    import torch
    L = synth.make_layer("qwen05b", 300, seed=7, B=16)
    off, alpha, mask, _ = mm.mlpmoe_slice(4864, 16)
    Wg_d, Wu_d, rWg, rWu = fade_and_compare(mm, L, off)
    nz = int((rWg & 0x7FFF != 0).sum() + (rWu & 0x7FFF != 0).sum())
    assert abs(nz / (2 * 4864 * 896) - (1 - 0.9 * 7.5 / 16)) < 0.01     # mean sparsity of the schedule
    out = mm.mlpmoe_forward_bf16(to_dev(L.x), Wg_d, Wu_d, to_dev(L.W_down), off, alpha, mask)
    ref = oracle_out(L.x, rWg, rWu, L.W_down, off, alpha, mask, "contract")
    assert oracle.rel_max_err(out.cpu().numpy(), ref) <= BF16_TOL


def test_fade_8b_block_size(mm):
    """One Llama-8B-sized branch block (896 x 4096 = 3.7 M entries per projection) among others."""
    L = synth.make_layer("llama8b", 1, seed=8, d_inter=3 * 896, B=3)
    off = np.array([0, 896, 1792, 2688], np.int32)
    fade_and_compare(mm, L, off, [0.0, 0.45, 0.84375])


def test_fade_neurons_matches_the_oracle(mm):
    """Structured form: kept set and scores of every neuron against the oracle, uneven branches."""
    widths = [96, 0, 200, 8, 333, 64]
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    L = synth.make_layer("qwen05b", 4, seed=71, d_model=520, d_inter=int(off[-1]))
    rng = np.random.default_rng(2)
    counts = np.array([int(rng.integers(0, w + 1)) for w in widths], np.int32)
    counts[0], counts[3] = widths[0], 0                       # keep all / keep none
    keep, sc = mm.mlpmoe_fade_neurons(to_dev(L.W_gate), to_dev(L.W_up), off, counts)
    rkeep, rsc = oracle.fade_neurons(L.W_gate, L.W_up, off, counts)
    assert np.allclose(sc, rsc, rtol=1e-13, atol=0)
    for b, w in enumerate(widths):
        assert keep[off[b]:off[b + 1]].sum() == counts[b]
    if not np.array_equal(keep, rkeep):
        # the two sums differ in their last bits: a disagreement is only valid between near-equal scores
        for b in range(len(widths)):
            lo, hi = off[b], off[b + 1]
            diff = np.nonzero(keep[lo:hi] != rkeep[lo:hi])[0]
            if diff.size:
                s = rsc[lo:hi][diff]
                assert s.max() - s.min() <= 1e-12 * s.max()


def test_fade_neurons_exact_ties_go_by_index(mm):
    """Small-integer weights: scores are exact and full of ties, so the kept set must agree exactly."""
    rng = np.random.default_rng(3)
    d_model, widths = 64, [40, 72, 16]
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    Wg = synth.f32_to_bf16_bits(rng.integers(-2, 3, size=(off[-1], d_model)).astype(np.float32))
    Wu = synth.f32_to_bf16_bits(rng.integers(-2, 3, size=(off[-1], d_model)).astype(np.float32))
    counts = np.array([17, 36, 5], np.int32)
    keep, sc = mm.mlpmoe_fade_neurons(to_dev(Wg), to_dev(Wu), off, counts)
    rkeep, rsc = oracle.fade_neurons(Wg, Wu, off, counts)
    assert np.array_equal(sc, rsc)
    assert len(np.unique(rsc)) < len(rsc) // 2               # the case really has ties
    assert np.array_equal(keep, rkeep)


def test_fade_neurons_then_slice_compact_forward(mm):
    """The whole preparation on the GPU side: scores -> kept neurons -> compacted layer -> forward, against the
    oracle's forward of the uncompacted layer with the dropped neurons' up rows zeroed."""
    B, d_b, d_model, T = 16, 160, 512, 300
    L = synth.make_layer("llama8b", T, seed=72, d_model=d_model, d_inter=B * d_b)
    off, alpha, mask, _ = mm.mlpmoe_slice(B * d_b, B)
    counts = np.array([int(np.floor(d_b * (1 - 0.4 * b / (B - 1)) + 0.5)) for b in range(B)], np.int32)
    Wg_d, Wu_d, Wd_d = to_dev(L.W_gate), to_dev(L.W_up), to_dev(L.W_down)
    keep, _ = mm.mlpmoe_fade_neurons(Wg_d, Wu_d, off, counts)
    rkeep, _ = oracle.fade_neurons(L.W_gate, L.W_up, off, counts)
    assert np.array_equal(keep, rkeep)
    offc, alphac, maskc, gather = mm.mlpmoe_slice(B * d_b, B, 0, keep, 8)
    Wg_c, Wu_c, Wd_c = mm.mlpmoe_compact(Wg_d, Wu_d, Wd_d, gather)
    got = mm.mlpmoe_forward_bf16(to_dev(L.x), Wg_c, Wu_c, Wd_c, offc, L.alpha_draw, maskc).cpu().numpy()
    Wu0 = L.W_up.copy()
    Wu0[keep == 0] = 0
    for mode in ("contract", "exact"):
        ref = oracle_out(L.x, L.W_gate, Wu0, L.W_down, off, L.alpha_draw, mask, mode)
        assert oracle.rel_max_err(got, ref) <= BF16_TOL, mode


def fade_and_compare_f32(mm, Wg, Wu, off, sparsity=None):
    """Float storage: the faded matrices bit for bit (signs of the zeros included), survivor counts exactly,
    thresholds to float rounding."""
    import torch
    Wg_d, Wu_d = torch.from_numpy(Wg).cuda(), torch.from_numpy(Wu).cuda()
    thr, kept = mm.mlpmoe_fade(Wg_d, Wu_d, off, sparsity)
    rWg, rWu, rthr, rkept = oracle.fractal_fade(Wg, Wu, off, sparsity)
    assert np.array_equal(Wg_d.cpu().numpy().view(np.uint32), rWg.view(np.uint32))
    assert np.array_equal(Wu_d.cpu().numpy().view(np.uint32), rWu.view(np.uint32))
    for b in range(len(off) - 1):
        for m in range(2):
            assert int(kept[b, m]) == rkept[b][m], (b, m)
            if rthr[b][m] is None:
                assert np.isnan(thr[b, m])
            else:
                assert float(thr[b, m]) == float(np.float32(rthr[b][m])), (b, m)


def test_fade_float_storage(mm):
    """Float weights: uneven, empty and one-row branches with the schedule of Sec. 3.2; explicit ratios with
    s = 1 (everything goes) and a ratio so small that only the minimum goes."""
    rng = np.random.default_rng(21)
    d_model, d_inter = 68, 1000
    Wg = (rng.standard_normal((d_inter, d_model)) * 0.02).astype(np.float32)
    Wu = (rng.standard_normal((d_inter, d_model)) * 0.02).astype(np.float32)
    Wg[5, 7] = -0.0
    off = np.array([0, 130, 130, 131, 400, 520, 777, 999, 1000], np.int32)
    fade_and_compare_f32(mm, Wg, Wu, off)
    fade_and_compare_f32(mm, Wg, Wu, np.arange(5, dtype=np.int32) * 250, [0.0, 1.0, 0.37, 1e-9])


def test_fade_float_storage_ties_and_close_values(mm):
    """Heavy ties (a handful of magnitudes) and magnitudes that differ only in their last bits, so that
    the two order statistics around the quantile share their upper bits or sit one unit apart."""
    rng = np.random.default_rng(22)
    d_model, d_inter = 64, 512
    Wg = (np.round(rng.standard_normal((d_inter, d_model)) * 4) / 200).astype(np.float32)
    base = np.float32(0.0173)
    Wu = (base.view(np.uint32) + rng.integers(0, 9, size=(d_inter, d_model)).astype(np.uint32)).view(np.float32)
    Wu *= rng.choice(np.array([-1, 1], np.float32), size=Wu.shape)
    off = np.arange(5, dtype=np.int32) * 128
    fade_and_compare_f32(mm, Wg, Wu, off, [0.25, 0.5, 0.9, 0.61803])


def test_fade_float_storage_8b_block(mm):
    """One 8B-sized branch block of floats (896 x 4096 entries) with the ratio of the last branch of 16."""
    rng = np.random.default_rng(23)
    Wg = (rng.standard_normal((2 * 896, 4096)) * 0.02).astype(np.float32)
    Wu = (rng.standard_normal((2 * 896, 4096)) * 0.02).astype(np.float32)
    fade_and_compare_f32(mm, Wg, Wu, np.array([0, 896, 1792], np.int32), [0.0, 0.84375])


def test_fade_neurons_float_storage(mm):
    """Structured form on float weights: scores to the last bits, kept set as the oracle's."""
    import torch
    widths = [96, 0, 200, 8, 333, 64]
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    rng = np.random.default_rng(24)
    Wg = (rng.standard_normal((int(off[-1]), 516)) * 0.02).astype(np.float32)
    Wu = (rng.standard_normal((int(off[-1]), 516)) * 0.02).astype(np.float32)
    counts = np.array([96, 0, 77, 0, 200, 1], np.int32)
    keep, sc = mm.mlpmoe_fade_neurons(torch.from_numpy(Wg).cuda(), torch.from_numpy(Wu).cuda(), off, counts)
    rkeep, rsc = oracle.fade_neurons(Wg, Wu, off, counts)
    assert np.allclose(sc, rsc, rtol=1e-13, atol=0)
    for b, w in enumerate(widths):
        assert keep[off[b]:off[b + 1]].sum() == counts[b]
    if not np.array_equal(keep, rkeep):
        for b in range(len(widths)):
            lo, hi = off[b], off[b + 1]
            diff = np.nonzero(keep[lo:hi] != rkeep[lo:hi])[0]
            if diff.size:
                s = rsc[lo:hi][diff]
                assert s.max() - s.min() <= 1e-12 * s.max()


def test_fade_float_storage_then_forward(mm):
    """Float layer with the schedule of Sec. 3.2 (B = 8): the faded weights feed the float forward, which must
    match the oracle's forward of the oracle's faded weights at the float tolerance."""
    import torch
    rng = np.random.default_rng(25)
    T, d_model, d_inter, B = 40, 96, 640, 8
    Wg, Wu, Wd = ((rng.standard_normal(sh) * 0.05).astype(np.float32) for sh in
                  ((d_inter, d_model), (d_inter, d_model), (d_model, d_inter)))
    x = rng.standard_normal((T, d_model)).astype(np.float32)
    off, alpha, mask, _ = mm.mlpmoe_slice(d_inter, B)
    Wg_d, Wu_d = torch.from_numpy(Wg).cuda(), torch.from_numpy(Wu).cuda()
    mm.mlpmoe_fade(Wg_d, Wu_d, off)
    rWg, rWu, _, _ = oracle.fractal_fade(Wg, Wu, off)
    assert np.array_equal(Wg_d.cpu().numpy().view(np.uint32), rWg.view(np.uint32))
    got = mm.mlpmoe_forward_f32(torch.from_numpy(x).cuda(), Wg_d, Wu_d, torch.from_numpy(Wd).cuda(), off, alpha, mask)
    ref = oracle.mlpmoe_forward(x.astype(np.float64), rWg.astype(np.float64), rWu.astype(np.float64),
                                Wd.astype(np.float64), off, alpha, mask, mode="exact")
    assert oracle.rel_max_err(got.cpu().numpy(), ref) <= 1e-5
