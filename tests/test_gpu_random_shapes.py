"""Seeded sweep over random shapes and branch tables: every kernel path (MFMA wide and narrow tiles, split K,
decode, generic), plain / routed / bf16-result entry points, against the oracle in contract mode.

Shapes are small enough for the oracle to take a fraction of a second each.  Branch widths are multiples of 8
(the fast paths) except where the case asks for an unaligned table (the generic kernels); every table keeps at
least 1000 active neurons so that a single flipped bf16 rounding of H cannot reach the tolerance (see the
tolerance derivation of the parity tests)."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, to_dev, widen
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2511_21089_amd import binding
    return binding


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    d_model = int(rng.choice([64, 72, 136, 256, 520, 1024]))
    B = int(rng.integers(1, 13))
    aligned = seed % 5 != 0
    unit = 8 if aligned else 1
    widths = [int(rng.integers(0, 40)) * unit + (0 if aligned else int(rng.integers(0, 8))) for _ in range(B)]
    mask = (rng.uniform(size=B) < 0.8).astype(np.uint8)
    # at least 1000 active neurons
    while sum(w for w, m in zip(widths, mask) if m) < 1000:
        b = int(rng.integers(0, B))
        widths[b] += 25 * unit
        mask[b] = 1
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    T = int(rng.choice([1, 3, 16, 17, 64, 255, 257, 600]))
    alpha = rng.uniform(0.8, 1.25, size=B).astype(np.float32)
    kind = ("plain", "routed", "bf16_out")[seed % 3]
    return d_model, off, mask, alpha, T, kind, rng


@pytest.mark.parametrize("seed", range(30))
def test_random_case(mm, seed):
    import torch
    d_model, off, mask, alpha, T, kind, rng = draw_case(seed)
    d_inter, B = int(off[-1]), len(alpha)
    print("case", seed, dict(d_model=d_model, widths=np.diff(off).tolist(), mask=mask.tolist(), T=T, kind=kind), flush=True)
    arrays = synth.random_layer(rng, T, d_model, d_inter, dtype="bf16")
    x, Wg, Wu, Wd = (to_dev(a) for a in arrays)
    host = tuple(widen(a) for a in arrays)
    if kind == "routed":
        route = (rng.uniform(size=(T, B)) < 0.6).astype(np.uint8)
        # keep the rms of the output representative: most tokens take most branches, one takes none
        route[rng.integers(0, T)] = 0
        got = mm.mlpmoe_forward_routed_bf16(x, Wg, Wu, Wd, off, alpha, mask, torch.from_numpy(route).cuda()).cpu().numpy()
        ref = oracle.mlpmoe_forward_routed(*host, off, alpha, mask, route, mode="contract")
        assert oracle.rel_max_err(got, ref) <= 2 * BF16_TOL      # fewer neurons per token than the 1000 of the table
    elif kind == "bf16_out":
        out = mm.mlpmoe_forward_bf16_out_bf16(x, Wg, Wu, Wd, off, alpha, mask)
        got = out.to(torch.float64).cpu().numpy()
        ref = oracle.round_to_bf16(oracle.mlpmoe_forward(*host, off, alpha, mask, mode="contract"))
        rms = float(np.sqrt(np.mean(ref * ref)))
        _, e = np.frexp(np.abs(ref))
        assert np.all(np.abs(got - ref) <= BF16_TOL * rms + np.ldexp(1.0, e - 8))
    else:
        got = mm.mlpmoe_forward_bf16(x, Wg, Wu, Wd, off, alpha, mask).cpu().numpy()
        ref = oracle.mlpmoe_forward(*host, off, alpha, mask, mode="contract")
        assert np.all(np.isfinite(got))
        assert oracle.rel_max_err(got, ref) <= BF16_TOL
