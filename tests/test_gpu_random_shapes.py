"""Seeded sweep over random shapes and branch tables: every kernel path (MFMA wide and narrow tiles, split K,
decode, generic), plain / routed / bf16-result entry points, against the oracle in contract mode.

Shapes are small enough for the oracle to take a fraction of a second each.  Branch widths are multiples of 8
(the fast paths) except where the case asks for an unaligned table (the generic kernels).  Tables may have
any number of active neurons, a handful included: the intermediate H is read back from the workspace and the
comparison accounts for the bf16 roundings of H that fp32 and the oracle decide differently (gpu_util)."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, check_bf16_flip_aware, flip_terms, run_gpu_with_hidden
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
    if seed % 4 == 1:
        # a thin layer: few active neurons (one thin branch of a faded or pruned layer)
        widths = [w // 8 // unit * unit for w in widths]
    if not any(w and m for w, m in zip(widths, mask)):
        widths[0], mask[0] = 8 * unit, 1
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    T = int(rng.choice([1, 3, 16, 17, 64, 255, 257, 600]))
    alpha = rng.uniform(0.8, 1.25, size=B).astype(np.float32)
    kind = ("plain", "routed", "bf16_out")[seed % 3]
    return d_model, off, mask, alpha, T, kind, rng


@pytest.mark.parametrize("seed", range(30))
def test_random_case(mm, seed):
    d_model, off, mask, alpha, T, kind, rng = draw_case(seed)
    d_inter, B = int(off[-1]), len(alpha)
    print("case", seed, dict(d_model=d_model, widths=np.diff(off).tolist(), mask=mask.tolist(), T=T, kind=kind), flush=True)
    x, Wg, Wu, Wd = synth.random_layer(rng, T, d_model, d_inter, dtype="bf16")
    args = (x, Wg, Wu, Wd, off, alpha, mask)
    label = "case %d (%s, %d active neurons):" % (seed, kind, int(sum(w for w, m in zip(np.diff(off), mask) if m)))
    if kind == "routed":
        route = (rng.uniform(size=(T, B)) < 0.6).astype(np.uint8)
        route[rng.integers(0, T)] = 0                       # one token takes nothing
        got, H = run_gpu_with_hidden(*args, route=route)
        check_bf16_flip_aware(got, H, *args, route=route, label=label)
        assert not np.any(got[~np.any(route[:, mask != 0], axis=1)])
    elif kind == "bf16_out":
        got, H = run_gpu_with_hidden(*args, out_bf16=True)
        f = flip_terms(H, *args, label=label)
        ref = oracle.round_to_bf16(f["ref_c"])
        _, e = np.frexp(np.abs(f["ref_c"]))
        # the fp32 sum rounded once: one bf16 unit of the reference on top of what the float result is allowed
        assert np.all(np.abs(got - ref) <= BF16_TOL * f["rms_c"] + f["allow_c"] + np.ldexp(1.0, e - 8) + 1e-30), label
        own = oracle.round_to_bf16(f["H"] @ f["Wd"].T)
        _, e = np.frexp(np.abs(own))
        assert np.all(np.abs(got - own) <= f["sum_err"] + np.ldexp(1.0, e - 8) + 1e-30), label
    else:
        got, H = run_gpu_with_hidden(*args)
        check_bf16_flip_aware(got, H, *args, label=label)
        # the entry point without a workspace argument gives the same bits
        import gpu_util
        assert np.array_equal(gpu_util.run_gpu(*args), got)
