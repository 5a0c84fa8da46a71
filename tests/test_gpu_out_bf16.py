"""GPU parity of the bf16 forward whose result is stored as bf16 (one more rounding, of the sum).

Against the contract oracle rounded the same way, an element may differ by one bf16 unit where the fp32 sum
and the oracle's double sum fall on different sides of a rounding boundary, on top of the usual tolerance; so
the bound per element is BF16_TOL * rms + one unit in the last place of the reference, and most elements
must agree exactly.  The float result of the plain entry point, rounded on the host, must agree bit for bit
where the kernels add up in the same order (prefill), and to one unit where they do not (decode)."""
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


def bf16_ulp(v):
    """Spacing of bf16 at |v| (normal range)."""
    _, e = np.frexp(np.abs(v))
    return np.ldexp(1.0, e - 8)


def check(mm, L, off, alpha, mask, T, path=None, same_sums=True):
    import torch
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x[:T], L.W_gate, L.W_up, L.W_down))
    out = torch.full((T, x.shape[1]), float("nan"), dtype=torch.bfloat16, device="cuda")
    if path is None:
        mm.mlpmoe_forward_bf16_out_bf16(x, Wg, Wu, Wd, off, alpha, mask, out=out)
        f32 = mm.mlpmoe_forward_bf16(x, Wg, Wu, Wd, off, alpha, mask)
    else:
        ws = mm.new_workspace(T, x.shape[1], Wg.shape[0], len(alpha))
        mm.mlpmoe_forward_bf16_out_bf16_ws(x, Wg, Wu, Wd, off, alpha, mask, ws, path=path, out=out)
        f32 = mm.mlpmoe_forward_bf16_ws(x, Wg, Wu, Wd, off, alpha, mask, ws, path=path)
    got = out.to(torch.float64).cpu().numpy()
    assert np.all(np.isfinite(got))
    # the same sums, rounded by the kernel or by the oracle's rule on the host: identical.  The decode kernels
    # add the two halves of K separately for a float result and in one pass for a bf16 one: a unit apart at most
    f32_rounded = oracle.round_to_bf16(f32.cpu().numpy().astype(np.float64))
    if same_sums:
        assert np.array_equal(got, f32_rounded)
    else:
        assert np.all(np.abs(got - f32_rounded) <= bf16_ulp(f32_rounded)) and np.mean(got == f32_rounded) >= 0.98
    ref = oracle.round_to_bf16(oracle.mlpmoe_forward(widen(L.x[:T]), widen(L.W_gate), widen(L.W_up),
                                                     widen(L.W_down), off, alpha, mask, mode="contract"))
    rms = float(np.sqrt(np.mean(ref * ref)))
    assert np.all(np.abs(got - ref) <= BF16_TOL * rms + bf16_ulp(ref))
    assert np.mean(got == ref) >= 0.9
    return got


def test_prefill_and_decode_paths(mm):
    L = synth.make_layer("qwen05b_pruned", 600, seed=61, d_model=256, d_inter=8 * 256)
    off, _, mask, _ = mm.mlpmoe_slice(8 * 256, 8)
    mask[L.inactive] = 0
    alpha = L.alpha_draw
    check(mm, L, off, alpha, mask, 600)                    # MFMA kernels, K split (few output tiles)
    for T in (1, 7, 16):
        check(mm, L, off, alpha, mask, T, same_sums=False)  # decode kernels
    check(mm, L, off, alpha, mask, 600, path=mm.PATH_GENERIC)
    check(mm, L, off, alpha, mask, 16, path=mm.PATH_MFMA)


def test_unsplit_down_projection_and_ragged_tail(mm):
    """Enough output tiles that K is not split: the down kernel itself rounds and stores."""
    L = synth.make_layer("qwen05b", 4096 + 300, seed=62, d_model=2048 + 64, d_inter=1024)
    off, alpha, mask, _ = mm.mlpmoe_slice(1024, 8)
    check(mm, L, off, L.alpha_draw, mask, 4096 + 300)


def test_unaligned_table_and_no_active_branch(mm):
    import torch
    L = synth.make_layer("qwen05b", 70, seed=63, d_model=72, d_inter=1403)
    off = np.array([0, 337, 337, 501, 950, 1403], np.int32)
    mask = np.array([1, 1, 0, 1, 1], np.uint8)
    alpha = np.random.default_rng(3).uniform(0.9, 1.2, size=5).astype(np.float32)
    check(mm, L, off, alpha, mask, 70)
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    out = torch.full((70, 72), float("nan"), dtype=torch.bfloat16, device="cuda")
    mm.mlpmoe_forward_bf16_out_bf16(x, Wg, Wu, Wd, off, alpha, np.zeros(5, np.uint8), out=out)
    assert torch.count_nonzero(out).item() == 0 and not torch.isnan(out).any()


def test_full_size(mm):
    """8B-shaped layer, T = 4096: every element of the bf16 result against the rounded contract oracle."""
    import torch
    L = synth.make_layer("llama8b", 4096, seed=64)
    off, _, mask, _ = mm.mlpmoe_slice(14336, 16)
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    out = mm.mlpmoe_forward_bf16_out_bf16(x, Wg, Wu, Wd, off, L.alpha_draw, mask)
    assert out.dtype == torch.bfloat16
    got = out.to(torch.float64).cpu().numpy()
    ref = oracle.round_to_bf16(oracle.mlpmoe_forward(widen(L.x), widen(L.W_gate), widen(L.W_up),
                                                     widen(L.W_down), off, L.alpha_draw, mask, mode="contract"))
    rms = float(np.sqrt(np.mean(ref * ref)))
    assert np.all(np.abs(got - ref) <= BF16_TOL * rms + bf16_ulp(ref))
    assert np.mean(got == ref) >= 0.9
