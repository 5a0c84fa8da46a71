"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (automatic
path, library workspace).  The oracle evaluates a seeded sample of token rows (tokens are
independent, so a row of the full result is the oracle's result for that row alone)."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, run_gpu, to_dev, widen
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu

N_SAMPLE = 12


def table_for(L, mm, pad_to=8):
    w = L.workload
    off, alpha, mask, gather = mm.mlpmoe_slice(w.d_inter, w.B, 0, L.neuron_keep, pad_to)
    mask = mask.copy()
    mask[L.inactive] = 0
    return off, L.alpha_draw, mask, gather


def check_sampled(got, L, Wg, Wu, Wd, off, alpha, mask, seed):
    T = L.T
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(T, size=min(N_SAMPLE, T), replace=False))
    xs = widen(L.x[rows])
    ref_c = oracle.mlpmoe_forward(xs, Wg, Wu, Wd, off, alpha, mask, mode="contract")
    ref_e = oracle.mlpmoe_forward(xs, Wg, Wu, Wd, off, alpha, mask, mode="exact")
    assert np.all(np.isfinite(got))
    e_c = oracle.rel_max_err(got[rows], ref_c)
    e_e = oracle.rel_max_err(got[rows], ref_e)
    print("T=%d rows=%d err(contract)=%.2e err(exact)=%.2e" % (T, len(rows), e_c, e_e))
    assert e_c <= BF16_TOL and e_e <= BF16_TOL
    return e_c, e_e


@pytest.mark.parametrize("name", ["qwen05b", "qwen05b_pruned", "llama8b", "llama8b_fade"])
def test_full_size_workload(name):
    import torch
    from paper_2511_21089_amd import binding as mm
    w = synth.WORKLOADS[name]
    Tmax = max(w.T_list)
    L = synth.make_layer(name, Tmax, seed=11)
    off, alpha, mask, gather = table_for(L, mm)
    dev_w = tuple(to_dev(a) for a in (L.W_gate, L.W_up, L.W_down))
    if L.neuron_keep is not None:
        dev_w = mm.mlpmoe_compact(dev_w[0], dev_w[1], dev_w[2], gather)
        # oracle side: the UNCOMPACTED layer with removed neurons' up rows zeroed
        Wu_ref = L.W_up.copy()
        Wu_ref[L.neuron_keep == 0] = 0
        o_off = (np.arange(w.B + 1) * (w.d_inter // w.B)).astype(np.int32)
        Wg, Wu, Wd = widen(L.W_gate), widen(Wu_ref), widen(L.W_down)
    else:
        o_off = off
        Wg, Wu, Wd = widen(L.W_gate), widen(L.W_up), widen(L.W_down)
    x_all = to_dev(L.x)
    d_inter_c = int(off[-1])
    for T in sorted(set(w.T_list)):
        out = torch.full((T, w.d_model), float("nan"), dtype=torch.float32, device="cuda")
        mm.mlpmoe_forward_bf16(x_all[:T], dev_w[0], dev_w[1], dev_w[2], off, alpha, mask, out=out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        Lt = synth.LayerInputs(w, T, L.x[:T], None, None, None, alpha, L.inactive)
        check_sampled(got, Lt, Wg, Wu, Wd, o_off, alpha, mask, seed=T)
    assert d_inter_c % 8 == 0
