"""GPU parity at the full benchmark sizes, through the entry point and launch configuration bench.py times
(mlpmoe_forward_bf16, automatic path).  The whole result is compared with the oracle, element by element, in
both oracle modes.  The workspace is a test-owned block handed over with mlpmoe_set_workspace and filled with
bf16 NaNs first, so that an intermediate tile that is never computed shows in the result; for the largest T the
intermediate H itself is read back and checked on one token row of every 16-row MFMA fragment."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, check_bf16_flip_aware, to_dev, widen
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


def table_for(L, mm, pad_to=8, pad_rows_to=64):
    w = L.workload
    off, alpha, mask, gather = mm.mlpmoe_slice(w.d_inter, w.B, 0, L.neuron_keep, pad_to, pad_rows_to)
    mask = mask.copy()
    mask[L.inactive] = 0
    return off, L.alpha_draw, mask, gather


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
        # the compacted layer as the kernels see it, for the check of H
        c_host = tuple(t.view(torch.int16).cpu().numpy().view(np.uint16) for t in dev_w)
    else:
        o_off = off
        Wg, Wu, Wd = widen(L.W_gate), widen(L.W_up), widen(L.W_down)
        c_host = (L.W_gate, L.W_up, L.W_down)
    x_all = to_dev(L.x)
    d_inter_c = int(off[-1])
    assert d_inter_c % 8 == 0
    ws = mm.new_workspace(Tmax, w.d_model, d_inter_c, w.B)
    mm.mlpmoe_set_workspace(ws)
    try:
        for T in sorted(set(w.T_list)):
            print("full size", name, "T =", T, flush=True)
            ws.fill_(0xFF)
            out = torch.full((T, w.d_model), float("nan"), dtype=torch.float32, device="cuda")
            before = torch.cuda.memory_allocated()
            mm.mlpmoe_forward_bf16(x_all[:T], dev_w[0], dev_w[1], dev_w[2], off, alpha, mask, out=out)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
            got = out.cpu().numpy()
            assert np.all(np.isfinite(got))
            xs = widen(L.x[:T])
            for mode in ("contract", "exact"):
                ref = oracle.mlpmoe_forward(xs, Wg, Wu, Wd, o_off, alpha, mask, mode=mode)
                err = oracle.rel_max_err(got, ref)
                print("  all %d x %d elements, err(%s) = %.2e" % (T, w.d_model, mode, err), flush=True)
                assert err <= BF16_TOL, (name, T, mode, err)
                del ref
            if T == Tmax:
                # H as the kernels left it: one token row of every 16-row fragment of every token tile
                rows = np.array([r for r in (16 * i + (7 * i) % 16 for i in range((T + 15) // 16)) if r < T])
                ld = mm.mlpmoe_hidden_ld(d_inter_c)
                Hb = ws[: T * ld * 2].view(torch.int16).view(T, ld)[torch.from_numpy(rows).cuda()][:, :d_inter_c]
                H = synth.bf16_bits_to_f32(Hb.cpu().numpy().view(np.uint16)).astype(np.float64)
                check_bf16_flip_aware(got[rows], H, L.x[rows], c_host[0], c_host[1], c_host[2], off, alpha, mask,
                                      label="%s T=%d, %d sampled rows:" % (name, T, len(rows)))
    finally:
        mm.mlpmoe_set_workspace(None)
