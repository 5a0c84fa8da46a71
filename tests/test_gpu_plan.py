"""The plan object: checked against the oracle, and the same bits as the plain entry point for every T it covers."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, FP32_TOL, to_dev, widen
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


def test_plan_forward_equals_plain_forward():
    import torch
    from paper_2511_21089_amd import binding as mm
    L = synth.make_layer("qwen05b_pruned", 600, seed=41, d_model=256, d_inter=8 * 256)
    off, _, mask, _ = mm.mlpmoe_slice(8 * 256, 8)
    mask[L.inactive] = 0
    alpha = L.alpha_draw
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    plan = mm.Plan(off, alpha, mask, 256, 8 * 256, max_T=600)
    for T in (1, 16, 17, 255, 256, 300, 600):
        print("plan case T =", T, flush=True)
        ref = mm.mlpmoe_forward_bf16(x[:T], Wg, Wu, Wd, off, alpha, mask)
        got = plan.forward(x[:T], Wg, Wu, Wd)
        torch.cuda.synchronize()
        assert torch.equal(ref, got), T
        for mode in ("contract", "exact"):               # 1536 active neurons: the plain tolerance applies
            o = oracle.mlpmoe_forward(widen(L.x[:T]), widen(L.W_gate), widen(L.W_up), widen(L.W_down), off, alpha,
                                      mask, mode=mode)
            assert oracle.rel_max_err(got.cpu().numpy(), o) <= BF16_TOL, (T, mode)
    with pytest.raises(mm.MlpMoeError) as ei:
        plan.forward(torch.cat([x, x[:1]]), Wg, Wu, Wd)
    assert ei.value.status == mm.ERR_SHAPE
    # an unaligned table takes the generic kernels through a plan as well
    off_u = np.array([0, 300, 300, 700, 1001, 1300, 1600, 1900, 2048], np.int32)
    plan_u = mm.Plan(off_u, alpha, mask, 256, 8 * 256, max_T=40)
    ref = mm.mlpmoe_forward_bf16(x[:40], Wg, Wu, Wd, off_u, alpha, mask)
    got_u = plan_u.forward(x[:40], Wg, Wu, Wd)
    assert torch.equal(ref, got_u)
    o = oracle.mlpmoe_forward(widen(L.x[:40]), widen(L.W_gate), widen(L.W_up), widen(L.W_down), off_u, alpha, mask,
                              mode="contract")
    assert oracle.rel_max_err(got_u.cpu().numpy(), o) <= BF16_TOL
    # float storage
    Lf = synth.make_layer("tiny_f32", 32, seed=1)
    offf, alf, mkf, _ = mm.mlpmoe_slice(256, 4)
    xf, Wgf, Wuf, Wdf = (to_dev(a) for a in (Lf.x, Lf.W_gate, Lf.W_up, Lf.W_down))
    plan_f = mm.Plan(offf, alf, mkf, 64, 256, max_T=32, elem_bytes=4)
    ref = mm.mlpmoe_forward_f32(xf, Wgf, Wuf, Wdf, offf, alf, mkf)
    got_f = plan_f.forward(xf, Wgf, Wuf, Wdf)
    assert torch.equal(ref, got_f)
    o = oracle.mlpmoe_forward(Lf.x, Lf.W_gate, Lf.W_up, Lf.W_down, offf, alf, mkf, mode="exact")
    assert oracle.rel_max_err(got_f.cpu().numpy(), o) <= FP32_TOL
    for p in (plan, plan_u, plan_f):
        p.destroy()


def test_plan_forward_in_a_graph():
    import torch
    from paper_2511_21089_amd import binding as mm
    L = synth.make_layer("qwen05b", 8, seed=42, d_model=256, d_inter=8 * 256)
    off, alpha, mask, _ = mm.mlpmoe_slice(8 * 256, 8)
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    plan = mm.Plan(off, alpha, mask, 256, 8 * 256, max_T=8)
    out = torch.empty((8, 256), dtype=torch.float32, device="cuda")
    plan.forward(x, Wg, Wu, Wd, out=out)
    torch.cuda.synchronize()
    eager = out.clone()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            plan.forward(x, Wg, Wu, Wd, out=out)
    for rep in range(3):
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        plan.forward(x, Wg, Wu, Wd)             # eager work between replays
        torch.cuda.synchronize()
    o = oracle.mlpmoe_forward(widen(L.x), widen(L.W_gate), widen(L.W_up), widen(L.W_down), off, alpha, mask,
                              mode="contract")
    assert oracle.rel_max_err(eager.cpu().numpy(), o) <= BF16_TOL
    plan.destroy()
