"""mlpmoe_set_workspace: with a caller-owned block set, the entry points that take no workspace argument
(here mlpmoe_forward, the signature the method's forward is specified with) allocate nothing, refuse calls
the block is too small for, and can be recorded into a HIP graph."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, to_dev, widen
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


def test_forward_in_the_callers_workspace():
    import torch
    from paper_2511_21089_amd import binding as mm
    L = synth.make_layer("qwen05b_pruned", 300, seed=71, d_model=256, d_inter=8 * 256)
    off, _, mask, _ = mm.mlpmoe_slice(8 * 256, 8)
    mask[L.inactive] = 0
    alpha = L.alpha_draw
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    host = tuple(widen(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    ws = mm.new_workspace(300, 256, 8 * 256, 8)
    out = torch.empty((300, 256), dtype=torch.float32, device="cuda")
    mm.mlpmoe_release()                                   # no library-owned block to fall back on
    mm.mlpmoe_set_workspace(ws)
    try:
        for T in (300, 16, 1):
            o = out[:T]
            ws.fill_(0xFF)
            o.fill_(float("nan"))
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            free_before = torch.cuda.mem_get_info()[0]
            mm.mlpmoe_forward(x[:T], Wg, Wu, Wd, off, alpha, mask, out=o)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
            assert torch.cuda.mem_get_info()[0] == free_before      # no hipMalloc behind PyTorch's back either
            ref = oracle.mlpmoe_forward(host[0][:T], host[1], host[2], host[3], off, alpha, mask, mode="contract")
            assert oracle.rel_max_err(o.cpu().numpy(), ref) <= BF16_TOL, T
            # H was written into the caller's block (it was all NaN before)
            assert not torch.isnan(ws[: 2 * 8].view(torch.bfloat16).float()).any()
        # a call the block is too small for is refused, nothing is allocated
        big = torch.cat([x, x, x])
        with pytest.raises(mm.MlpMoeError) as ei:
            mm.mlpmoe_forward(big, Wg, Wu, Wd, off, alpha, mask)
        assert ei.value.status == mm.ERR_WORKSPACE
        assert torch.cuda.mem_get_info()[0] == free_before
        # recorded into a graph through the plain signature; replays interleaved with eager work
        for T in (5, 300):
            o = out[:T]
            mm.mlpmoe_forward(x[:T], Wg, Wu, Wd, off, alpha, mask, out=o)
            torch.cuda.synchronize()
            eager = o.clone()
            stream = torch.cuda.Stream()
            stream.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(stream):
                with torch.cuda.graph(graph, stream=stream):
                    mm.mlpmoe_forward(x[:T], Wg, Wu, Wd, off, alpha, mask, out=o)
            for rep in range(3):
                o.fill_(float("nan"))
                graph.replay()
                torch.cuda.synchronize()
                assert torch.equal(o, eager), (T, rep)
                mm.mlpmoe_forward(x[:T], Wg, Wu, Wd, off, alpha, mask)       # eager work between replays
                torch.cuda.synchronize()
    finally:
        mm.mlpmoe_set_workspace(None)
    # cleared: the library-owned block is back (and grows as before)
    got = mm.mlpmoe_forward(x, Wg, Wu, Wd, off, alpha, mask)
    ref = oracle.mlpmoe_forward(*host, off, alpha, mask, mode="contract")
    assert oracle.rel_max_err(got.cpu().numpy(), ref) <= BF16_TOL


def test_library_workspace_growth_is_refused_while_capturing():
    import torch
    from paper_2511_21089_amd import binding as mm
    L = synth.make_layer("qwen05b", 40, seed=72, d_model=128, d_inter=8 * 128)
    off, alpha, mask, _ = mm.mlpmoe_slice(8 * 128, 8)
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    out = torch.empty((40, 128), dtype=torch.float32, device="cuda")
    mm.mlpmoe_release()                                   # the next call would have to allocate
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    status = None
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            out.zero_()                                   # so that the recorded graph is not empty
            try:
                mm.mlpmoe_forward(x, Wg, Wu, Wd, off, alpha, mask, out=out)
            except mm.MlpMoeError as e:
                status = e.status
    assert status == mm.ERR_WORKSPACE
    torch.cuda.synchronize()
    mm.mlpmoe_forward(x, Wg, Wu, Wd, off, alpha, mask, out=out)              # outside a capture it allocates and runs
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
