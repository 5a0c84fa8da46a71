"""The caller-workspace entry point allocates nothing and synchronises nothing, so a forward can be
captured in a HIP graph.  Every replay must reproduce the eager result bit for bit, also with the
program's own eager launches and synchronisations between replays and with new inputs written
into the captured buffers."""
import numpy as np
import pytest

from gpu_util import to_dev
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T", [5, 300])        # decode kernels, MFMA kernels (with split-K reduce)
def test_forward_in_a_graph_replays_exactly(T):
    import torch
    from paper_2511_21089_amd import binding as mm
    L = synth.make_layer("qwen05b_pruned", T, seed=31, d_model=256, d_inter=8 * 256)
    off, _, mask, _ = mm.mlpmoe_slice(8 * 256, 8)
    mask[L.inactive] = 0
    alpha = L.alpha_draw
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    ws = mm.new_workspace(T, 256, 8 * 256, 8)
    out = torch.empty((T, 256), dtype=torch.float32, device="cuda")

    def forward():
        mm.mlpmoe_forward_bf16_ws(x, Wg, Wu, Wd, off, alpha, mask, ws, out=out)

    forward()                                   # first call does the per-device set-up
    torch.cuda.synchronize()
    eager = out.clone()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            forward()
    torch.cuda.synchronize()
    x0 = x.clone()
    for rep in range(4):
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        # eager work of the same library and a changed input between replays
        x.copy_(torch.roll(x0, 1, dims=0))
        forward()
        torch.cuda.synchronize()
        rolled = out.clone()
        out.fill_(float("nan"))
        graph.replay()                          # the graph reads the buffers, not a snapshot
        torch.cuda.synchronize()
        assert torch.equal(out, rolled), rep
        x.copy_(x0)
