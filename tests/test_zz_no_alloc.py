"""mlpmoe_forward_bf16_noalloc: the forward in the library's fixed scratch block, for callers that cannot
allocate.  Through the C ABI, against mlpmoe_forward_bf16_ws (same kernels: the results must be identical bit
for bit) on two calls in a row, the second with a smaller input, with PyTorch's and the device's free memory
unchanged; sizes beyond the block are refused."""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, to_dev, widen
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


def test_no_alloc_entry_point_matches_workspace_entry_point():
    import torch
    from paper_2511_21089_amd import binding as mm
    L = synth.make_layer("qwen05b_pruned", 600, seed=91, d_model=512, d_inter=8 * 320)
    off, _, mask, _ = mm.mlpmoe_slice(8 * 320, 8)
    mask[L.inactive] = 0
    alpha = L.alpha_draw
    x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    host = tuple(widen(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
    ws = mm.new_workspace(600, 512, 8 * 320, 8)
    want = {}
    for T in (600, 16, 7, 1):
        want[T] = mm.mlpmoe_forward_bf16_ws(x[:T], Wg, Wu, Wd, off, alpha, mask, ws)
    outs = {T: torch.full((T, 512), float("nan"), dtype=torch.float32, device="cuda") for T in want}
    # A first pass lets the runtime do what it does once per process (look the block's address up, load code
    # objects, size its own queues); from then on neither PyTorch's allocator nor the device's free memory may move.
    for T in (600, 16, 7, 1):
        mm.mlpmoe_forward_bf16_noalloc(x[:T], Wg, Wu, Wd, off, alpha, mask, outs[T])
        torch.cuda.synchronize()
        assert torch.equal(outs[T], want[T]), T
        print("first pass T=%d free=%d" % (T, torch.cuda.mem_get_info()[0]), flush=True)
    before = torch.cuda.memory_allocated()
    free_before = torch.cuda.mem_get_info()[0]
    for T in (600, 16, 600, 7, 1):                         # in a row, smaller after larger and back
        outs[T].fill_(float("nan"))
        mm.mlpmoe_forward_bf16_noalloc(x[:T], Wg, Wu, Wd, off, alpha, mask, outs[T])
        torch.cuda.synchronize()
        print("T=%d free=%d" % (T, torch.cuda.mem_get_info()[0]), flush=True)
        assert torch.equal(outs[T], want[T]), T
    assert torch.cuda.memory_allocated() == before
    assert torch.cuda.mem_get_info()[0] == free_before
    for T in (600, 7):
        ref = oracle.mlpmoe_forward(host[0][:T], host[1], host[2], host[3], off, alpha, mask, mode="contract")
        assert oracle.rel_max_err(outs[T].cpu().numpy(), ref) <= BF16_TOL, T


def test_no_alloc_entry_point_refuses_what_does_not_fit():
    import torch
    from paper_2511_21089_amd import binding as mm
    assert mm.mlpmoe_workspace_bytes(4096, 4096, 14336, 16) > mm.NOALLOC_SCRATCH_BYTES
    off, alpha, mask, _ = mm.mlpmoe_slice(14336, 16)
    # argument check only: the size test comes before any device access, so small stand-in tensors do
    x = torch.zeros((8, 8), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    import ctypes
    rc = mm.lib.mlpmoe_forward_bf16_noalloc(ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(x.data_ptr()),
                                            ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(x.data_ptr()),
                                            off.ctypes.data, alpha.ctypes.data, mask.ctypes.data, 4096, 4096, 14336, 16,
                                            ctypes.c_void_p(out.data_ptr()), None)
    assert rc == mm.ERR_WORKSPACE
    assert "16777216" in mm.last_error_detail()
    # the decode sizes of the 8B-shaped layer fit
    assert mm.mlpmoe_workspace_bytes(16, 4096, 14336, 16) <= mm.NOALLOC_SCRATCH_BYTES
