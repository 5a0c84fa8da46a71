"""Helpers shared by the GPU parity tests: upload inputs, run a path through the C ABI, compare."""
import numpy as np

import oracle
from paper_2511_21089_amd import synth

FP32_TOL = 1e-5      # max|err| / rms(out), float storage
BF16_TOL = 1e-2      # bf16 storage with fp32 accumulation


def to_dev(a):
    import torch
    from paper_2511_21089_amd import binding as mm
    if a.dtype == np.uint16:
        return mm.bf16_tensor(a)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def widen(a):
    return synth.bf16_bits_to_f32(a) if a.dtype == np.uint16 else np.asarray(a, dtype=np.float32)


def run_gpu(x, Wg, Wu, Wd, off, alpha, mask, path=None, dev=None):
    """Forward through the C ABI; returns a float32 numpy array [T, d_model]."""
    import torch
    from paper_2511_21089_amd import binding as mm
    bf16 = x.dtype == np.uint16
    d = dev if dev is not None else tuple(to_dev(a) for a in (x, Wg, Wu, Wd))
    T, d_model = x.shape
    d_inter = Wg.shape[0]
    B = len(alpha)
    # poison the output so that unwritten elements are caught
    out = torch.full((T, d_model), float("nan"), dtype=torch.float32, device="cuda")
    if path is None:
        f = mm.mlpmoe_forward_bf16 if bf16 else mm.mlpmoe_forward_f32
        f(d[0], d[1], d[2], d[3], off, alpha, mask, out=out)
    else:
        ws = mm.new_workspace(T, d_model, d_inter, B, 2 if bf16 else 4)
        ws.fill_(0xFF)
        if bf16:
            mm.mlpmoe_forward_bf16_ws(d[0], d[1], d[2], d[3], off, alpha, mask, ws, path=path, out=out)
        else:
            mm.mlpmoe_forward_f32_ws(d[0], d[1], d[2], d[3], off, alpha, mask, ws, out=out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_out(x, Wg, Wu, Wd, off, alpha, mask, mode):
    return oracle.mlpmoe_forward(widen(x), widen(Wg), widen(Wu), widen(Wd), off, alpha, mask, mode=mode)
