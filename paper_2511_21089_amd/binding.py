"""ctypes binding of libmlpmoe.so: argument marshalling only.

Function names mirror include/mlpmoe.h.  Tensors are torch tensors on the GPU
(PyTorch supplies device memory and streams, nothing else); branch tables are
numpy arrays / sequences on the host.  Importing this module loads the shared
library and raises if it has not been built: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmlpmoe.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_OFFSETS, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_ALIGN = -1, -2, -3, -4, -5, -6, -7
PATH_AUTO, PATH_GENERIC, PATH_MFMA, PATH_DECODE = 0, 1, 2, 3
PATH_MFMA_WIDE, PATH_MFMA_NARROW, PATH_MFMA_SMALL, PATH_MFMA_MIXED, PATH_MFMA_DEEP, PATH_MFMA_SLIM = 4, 5, 6, 7, 8, 9
MAX_BRANCHES = 64

EXPORTS = ["mlpmoe_status_string", "mlpmoe_last_error_detail", "mlpmoe_slice", "mlpmoe_slice_rows", "mlpmoe_compact", "mlpmoe_fade", "mlpmoe_fade_neurons", "mlpmoe_workspace_bytes",
           "mlpmoe_forward_bf16", "mlpmoe_forward", "mlpmoe_forward_f32", "mlpmoe_forward_bf16_ws",
           "mlpmoe_forward_f32_ws", "mlpmoe_release", "mlpmoe_profile_enable",
           "mlpmoe_profile_collect", "mlpmoe_profile_disable", "mlpmoe_plan_create", "mlpmoe_plan_forward",
           "mlpmoe_plan_destroy", "mlpmoe_forward_routed_bf16", "mlpmoe_forward_routed_bf16_ws",
           "mlpmoe_forward_bf16_out_bf16", "mlpmoe_forward_bf16_out_bf16_ws",
           "mlpmoe_forward_routed_f32", "mlpmoe_forward_routed_f32_ws", "mlpmoe_set_workspace", "mlpmoe_hidden_ld",
           "mlpmoe_forward_bf16_noalloc"]


class MlpMoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = last_error_detail() if status == ERR_HIP else ""
        super().__init__("%s failed: %s (%d)%s" % (where, status_string(status), status,
                                                   " [" + detail + "]" if detail else ""))


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        # nothing built yet: build once (hipcc cross-compiles; no GPU needed)
        _build.build(force=True)
    # The library and PyTorch must share ONE HIP runtime (device pointers and streams cross between
    # them).  PyTorch ships its own libamdhip64 / libhsa-runtime64; loading it first makes the
    # dynamic loader satisfy this library's libamdhip64.so.7 dependency with that same copy.  In
    # the other order the system runtime would be loaded beside PyTorch's, and the one that
    # initialises second reports "no ROCm-capable device".
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, ip, fp, bp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    i, sz = ctypes.c_int, ctypes.c_size_t
    lib.mlpmoe_status_string.argtypes = [i]
    lib.mlpmoe_status_string.restype = ctypes.c_char_p
    lib.mlpmoe_last_error_detail.argtypes = []
    lib.mlpmoe_last_error_detail.restype = ctypes.c_char_p
    lib.mlpmoe_slice.argtypes = [i, i, i, bp, i, ip, fp, bp, ip, i]
    lib.mlpmoe_slice.restype = i
    lib.mlpmoe_slice_rows.argtypes = [i, i, i, bp, i, i, ip, fp, bp, ip, i]
    lib.mlpmoe_slice_rows.restype = i
    lib.mlpmoe_compact.argtypes = [vp, vp, vp, vp, i, i, i, i, vp, vp, vp, vp]
    lib.mlpmoe_compact.restype = i
    lib.mlpmoe_plan_create.argtypes = [ip, fp, bp, i, i, i, i, i, ctypes.POINTER(ctypes.c_void_p)]
    lib.mlpmoe_plan_create.restype = i
    lib.mlpmoe_plan_forward.argtypes = [vp, vp, vp, vp, vp, i, vp, vp]
    lib.mlpmoe_plan_forward.restype = i
    lib.mlpmoe_plan_destroy.argtypes = [vp]
    lib.mlpmoe_plan_destroy.restype = i
    lib.mlpmoe_forward_routed_bf16.argtypes = [vp, vp, vp, vp, ip, fp, bp, vp, i, i, i, i, vp, vp]
    lib.mlpmoe_forward_routed_bf16.restype = i
    lib.mlpmoe_forward_routed_bf16_ws.argtypes = [vp, vp, vp, vp, ip, fp, bp, vp, i, i, i, i, vp, vp, sz, vp]
    lib.mlpmoe_forward_routed_bf16_ws.restype = i
    lib.mlpmoe_forward_routed_f32.argtypes = lib.mlpmoe_forward_routed_bf16.argtypes
    lib.mlpmoe_forward_routed_f32.restype = i
    lib.mlpmoe_forward_routed_f32_ws.argtypes = lib.mlpmoe_forward_routed_bf16_ws.argtypes
    lib.mlpmoe_forward_routed_f32_ws.restype = i
    lib.mlpmoe_fade.argtypes = [vp, vp, ip, vp, i, i, i, i, vp, vp, vp]
    lib.mlpmoe_fade.restype = i
    lib.mlpmoe_fade_neurons.argtypes = [vp, vp, ip, ip, i, i, i, i, bp, ctypes.POINTER(ctypes.c_double), vp]
    lib.mlpmoe_fade_neurons.restype = i
    lib.mlpmoe_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.mlpmoe_workspace_bytes.restype = sz
    fwd = [vp, vp, vp, vp, ip, fp, bp, i, i, i, i, vp, vp]
    for name in ("mlpmoe_forward_bf16", "mlpmoe_forward", "mlpmoe_forward_f32", "mlpmoe_forward_bf16_noalloc"):
        getattr(lib, name).argtypes = fwd
        getattr(lib, name).restype = i
    lib.mlpmoe_forward_bf16_ws.argtypes = [vp, vp, vp, vp, ip, fp, bp, i, i, i, i, vp, vp, sz, i, vp]
    lib.mlpmoe_forward_bf16_ws.restype = i
    lib.mlpmoe_forward_bf16_out_bf16.argtypes = fwd
    lib.mlpmoe_forward_bf16_out_bf16.restype = i
    lib.mlpmoe_forward_bf16_out_bf16_ws.argtypes = [vp, vp, vp, vp, ip, fp, bp, i, i, i, i, vp, vp, sz, i, vp]
    lib.mlpmoe_forward_bf16_out_bf16_ws.restype = i
    lib.mlpmoe_forward_f32_ws.argtypes = [vp, vp, vp, vp, ip, fp, bp, i, i, i, i, vp, vp, sz, vp]
    lib.mlpmoe_forward_f32_ws.restype = i
    lib.mlpmoe_release.argtypes = []
    lib.mlpmoe_release.restype = i
    lib.mlpmoe_set_workspace.argtypes = [vp, sz]
    lib.mlpmoe_set_workspace.restype = i
    lib.mlpmoe_hidden_ld.argtypes = [i]
    lib.mlpmoe_hidden_ld.restype = i
    lib.mlpmoe_profile_enable.argtypes = [i]
    lib.mlpmoe_profile_enable.restype = i
    lib.mlpmoe_profile_collect.argtypes = [vp, vp, i]
    lib.mlpmoe_profile_collect.restype = i
    lib.mlpmoe_profile_disable.argtypes = []
    lib.mlpmoe_profile_disable.restype = i
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.mlpmoe_status_string(int(status)).decode()


def last_error_detail() -> str:
    """What the HIP runtime said when a call of this thread last failed with ERR_HIP ("" if none)."""
    return lib.mlpmoe_last_error_detail().decode()


def _check(status: int, where: str):
    if status != OK:
        raise MlpMoeError(status, where)


def _host(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _dev_ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


# --------------------------------------------------------------------------- host-only
def mlpmoe_slice(d_inter: int, B: int, K_keep: int = 0, neuron_keep=None, pad_to: int = 1, pad_rows_to: int = 1):
    """Branch table of one MLP.  Returns (branch_offsets[B+1], alpha[B], active_mask[B], gather_index).
    pad_rows_to > 1 goes through mlpmoe_slice_rows (row count of the compacted layer rounded up)."""
    n = max(int(B), 0)
    off = np.zeros(n + 1, dtype=np.int32)
    alpha = np.zeros(n, dtype=np.float32)
    mask = np.zeros(n, dtype=np.uint8)
    cap = max(int(d_inter), 0) + n * max(int(pad_to) - 1, 0) + max(int(pad_rows_to) - 1, 0)
    gather = np.full(max(cap, 1), -2, dtype=np.int32)
    keep = None if neuron_keep is None else _host(neuron_keep, np.uint8)
    if keep is not None and keep.shape != (d_inter,):
        raise ValueError("neuron_keep must have d_inter entries")
    if int(pad_rows_to) == 1:
        rc = lib.mlpmoe_slice(int(d_inter), int(B), int(K_keep), None if keep is None else keep.ctypes.data,
                              int(pad_to), off.ctypes.data, alpha.ctypes.data, mask.ctypes.data,
                              gather.ctypes.data, cap)
    else:
        rc = lib.mlpmoe_slice_rows(int(d_inter), int(B), int(K_keep), None if keep is None else keep.ctypes.data,
                                   int(pad_to), int(pad_rows_to), off.ctypes.data, alpha.ctypes.data,
                                   mask.ctypes.data, gather.ctypes.data, cap)
    _check(rc, "mlpmoe_slice")
    return off, alpha, mask, gather[: int(off[-1])].copy()


def mlpmoe_workspace_bytes(T, d_model, d_inter, B, elem_bytes=2) -> int:
    return int(lib.mlpmoe_workspace_bytes(int(T), int(d_model), int(d_inter), int(B), int(elem_bytes)))


# --------------------------------------------------------------------------- device
def mlpmoe_compact(W_gate, W_up, W_down, gather_index, stream=None):
    """Compacted copies of the three weight matrices (rows of gate/up, columns of down)."""
    import torch
    d_inter_src, d_model = W_gate.shape
    g = gather_index if hasattr(gather_index, "is_cuda") else torch.as_tensor(
        np.ascontiguousarray(gather_index, dtype=np.int32), device=W_gate.device)
    n_rows = int(g.numel())
    Wg_c = torch.empty((n_rows, d_model), dtype=W_gate.dtype, device=W_gate.device)
    Wu_c = torch.empty((n_rows, d_model), dtype=W_gate.dtype, device=W_gate.device)
    Wd_c = torch.empty((d_model, n_rows), dtype=W_gate.dtype, device=W_gate.device)
    rc = lib.mlpmoe_compact(_dev_ptr(W_gate), _dev_ptr(W_up), _dev_ptr(W_down), _dev_ptr(g), n_rows,
                            int(d_model), int(d_inter_src), int(W_gate.element_size()),
                            _dev_ptr(Wg_c), _dev_ptr(Wu_c), _dev_ptr(Wd_c), _stream_ptr(stream))
    _check(rc, "mlpmoe_compact")
    return Wg_c, Wu_c, Wd_c


def mlpmoe_fade(W_gate, W_up, branch_offsets, sparsity=None, stream=None):
    """Fractal Fade (Sec. 3.2) of W_gate and W_up in place on the device.

    Returns (thresholds [B, 2] float32 with NaN for untouched branches, kept [B, 2] int64).
    """
    off = _host(branch_offsets, np.int32)
    B = off.shape[0] - 1
    d_inter, d_model = W_gate.shape
    sp = None
    if sparsity is not None:
        sp = np.ascontiguousarray(sparsity, dtype=np.float64)
        if sp.shape != (B,):
            raise ValueError("sparsity needs B entries")
    thr = np.zeros((B, 2), dtype=np.float32)
    kept = np.zeros((B, 2), dtype=np.int64)
    rc = lib.mlpmoe_fade(_dev_ptr(W_gate), _dev_ptr(W_up), off.ctypes.data,
                         sp.ctypes.data if sp is not None else None, int(d_model), int(d_inter), int(B),
                         int(W_gate.element_size()), thr.ctypes.data, kept.ctypes.data, _stream_ptr(stream))
    _check(rc, "mlpmoe_fade")
    return thr, kept


def mlpmoe_fade_neurons(W_gate, W_up, branch_offsets, keep_count, stream=None):
    """Structured form of the fade: branch b keeps its keep_count[b] neurons with the largest squared norm of
    gate and up row together.  Returns (neuron_keep [d_inter] uint8, scores [d_inter] float64); feed
    neuron_keep to mlpmoe_slice and the gather list it returns to mlpmoe_compact."""
    off = _host(branch_offsets, np.int32)
    B = off.shape[0] - 1
    cnt = _host(keep_count, np.int32)
    if cnt.shape != (B,):
        raise ValueError("keep_count needs B entries")
    d_inter, d_model = W_gate.shape
    keep = np.zeros(max(int(d_inter), 1), dtype=np.uint8)
    scores = np.zeros(max(int(d_inter), 1), dtype=np.float64)
    rc = lib.mlpmoe_fade_neurons(_dev_ptr(W_gate), _dev_ptr(W_up), off.ctypes.data, cnt.ctypes.data, int(d_model),
                                 int(d_inter), int(B), int(W_gate.element_size()), keep.ctypes.data,
                                 scores.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), _stream_ptr(stream))
    _check(rc, "mlpmoe_fade_neurons")
    return keep[:d_inter], scores[:d_inter]


def _table(branch_offsets, alpha, active_mask):
    off = _host(branch_offsets, np.int32)
    al = _host(alpha, np.float32)
    mk = _host(active_mask, np.uint8)
    B = off.shape[0] - 1
    if al.shape != (B,) or mk.shape != (B,):
        raise ValueError("alpha and active_mask need B entries, branch_offsets B+1")
    return off, al, mk, B


def _forward(name, x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out, stream,
             workspace=None, path=None, out_dtype=None):
    import torch
    off, al, mk, B = _table(branch_offsets, alpha, active_mask)
    T, d_model = x.shape
    d_inter = W_gate.shape[0]
    out_dtype = torch.float32 if out_dtype is None else out_dtype
    if out is None:
        out = torch.empty((T, d_model), dtype=out_dtype, device=x.device)
    elif out.dtype != out_dtype or tuple(out.shape) != (T, d_model) or not out.is_contiguous():
        raise ValueError("out must be a contiguous [T, d_model] tensor of %s" % out_dtype)
    args = [_dev_ptr(x), _dev_ptr(W_gate), _dev_ptr(W_up), _dev_ptr(W_down), off.ctypes.data,
            al.ctypes.data, mk.ctypes.data, int(T), int(d_model), int(d_inter), int(B), _dev_ptr(out)]
    if workspace is not None:
        args += [_dev_ptr(workspace), workspace.numel() * workspace.element_size()]
        if path is not None:
            args.append(int(path))
    args.append(_stream_ptr(stream))
    _check(getattr(lib, name)(*args), name)
    return out


def mlpmoe_forward_bf16(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out=None, stream=None):
    return _forward("mlpmoe_forward_bf16", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out, stream)


def mlpmoe_forward(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out=None, stream=None):
    return _forward("mlpmoe_forward", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out, stream)


def mlpmoe_forward_f32(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out=None, stream=None):
    return _forward("mlpmoe_forward_f32", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out, stream)


NOALLOC_SCRATCH_BYTES = 16 << 20


def mlpmoe_forward_bf16_noalloc(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out, stream=None):
    """The bf16 forward in the library's fixed scratch block: allocates nothing (out must be given)."""
    if out is None:
        raise ValueError("mlpmoe_forward_bf16_noalloc needs the output tensor")
    return _forward("mlpmoe_forward_bf16_noalloc", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out,
                    stream)


def mlpmoe_forward_bf16_ws(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, workspace,
                           path=PATH_AUTO, out=None, stream=None):
    return _forward("mlpmoe_forward_bf16_ws", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask,
                    out, stream, workspace=workspace, path=path)


def mlpmoe_forward_bf16_out_bf16(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, out=None, stream=None):
    """The bf16 forward with the result rounded once to bf16 (out: [T, d_model] torch.bfloat16)."""
    import torch
    return _forward("mlpmoe_forward_bf16_out_bf16", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask,
                    out, stream, out_dtype=torch.bfloat16)


def mlpmoe_forward_bf16_out_bf16_ws(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, workspace,
                                    path=PATH_AUTO, out=None, stream=None):
    import torch
    return _forward("mlpmoe_forward_bf16_out_bf16_ws", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask,
                    out, stream, workspace=workspace, path=path, out_dtype=torch.bfloat16)


def mlpmoe_forward_f32_ws(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, workspace,
                          out=None, stream=None):
    return _forward("mlpmoe_forward_f32_ws", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask,
                    out, stream, workspace=workspace)


def mlpmoe_release():
    _check(lib.mlpmoe_release(), "mlpmoe_release")


def mlpmoe_set_workspace(workspace):
    """Caller-owned workspace (a torch byte tensor on the current device) for the entry points that take none;
    None clears it.  The caller keeps the tensor alive while it is set."""
    if workspace is None:
        _check(lib.mlpmoe_set_workspace(None, 0), "mlpmoe_set_workspace")
    else:
        _check(lib.mlpmoe_set_workspace(_dev_ptr(workspace), int(workspace.numel() * workspace.element_size())),
               "mlpmoe_set_workspace")


def mlpmoe_hidden_ld(d_inter: int) -> int:
    """Leading dimension of the gated intermediate H at the start of a workspace."""
    return int(lib.mlpmoe_hidden_ld(int(d_inter)))


def mlpmoe_forward_routed_f32(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, out=None,
                              workspace=None, stream=None):
    """The routed forward for float32 x and weights."""
    return _forward_routed("mlpmoe_forward_routed_f32", x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask,
                           route, out, workspace, stream)


def mlpmoe_forward_routed_bf16(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, out=None,
                               workspace=None, stream=None):
    """Forward with a per-token branch set: route is a [T, B] uint8 GPU tensor (nonzero = token takes branch)."""
    return _forward_routed("mlpmoe_forward_routed_bf16", x, W_gate, W_up, W_down, branch_offsets, alpha,
                           active_mask, route, out, workspace, stream)


def _forward_routed(name, x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, out, workspace, stream):
    import torch
    off, al, mk, B = _table(branch_offsets, alpha, active_mask)
    T, d_model = int(x.shape[0]), int(x.shape[1])
    d_inter = int(off[-1])
    if route.dtype != torch.uint8 or tuple(route.shape) != (T, B):
        raise ValueError("route must be a [T, B] uint8 tensor")
    if out is None:
        out = torch.empty((T, d_model), dtype=torch.float32, device=x.device)
    common = (_dev_ptr(x), _dev_ptr(W_gate), _dev_ptr(W_up), _dev_ptr(W_down), off.ctypes.data, al.ctypes.data,
              mk.ctypes.data, _dev_ptr(route) if T else None, T, d_model, d_inter, B, _dev_ptr(out))
    if workspace is None:
        _check(getattr(lib, name)(*common, _stream_ptr(stream)), name)
    else:
        _check(getattr(lib, name + "_ws")(*common, _dev_ptr(workspace), int(workspace.numel() * workspace.element_size()),
                                          _stream_ptr(stream)), name + "_ws")
    return out


class Plan:
    """A layer's branch table prepared once, with a device workspace for any T <= max_T."""

    def __init__(self, branch_offsets, alpha, active_mask, d_model, d_inter, max_T, elem_bytes=2):
        off, al, mk, B = _table(branch_offsets, alpha, active_mask)
        self.d_model, self.d_inter, self.max_T = int(d_model), int(d_inter), int(max_T)
        self._h = ctypes.c_void_p()
        _check(lib.mlpmoe_plan_create(off.ctypes.data, al.ctypes.data, mk.ctypes.data, self.d_model, self.d_inter,
                                      B, int(elem_bytes), self.max_T, ctypes.byref(self._h)), "mlpmoe_plan_create")

    def forward(self, x, W_gate, W_up, W_down, out=None, stream=None):
        import torch
        T = int(x.shape[0])
        if out is None:
            out = torch.empty((T, self.d_model), dtype=torch.float32, device=x.device)
        _check(lib.mlpmoe_plan_forward(self._h, _dev_ptr(x), _dev_ptr(W_gate), _dev_ptr(W_up), _dev_ptr(W_down), T,
                                       _dev_ptr(out), _stream_ptr(stream)), "mlpmoe_plan_forward")
        return out

    def destroy(self):
        if self._h:
            h, self._h = self._h, ctypes.c_void_p()
            _check(lib.mlpmoe_plan_destroy(h), "mlpmoe_plan_destroy")

    def __del__(self):
        # At interpreter shutdown the HIP runtime may already be tearing down: leave the block to the
        # process exit rather than calling into the runtime from a finaliser.
        import sys
        if sys is None or sys.is_finalizing():
            return
        try:
            self.destroy()
        except Exception:
            pass


KERNEL_NAMES = {1: "gate_up_mfma", 2: "down_mfma", 3: "splitk_reduce", 4: "decode_gate_up",
                5: "decode_down", 6: "gate_up_generic", 7: "down_generic", 8: "fill_zero",
                9: "route_tiles"}


def mlpmoe_profile_enable(capacity: int):
    _check(lib.mlpmoe_profile_enable(int(capacity)), "mlpmoe_profile_enable")


def mlpmoe_profile_collect(capacity: int):
    """Returns [(kernel_name, milliseconds), ...] in launch order and clears the record list."""
    ids = np.zeros(capacity, dtype=np.int32)
    ms = np.zeros(capacity, dtype=np.float32)
    n = lib.mlpmoe_profile_collect(ids.ctypes.data, ms.ctypes.data, int(capacity))
    if n < 0:
        raise MlpMoeError(n, "mlpmoe_profile_collect")
    return [(KERNEL_NAMES.get(int(ids[k]), str(ids[k])), float(ms[k])) for k in range(n)]


def mlpmoe_profile_disable():
    _check(lib.mlpmoe_profile_disable(), "mlpmoe_profile_disable")


def new_workspace(T, d_model, d_inter, B, elem_bytes=2, device="cuda"):
    """A torch byte tensor large enough for one forward call (256-byte aligned by the allocator)."""
    import torch
    return torch.empty(mlpmoe_workspace_bytes(T, d_model, d_inter, B, elem_bytes), dtype=torch.uint8,
                       device=device)


def bf16_tensor(bits: np.ndarray, device="cuda"):
    """Upload bf16 bit patterns (uint16 numpy) as a torch.bfloat16 tensor."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.bfloat16)
