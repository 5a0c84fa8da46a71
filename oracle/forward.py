"""ctypes front end of oracle/mlpmoe_oracle.c (plain C, double accumulation).

Test infrastructure: see the header of mlpmoe_oracle.c.  The shared object is
compiled with gcc on first use (or by build_oracle()); it links nothing but
libm and libgomp.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mlpmoe_oracle.c")
_SO = os.path.join(_HERE, "libmlpmoe_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc; returns the path of the shared object."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-Wall", "-Wextra", "-shared",
                               "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        bp = ctypes.POINTER(ctypes.c_uint8)
        lib.oracle_mlpmoe_forward.argtypes = [fp, fp, fp, fp, ip, fp, bp] + [ctypes.c_int] * 5 + [dp]
        lib.oracle_mlpmoe_forward.restype = ctypes.c_int
        lib.oracle_mlpmoe_forward_routed.argtypes = [fp, fp, fp, fp, ip, fp, bp, bp] + [ctypes.c_int] * 5 + [dp]
        lib.oracle_mlpmoe_forward_routed.restype = ctypes.c_int
        lib.oracle_mlpmoe_hidden.argtypes = [fp, fp, fp, ip, fp, bp] + [ctypes.c_int] * 5 + [dp] * 5
        lib.oracle_mlpmoe_hidden.restype = ctypes.c_int
        lib.oracle_dense_swiglu.argtypes = [fp, fp, fp, fp] + [ctypes.c_int] * 3 + [dp]
        lib.oracle_dense_swiglu.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.shape != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a


def _ptr(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def mlpmoe_forward(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, mode="exact"):
    """sum_b alpha_b W_down^(b)[SiLU(W_gate^(b) x) * W_up^(b) x]  (Sec. 3.1), fp64 result [T,d_model].

    x [T,d_model], W_gate/W_up [d_inter,d_model], W_down [d_model,d_inter], all float32 values
    (bf16 inputs are widened by the caller).  mode: "exact" or "contract" (one bf16 rounding of
    alpha_b*h, see the C header).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, d_model = x.shape
    off = np.ascontiguousarray(branch_offsets, dtype=np.int32)
    B = off.shape[0] - 1
    d_inter = int(off[-1])
    Wg = _f32(W_gate, (d_inter, d_model))
    Wu = _f32(W_up, (d_inter, d_model))
    Wd = _f32(W_down, (d_model, d_inter))
    al = _f32(alpha, (B,))
    mk = np.ascontiguousarray(active_mask, dtype=np.uint8)
    if mk.shape != (B,):
        raise ValueError("active_mask must have B entries")
    out = np.empty((T, d_model), dtype=np.float64)
    m = {"exact": 0, "contract": 1}[mode]
    rc = _load().oracle_mlpmoe_forward(_ptr(x, ctypes.c_float), _ptr(Wg, ctypes.c_float),
                                       _ptr(Wu, ctypes.c_float), _ptr(Wd, ctypes.c_float),
                                       _ptr(off, ctypes.c_int32), _ptr(al, ctypes.c_float),
                                       _ptr(mk, ctypes.c_uint8), T, d_model, d_inter, B, m,
                                       _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_mlpmoe_forward rejected its arguments (rc=%d)" % rc)
    return out


def mlpmoe_forward_routed(x, W_gate, W_up, W_down, branch_offsets, alpha, active_mask, route, mode="exact"):
    """The branched forward with a per-token branch set: token t sums the branches b with
    active_mask[b] and route[t, b] nonzero (route: [T, B] uint8).  Same modes as mlpmoe_forward."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, d_model = x.shape
    off = np.ascontiguousarray(branch_offsets, dtype=np.int32)
    B = off.shape[0] - 1
    d_inter = int(off[-1])
    Wg = _f32(W_gate, (d_inter, d_model))
    Wu = _f32(W_up, (d_inter, d_model))
    Wd = _f32(W_down, (d_model, d_inter))
    al = _f32(alpha, (B,))
    mk = np.ascontiguousarray(active_mask, dtype=np.uint8)
    rt = np.ascontiguousarray(route, dtype=np.uint8)
    if mk.shape != (B,) or rt.shape != (T, B):
        raise ValueError("active_mask must have B entries and route T x B")
    out = np.empty((T, d_model), dtype=np.float64)
    m = {"exact": 0, "contract": 1}[mode]
    rc = _load().oracle_mlpmoe_forward_routed(_ptr(x, ctypes.c_float), _ptr(Wg, ctypes.c_float),
                                              _ptr(Wu, ctypes.c_float), _ptr(Wd, ctypes.c_float),
                                              _ptr(off, ctypes.c_int32), _ptr(al, ctypes.c_float),
                                              _ptr(mk, ctypes.c_uint8), _ptr(rt, ctypes.c_uint8), T, d_model,
                                              d_inter, B, m, _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_mlpmoe_forward_routed rejected its arguments (rc=%d)" % rc)
    return out


def mlpmoe_hidden(x, W_gate, W_up, branch_offsets, alpha, active_mask, mode="exact", details=False):
    """The gated intermediate alpha_b * SiLU(W_gate x) * W_up x of Sec. 3.1's bracket, [T, d_inter] fp64
    (0 for neurons of inactive branches).  mode "contract": formed in float and rounded once to bf16.
    details=True also returns (g, u, abs_g, abs_u): the two dot products and the sums of the
    absolute values of their terms."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, d_model = x.shape
    off = np.ascontiguousarray(branch_offsets, dtype=np.int32)
    B = off.shape[0] - 1
    d_inter = int(off[-1])
    Wg = _f32(W_gate, (d_inter, d_model))
    Wu = _f32(W_up, (d_inter, d_model))
    al = _f32(alpha, (B,))
    mk = np.ascontiguousarray(active_mask, dtype=np.uint8)
    if mk.shape != (B,):
        raise ValueError("active_mask must have B entries")
    h = np.empty((T, d_inter), dtype=np.float64)
    extra = [np.empty((T, d_inter), dtype=np.float64) for _ in range(4)] if details else [None] * 4
    m = {"exact": 0, "contract": 1}[mode]
    rc = _load().oracle_mlpmoe_hidden(_ptr(x, ctypes.c_float), _ptr(Wg, ctypes.c_float), _ptr(Wu, ctypes.c_float),
                                      _ptr(off, ctypes.c_int32), _ptr(al, ctypes.c_float), _ptr(mk, ctypes.c_uint8),
                                      T, d_model, d_inter, B, m, _ptr(h, ctypes.c_double),
                                      *[None if e is None else _ptr(e, ctypes.c_double) for e in extra])
    if rc != 0:
        raise ValueError("oracle_mlpmoe_hidden rejected its arguments (rc=%d)" % rc)
    return (h, *extra) if details else h


def dense_swiglu(x, W_gate, W_up, W_down):
    """W_down [SiLU(W_gate x) * W_up x] with no branch structure (Sec. 2.2, left-hand side)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, d_model = x.shape
    d_inter = np.asarray(W_gate).shape[0]
    Wg = _f32(W_gate, (d_inter, d_model))
    Wu = _f32(W_up, (d_inter, d_model))
    Wd = _f32(W_down, (d_model, d_inter))
    out = np.empty((T, d_model), dtype=np.float64)
    rc = _load().oracle_dense_swiglu(_ptr(x, ctypes.c_float), _ptr(Wg, ctypes.c_float),
                                     _ptr(Wu, ctypes.c_float), _ptr(Wd, ctypes.c_float),
                                     T, d_model, d_inter, _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_dense_swiglu rejected its arguments (rc=%d)" % rc)
    return out


def num_threads() -> int:
    """Threads the oracle's token loop runs on."""
    return int(_load().oracle_num_threads())


def rel_max_err(got, ref) -> float:
    """The parity metric: max |got - ref| / rms(ref)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    num = float(np.max(np.abs(got - ref)))
    if rms == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / rms


def round_to_bf16(a):
    """Values of `a` rounded to the nearest bfloat16 (ties to even), returned as float64.

    From the format's definition (1 sign, 8 exponent, 7 fraction bits, the exponent range of
    binary32): a normal magnitude m * 2^e with m in [0.5, 1) keeps 8 significant bits, i.e. it is
    rint(m * 256) / 256 * 2^e; below 2^-126 the spacing is the fixed 2^-133; magnitudes that round to
    2^128 or more become infinite.  numpy's rint rounds halves to even.  Used for the forward whose
    result is stored as bf16: the sum of Sec. 3.1 rounded once."""
    a = np.asarray(a, dtype=np.float64)
    mag = np.abs(a)
    m, e = np.frexp(mag)
    normal = np.ldexp(np.rint(m * 256.0) / 256.0, e)
    sub = np.rint(mag / 2.0 ** -133) * 2.0 ** -133
    r = np.where(mag < 2.0 ** -126, sub, normal)
    r = np.where(r >= 2.0 ** 128, np.inf, r)
    r = np.where(np.isfinite(mag), r, mag)          # inf and nan pass through
    return np.copysign(r, a)
