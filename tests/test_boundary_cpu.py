"""Host-side checks of the C-ABI library that need no GPU: exported symbols, the slicing
call against its oracle, and argument validation (errors are reported before any GPU work)."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import oracle
from paper_2511_21089_amd import binding as mm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            names += re.findall(r"MLPMOE_API\s+[\w\s\*]+?\b(mlpmoe_\w+)\s*\(", text)
    return names


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 10 and len(set(names)) == len(names)
    for n in names:
        assert hasattr(mm.lib, n), n
    assert sorted(names) == sorted(mm.EXPORTS)


def test_binding_signatures_match_the_header():
    """Every exported function has ctypes argument types, as many as the header declares, with
    pointers, size_t and int in the same places (an undeclared signature would pass 64-bit
    pointers as C ints)."""
    import ctypes
    text = "".join(open(os.path.join(ROOT, "include", fn)).read()
                   for fn in sorted(os.listdir(os.path.join(ROOT, "include"))) if fn.endswith(".h"))
    decls = re.findall(r"MLPMOE_API\s+([\w\s\*]+?)\b(mlpmoe_\w+)\s*\(([^;]*?)\)\s*;", text, flags=re.S)
    assert len(decls) == len(mm.EXPORTS)
    for ret, name, params in decls:
        params = [p.strip() for p in params.replace("\n", " ").split(",")]
        if params == ["void"]:
            params = []
        fn = getattr(mm.lib, name)
        assert fn.argtypes is not None, name
        assert len(fn.argtypes) == len(params), (name, len(fn.argtypes), params)
        for want, p in zip(fn.argtypes, params):
            is_ptr = "*" in p
            got_ptr = want is ctypes.c_void_p or want is ctypes.c_char_p or hasattr(want, "contents")
            assert is_ptr == got_ptr, (name, p, want)
            if not is_ptr:
                assert (want is ctypes.c_size_t) == p.startswith("size_t"), (name, p, want)
                assert (want is ctypes.c_int) == p.startswith("int"), (name, p, want)
        if "char" in ret:
            assert fn.restype is ctypes.c_char_p, name
        elif "size_t" in ret:
            assert fn.restype is ctypes.c_size_t, name
        else:
            assert fn.restype is ctypes.c_int, name


def test_status_strings():
    assert mm.status_string(0) == "ok"
    for code in range(-7, 0):
        assert mm.status_string(code) not in ("ok", "unknown status")
    assert mm.status_string(-99) == "unknown status"


@pytest.mark.parametrize("d_inter,B,K,pad", [(4864, 8, 0, 1), (4864, 8, 6, 1), (14336, 16, 0, 8), (100, 7, 3, 4),
                                             (5, 8, 0, 1), (4864, 16, 16, 1), (14336, 32, 24, 32), (0, 3, 0, 1)])
def test_slice_matches_oracle(d_inter, B, K, pad):
    rng = np.random.default_rng(d_inter + B)
    for keep in (None, (rng.uniform(size=d_inter) < 0.7).astype(np.uint8)):
        off, alpha, mask, gather = mm.mlpmoe_slice(d_inter, B, K, keep, pad)
        o_off, o_alpha, o_mask, o_gather = oracle.slice_plan(d_inter, B, K, keep, pad)
        assert np.array_equal(off, o_off)
        assert np.array_equal(mask, o_mask)
        assert np.array_equal(gather, o_gather)
        assert np.allclose(alpha, o_alpha, rtol=1e-7, atol=0)
        assert np.all(np.diff(off) % pad == 0)
        # the row count of the whole layer rounded up as well: more padding rows at the end of the last branch
        for rows_to in (64, 5):
            off_r, alpha_r, mask_r, gather_r = mm.mlpmoe_slice(d_inter, B, K, keep, pad, rows_to)
            o_off, _, _, o_gather = oracle.slice_plan(d_inter, B, K, keep, pad, rows_to)
            assert np.array_equal(off_r, o_off) and np.array_equal(gather_r, o_gather)
            assert off_r[-1] % rows_to == 0 and 0 <= off_r[-1] - off[-1] < rows_to
            assert np.array_equal(off_r[:-1], off[:-1]) and np.array_equal(gather_r[:len(gather)], gather)
            assert np.all(gather_r[len(gather):] == -1)
            assert np.array_equal(alpha_r, alpha) and np.array_equal(mask_r, mask)


def test_slice_compensated_alpha_closed_form():
    _, alpha, mask, _ = mm.mlpmoe_slice(4864, 8, 6)
    assert alpha[0] == np.float32(math.sqrt(8 / 6)) and alpha[7] == 0 and list(mask) == [1] * 6 + [0, 0]


def test_slice_errors():
    off = np.zeros(5, np.int32)
    al = np.zeros(4, np.float32)
    mk = np.zeros(4, np.uint8)
    f = mm.lib.mlpmoe_slice
    assert f(16, 4, 0, None, 1, None, al.ctypes.data, mk.ctypes.data, None, 0) == mm.ERR_NULL
    assert f(16, 0, 0, None, 1, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.ERR_SHAPE
    assert f(16, 65, 0, None, 1, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.ERR_SHAPE
    assert f(-1, 4, 0, None, 1, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.ERR_SHAPE
    g = mm.lib.mlpmoe_slice_rows
    assert g(16, 4, 0, None, 1, 0, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.ERR_SHAPE
    assert g(16, 4, 0, None, 1, 4097, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.ERR_SHAPE
    small = np.zeros(17, np.int32)       # 16 rows rounded up to 64 do not fit 17 entries
    assert g(16, 4, 0, None, 1, 64, off.ctypes.data, al.ctypes.data, mk.ctypes.data, small.ctypes.data, 17) == mm.ERR_SHAPE
    assert g(16, 4, 0, None, 1, 64, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.OK and off[4] == 64
    assert f(16, 4, 0, None, 0, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.ERR_SHAPE
    g = np.zeros(8, np.int32)
    assert f(16, 4, 0, None, 1, off.ctypes.data, al.ctypes.data, mk.ctypes.data, g.ctypes.data, 8) == mm.ERR_SHAPE
    assert f(16, 4, 0, None, 1, off.ctypes.data, al.ctypes.data, mk.ctypes.data, None, 0) == mm.OK


def test_workspace_bytes():
    assert mm.mlpmoe_workspace_bytes(0, 64, 256, 4) > 0
    assert mm.mlpmoe_workspace_bytes(-1, 64, 256, 4) == 0
    assert mm.mlpmoe_workspace_bytes(4, 64, 256, 4, elem_bytes=3) == 0
    a = mm.mlpmoe_workspace_bytes(4096, 4096, 14336, 16)
    assert a >= 4096 * 14336 * 2


def test_set_workspace_validation_and_hidden_ld():
    f = mm.lib.mlpmoe_set_workspace
    assert f(ctypes.c_void_p(0x1010), 4096) == mm.ERR_WORKSPACE      # not 256-byte aligned
    assert f(ctypes.c_void_p(0x1000), 0) == mm.ERR_WORKSPACE         # a block of no bytes
    assert mm.mlpmoe_hidden_ld(4864) == 4864 and mm.mlpmoe_hidden_ld(4870) == 4928
    assert mm.mlpmoe_hidden_ld(0) == 64 and mm.mlpmoe_hidden_ld(-1) == 0
    # leading dimensions beyond what the kernels' 32-bit row offsets hold are refused up front
    off = np.array([0, (1 << 22) + 8], np.int32)
    al = np.ones(1, np.float32)
    mk = np.ones(1, np.uint8)
    vp = ctypes.c_void_p
    assert mm.lib.mlpmoe_forward_bf16(vp(0x1000), vp(0x1000), vp(0x1000), vp(0x1000), off.ctypes.data, al.ctypes.data,
                                      mk.ctypes.data, 4, 64, (1 << 22) + 8, 1, vp(0x1000), None) == mm.ERR_SHAPE


def _fwd_args(off, al, mk, T=4, d_model=64, d_inter=256, B=4, x=0x1000, w=0x1000, out=0x1000):
    vp = ctypes.c_void_p
    return [vp(x), vp(w), vp(w), vp(w), off.ctypes.data, al.ctypes.data, mk.ctypes.data, T, d_model,
            d_inter, B, vp(out)]


def test_forward_argument_validation_needs_no_gpu():
    """Bad arguments are rejected on the host; the fake device addresses are never touched."""
    off = np.array([0, 64, 128, 192, 256], np.int32)
    al = np.ones(4, np.float32)
    mk = np.ones(4, np.uint8)
    ws = [ctypes.c_void_p(0x1000), 1 << 30, mm.PATH_AUTO, None]
    f = mm.lib.mlpmoe_forward_bf16_ws
    assert f(*(_fwd_args(off, al, mk, B=0) + ws)) == mm.ERR_SHAPE
    assert f(*(_fwd_args(off, al, mk, B=65) + ws)) == mm.ERR_SHAPE
    assert f(*(_fwd_args(off, al, mk, T=-1) + ws)) == mm.ERR_SHAPE
    assert f(*(_fwd_args(off, al, mk, d_model=0) + ws)) == mm.ERR_SHAPE
    assert f(*(_fwd_args(off, al, mk, d_inter=255) + ws)) == mm.ERR_OFFSETS
    bad = off.copy()
    bad[0] = 1
    assert f(*(_fwd_args(bad, al, mk) + ws)) == mm.ERR_OFFSETS
    bad = np.array([0, 128, 64, 192, 256], np.int32)
    assert f(*(_fwd_args(bad, al, mk) + ws)) == mm.ERR_OFFSETS
    assert f(*(_fwd_args(off, al, mk, x=0) + ws)) == mm.ERR_NULL
    assert f(*(_fwd_args(off, al, mk, out=0) + ws)) == mm.ERR_NULL
    assert f(*(_fwd_args(off, al, mk, w=0) + ws)) == mm.ERR_NULL
    assert f(*(_fwd_args(off, al, mk, x=0x1008) + ws)) == mm.ERR_ALIGN
    a = _fwd_args(off, al, mk)
    a[4] = None
    assert f(*(a + ws)) == mm.ERR_NULL
    # T == 0 is a successful no-op even with null tensors
    assert f(*(_fwd_args(off, al, mk, T=0, x=0, out=0) + ws)) == mm.OK
    assert mm.lib.mlpmoe_forward_f32_ws(*(_fwd_args(off, al, mk, T=0) + ws[:2] + [None])) == mm.OK
    # workspace problems and impossible paths are host-side errors too
    assert f(*(_fwd_args(off, al, mk) + [None, 0, mm.PATH_AUTO, None])) == mm.ERR_WORKSPACE
    assert f(*(_fwd_args(off, al, mk) + [ctypes.c_void_p(0x1000), 16, mm.PATH_AUTO, None])) == mm.ERR_WORKSPACE
    assert f(*(_fwd_args(off, al, mk) + [ctypes.c_void_p(0x1010), 1 << 30, mm.PATH_AUTO, None])) == mm.ERR_WORKSPACE
    assert f(*(_fwd_args(off, al, mk) + [ctypes.c_void_p(0x1000), 1 << 30, mm.PATH_MFMA_SLIM + 1, None])) == mm.ERR_UNSUPPORTED
    assert f(*(_fwd_args(off, al, mk, T=17) + [ctypes.c_void_p(0x1000), 1 << 30, mm.PATH_DECODE, None])) == mm.ERR_UNSUPPORTED
    odd = np.array([0, 60, 128, 192, 256], np.int32)      # branch boundary not a multiple of 8 ...
    mk2 = np.array([1, 0, 1, 1], np.uint8)                # ... and exposed as a run boundary
    assert f(*(_fwd_args(odd, al, mk2) + [ctypes.c_void_p(0x1000), 1 << 30, mm.PATH_MFMA, None])) == mm.ERR_UNSUPPORTED


def test_routed_and_bf16_out_argument_validation():
    """The routed and the bf16-result entry points reject bad arguments on the host like the plain ones."""
    vp = ctypes.c_void_p
    off = np.array([0, 64, 128, 192, 256], np.int32)
    al = np.ones(4, np.float32)
    mk = np.ones(4, np.uint8)
    ws = [vp(0x1000), 1 << 30]

    def routed(route=0x1000, **kw):
        a = _fwd_args(off, al, mk, **kw)
        return a[:7] + [vp(route)] + a[7:]

    f = mm.lib.mlpmoe_forward_routed_bf16_ws
    assert f(*(routed(B=0) + ws + [None])) == mm.ERR_SHAPE
    assert f(*(routed(x=0) + ws + [None])) == mm.ERR_NULL
    assert f(*(routed(route=0) + ws + [None])) == mm.ERR_NULL
    assert f(*(routed(x=0x1004) + ws + [None])) == mm.ERR_ALIGN
    assert f(*(routed(T=0, x=0, out=0, route=0) + ws + [None])) == mm.OK
    assert f(*(routed() + [None, 0, None])) == mm.ERR_WORKSPACE
    assert f(*(routed() + [vp(0x1000), 64, None])) == mm.ERR_WORKSPACE
    assert mm.lib.mlpmoe_forward_routed_bf16(*(routed(T=-1) + [None])) == mm.ERR_SHAPE
    assert mm.lib.mlpmoe_forward_routed_bf16(*(routed(T=0, x=0, out=0, route=0) + [None])) == mm.OK

    g = mm.lib.mlpmoe_forward_bf16_out_bf16_ws
    tail = ws + [mm.PATH_AUTO, None]
    assert g(*(_fwd_args(off, al, mk, d_model=0) + tail)) == mm.ERR_SHAPE
    assert g(*(_fwd_args(off, al, mk, out=0) + tail)) == mm.ERR_NULL
    assert g(*(_fwd_args(off, al, mk, out=0x1002) + tail)) == mm.ERR_ALIGN
    assert g(*(_fwd_args(off, al, mk, T=0, x=0, out=0) + tail)) == mm.OK
    assert g(*(_fwd_args(off, al, mk) + [vp(0x1000), 16, mm.PATH_AUTO, None])) == mm.ERR_WORKSPACE
    assert g(*(_fwd_args(off, al, mk, T=17) + ws + [mm.PATH_DECODE, None])) == mm.ERR_UNSUPPORTED
    assert mm.lib.mlpmoe_forward_bf16_out_bf16(*(_fwd_args(off, al, mk, B=99) + [None])) == mm.ERR_SHAPE
    # the workspace of a routed call is part of the common size
    assert mm.mlpmoe_workspace_bytes(4096, 4096, 14336, 16) > 4096 * 14336 * 2 + 16 * 64


def test_compact_validation():
    vp = ctypes.c_void_p
    f = mm.lib.mlpmoe_compact
    assert f(vp(16), vp(16), vp(16), vp(16), 4, 8, 8, 3, vp(16), vp(16), vp(16), None) == mm.ERR_SHAPE
    assert f(vp(16), vp(16), vp(16), vp(16), -1, 8, 8, 2, vp(16), vp(16), vp(16), None) == mm.ERR_SHAPE
    assert f(None, vp(16), vp(16), vp(16), 4, 8, 8, 2, vp(16), vp(16), vp(16), None) == mm.ERR_NULL
    assert f(None, None, None, None, 0, 8, 8, 2, None, None, None, None) == mm.OK


def test_fade_argument_validation():
    """mlpmoe_fade refuses bad tables and unsupported storage before touching the GPU."""
    import ctypes
    lib = mm.lib
    off = np.array([0, 8, 16], np.int32)
    fake = ctypes.c_void_p(0x1000)
    call = lambda offs, sp, dm, di, B, eb, wg=fake: lib.mlpmoe_fade(
        wg, fake, offs.ctypes.data, sp.ctypes.data if sp is not None else None, dm, di, B, eb, None, None, None)
    assert call(off, None, 64, 16, 0, 2) == mm.ERR_SHAPE
    assert call(off, None, 64, 17, 2, 2) == mm.ERR_OFFSETS
    assert call(np.array([0, 9, 8], np.int32), None, 64, 8, 2, 2) == mm.ERR_OFFSETS
    assert call(off, np.array([0.0, 1.5]), 64, 16, 2, 2) == mm.ERR_SHAPE
    assert call(off, np.array([0.0, float("nan")]), 64, 16, 2, 2) == mm.ERR_SHAPE
    assert call(off, None, 64, 16, 2, 8) == mm.ERR_UNSUPPORTED          # neither bf16 nor float storage
    assert call(off, None, 60, 16, 2, 2) == mm.ERR_UNSUPPORTED          # bf16: d_model not a multiple of 8
    assert call(off, None, 62, 16, 2, 4) == mm.ERR_UNSUPPORTED          # float: not a multiple of 4
    assert call(off, None, 64, 16, 2, 2, ctypes.c_void_p(0x1004)) == mm.ERR_ALIGN
    assert call(off, None, 64, 16, 2, 2, None) == mm.ERR_NULL
    # nothing to do: d_inter == 0 is accepted without pointers
    assert call(np.array([0, 0], np.int32), None, 64, 0, 1, 2, None) == mm.OK


def test_fade_neurons_argument_validation():
    """mlpmoe_fade_neurons refuses bad tables, counts and storage before touching the GPU."""
    import ctypes
    lib = mm.lib
    off = np.array([0, 8, 16], np.int32)
    cnt = np.array([8, 3], np.int32)
    fake = ctypes.c_void_p(0x1000)
    keep = np.zeros(16, np.uint8)
    call = lambda offs, c, dm, di, B, eb, wg=fake, out=keep: lib.mlpmoe_fade_neurons(
        wg, fake, offs.ctypes.data, c.ctypes.data if c is not None else None, dm, di, B, eb,
        out.ctypes.data if out is not None else None, None, None)
    assert call(off, cnt, 64, 16, 0, 2) == mm.ERR_SHAPE
    assert call(off, cnt, 64, 17, 2, 2) == mm.ERR_OFFSETS
    assert call(off, None, 64, 16, 2, 2) == mm.ERR_NULL
    assert call(off, np.array([9, 3], np.int32), 64, 16, 2, 2) == mm.ERR_SHAPE      # more than the branch holds
    assert call(off, np.array([8, -1], np.int32), 64, 16, 2, 2) == mm.ERR_SHAPE
    assert call(off, cnt, 64, 16, 2, 1) == mm.ERR_UNSUPPORTED
    assert call(off, cnt, 60, 16, 2, 2) == mm.ERR_UNSUPPORTED
    assert call(off, cnt, 62, 16, 2, 4) == mm.ERR_UNSUPPORTED
    assert call(off, cnt, 64, 16, 2, 2, ctypes.c_void_p(0x1008)) == mm.ERR_ALIGN
    assert call(off, cnt, 64, 16, 2, 2, None) == mm.ERR_NULL
    assert call(off, cnt, 64, 16, 2, 2, fake, None) == mm.ERR_NULL
    assert call(np.array([0, 0], np.int32), np.array([0], np.int32), 64, 0, 1, 2, None, None) == mm.OK


def test_plan_argument_validation():
    """mlpmoe_plan_create checks the table before it touches the GPU; a NULL plan is harmless."""
    import ctypes
    lib = mm.lib
    h = ctypes.c_void_p()
    off = np.array([0, 8, 16], np.int32)
    al = np.ones(2, np.float32)
    mk = np.ones(2, np.uint8)
    create = lambda o, dm, di, B, eb, mt: lib.mlpmoe_plan_create(o.ctypes.data, al.ctypes.data, mk.ctypes.data,
                                                                 dm, di, B, eb, mt, ctypes.byref(h))
    assert create(off, 64, 16, 2, 3, 16) == mm.ERR_SHAPE          # element size
    assert create(off, 64, 16, 2, 2, 0) == mm.ERR_SHAPE           # max_T
    assert create(off, 64, 17, 2, 2, 16) == mm.ERR_OFFSETS
    assert create(off, 64, 16, 65, 2, 16) == mm.ERR_SHAPE
    assert not h.value
    assert lib.mlpmoe_plan_create(off.ctypes.data, al.ctypes.data, mk.ctypes.data, 64, 16, 2, 2, 16, None) == mm.ERR_NULL
    assert lib.mlpmoe_plan_forward(None, None, None, None, None, 1, None, None) == mm.ERR_NULL
    assert lib.mlpmoe_plan_destroy(None) == mm.OK
