"""GPU parity: every kernel path of the C-ABI library against the CPU oracle, element by element.

Tolerances (max|err| / rms(oracle)): 1e-5 for float storage, 1e-2 for bf16 storage with fp32
accumulation.  bf16 paths are gated against the oracle's contract mode (same single rounding of
alpha*h to bf16) and, additionally, against its exact mode.
"""
import numpy as np
import pytest

import oracle
from gpu_util import BF16_TOL, FP32_TOL, check_bf16_flip_aware, oracle_out, run_gpu, run_gpu_with_hidden, to_dev
from paper_2511_21089_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2511_21089_amd import binding
    return binding


def equal_offsets(d_inter, B):
    return (np.arange(B + 1) * (d_inter // B)).astype(np.int32)


# ------------------------------------------------------------------ float path
def test_tiny_f32_equals_dense_mlp(mm):
    """d_model 64, d_inter 256, B=4, T=32, alpha=1, all active: must equal the dense MLP."""
    L = synth.make_layer("tiny_f32", 32, seed=0)
    off, alpha, mask, _ = mm.mlpmoe_slice(256, 4)
    got = run_gpu(L.x, L.W_gate, L.W_up, L.W_down, off, alpha, mask)
    dense = oracle.dense_swiglu(L.x, L.W_gate, L.W_up, L.W_down)
    ref = oracle_out(L.x, L.W_gate, L.W_up, L.W_down, off, alpha, mask, "exact")
    assert oracle.rel_max_err(got, dense) <= FP32_TOL
    assert oracle.rel_max_err(got, ref) <= FP32_TOL


@pytest.mark.parametrize("T,dm,di,off,mask", [
    (70, 50, 130, [0, 33, 33, 77, 130], [1, 1, 0, 1]),          # ragged everything, empty + pruned branch
    (1, 7, 5, [0, 5], [1]),
    (129, 64, 192, [0, 64, 128, 192], [0, 1, 1]),
])
def test_f32_general_shapes(mm, T, dm, di, off, mask):
    rng = np.random.default_rng(T + dm)
    x, Wg, Wu, Wd = synth.random_layer(rng, T, dm, di, w_scale=0.1)
    off = np.array(off, np.int32)
    mask = np.array(mask, np.uint8)
    alpha = rng.uniform(0.5, 1.5, size=len(mask)).astype(np.float32)
    got = run_gpu(x, Wg, Wu, Wd, off, alpha, mask)
    ref = oracle_out(x, Wg, Wu, Wd, off, alpha, mask, "exact")
    assert oracle.rel_max_err(got, ref) <= FP32_TOL


# ------------------------------------------------------------------ bf16 paths at sizes spanning tiles + tails
def check_bf16(got, args):
    """Both oracle modes at the stated tolerance.  Against the contract mode the only differences
    are fp32 summation order and the rare element where alpha*h sits so close to a bf16 rounding
    boundary that fp32 and double disagree about the side; with >= 1000 active neurons one such
    flip moves an output by well under the tolerance."""
    ref_c = oracle_out(*args, "contract")
    ref_e = oracle_out(*args, "exact")
    e_c, e_e = oracle.rel_max_err(got, ref_c), oracle.rel_max_err(got, ref_e)
    assert np.all(np.isfinite(got))
    print("err(contract)=%.2e err(exact)=%.2e" % (e_c, e_e))
    assert e_c <= BF16_TOL, ("contract", e_c)
    assert e_e <= BF16_TOL, ("exact", e_e)
    return e_c, e_e


def small_bf16_case(seed, T, dm, off, mask, w_scale=0.08):
    rng = np.random.default_rng(seed)
    di = off[-1]
    x, Wg, Wu, Wd = synth.random_layer(rng, T, dm, di, dtype="bf16", w_scale=w_scale)
    alpha = rng.uniform(0.9, 1.2, size=len(mask)).astype(np.float32)
    return x, Wg, Wu, Wd, np.array(off, np.int32), alpha, np.array(mask, np.uint8)


def test_bf16_generic_unaligned_branches(mm):
    args = small_bf16_case(1, 75, 72, [0, 337, 337, 501, 950, 1403], [1, 1, 0, 1, 1])
    got = run_gpu(*args, path=mm.PATH_GENERIC)
    check_bf16(got, args)
    # the automatic choice must route unaligned tables to the same kernels
    assert np.array_equal(run_gpu(*args), got)


MFMA_CASES = [
    # T, d_model, offsets, mask
    (300, 136, [0, 520, 520, 904, 1672], [1, 1, 0, 1]),    # 2 M tiles with tail, K tail (136 = 2*64+8), runs
    (64, 64, [0, 1024], [1]),
    (257, 264, [0, 8, 264, 272, 1400], [1, 0, 1, 1]),      # 8-wide branch, run starting mid tile
    (40, 512, [0, 512, 1024, 1536], [1, 1, 1]),            # split-K candidates
]


@pytest.mark.parametrize("T,dm,off,mask", MFMA_CASES)
def test_bf16_mfma_path(mm, T, dm, off, mask):
    args = small_bf16_case(T, T, dm, off, mask)
    got = run_gpu(*args, path=mm.PATH_MFMA)
    check_bf16(got, args)
    again = run_gpu(*args, path=mm.PATH_MFMA)
    assert np.array_equal(got, again)                      # bitwise reproducible


MFMA_TILE_CASES = MFMA_CASES + [
    (600, 200, [0, 64, 192, 200, 776, 1416], [1, 1, 1, 0, 1]),   # five 128-token tiles (tail of 88), runs of 200 and 640
    (129, 1032, [0, 1096], [1]),                                  # 17 K tiles (tail of 8), one token past a tile
    (1000, 384, [0, 520, 1040], [1, 1]),                          # enough output tiles for several K splits
]


@pytest.mark.parametrize("T,dm,off,mask", MFMA_TILE_CASES)
def test_bf16_mfma_every_tile_shape(mm, T, dm, off, mask):
    """Each tile shape of the MFMA kernels forced for both launches (256 x (128+128), 256 x (64+64), 128 x (64+64)
    with both ring depths, 64 x (64+64) with the staged ring):
    H and the result element by element, bitwise reproducible."""
    args = small_bf16_case(900 + T, T, dm, off, mask)
    for p in (mm.PATH_MFMA_WIDE, mm.PATH_MFMA_NARROW, mm.PATH_MFMA_SMALL, mm.PATH_MFMA_DEEP, mm.PATH_MFMA_SLIM):
        got, H = run_gpu_with_hidden(*args, path=p)
        check_bf16_flip_aware(got, H, *args, label="T=%d d_model=%d tile shape %d:" % (T, dm, p - mm.PATH_MFMA_WIDE))
        if sum(w for w, m in zip(np.diff(off), mask) if m) >= 1000:
            check_bf16(got, args)
        assert np.array_equal(got, run_gpu(*args, path=p))


DECODE_CASES = [
    (1, 136, [0, 520, 520, 904, 1672], [1, 1, 0, 1]),
    (5, 264, [0, 8, 264, 272, 1400], [1, 0, 1, 1]),
    (16, 512, [0, 512, 1024, 1536], [1, 1, 1]),
    (8, 64, [0, 1048], [1]),
    (16, 1096, [0, 1000, 2072], [1, 1]),                   # K tails in both kernels
]


WIDE_MODEL_DECODE_CASES = [
    # d_model beyond 4096: the gate+up kernel variants (x fragments of 16 blocks in registers; x staged in LDS;
    # one workgroup per tile) and the down kernel that splits K over two workgroups
    (16, 4104, [0, 64, 136], [1, 1]),                      # 65 K blocks: 9 per wave, padded to 16
    (5, 8192, [0, 72], [1]),
    (3, 8200, [0, 64, 128], [1, 1]),                       # 129 K blocks: x staged in LDS
    (16, 8200, [0, 64, 128], [0, 1]),                      # ... too large for the LDS at 16 tokens
]


@pytest.mark.parametrize("T,dm,off,mask", WIDE_MODEL_DECODE_CASES)
def test_bf16_decode_wide_models(mm, T, dm, off, mask):
    args = small_bf16_case(300 + T + dm, T, dm, off, mask, w_scale=0.02)
    got, H = run_gpu_with_hidden(*args, path=mm.PATH_DECODE)
    check_bf16_flip_aware(got, H, *args, label="decode T=%d d_model=%d:" % (T, dm))
    assert np.array_equal(got, run_gpu(*args, path=mm.PATH_DECODE))
    g2, H2 = run_gpu_with_hidden(*args, path=mm.PATH_GENERIC)
    check_bf16_flip_aware(g2, H2, *args, label="generic T=%d d_model=%d:" % (T, dm))


@pytest.mark.parametrize("T,dm,off,mask", DECODE_CASES)
def test_bf16_decode_path(mm, T, dm, off, mask):
    args = small_bf16_case(100 + T, T, dm, off, mask)
    got = run_gpu(*args, path=mm.PATH_DECODE)
    check_bf16(got, args)
    assert np.array_equal(got, run_gpu(*args, path=mm.PATH_DECODE))
    assert np.array_equal(got, run_gpu(*args))            # automatic choice for T <= 16


def test_paths_agree_on_contract(mm):
    """Generic, MFMA and decode kernels implement one rounding contract: they differ only by fp32 summation order."""
    args = small_bf16_case(7, 16, 256, [0, 512, 1024, 1536], [1, 1, 1])
    outs = [run_gpu(*args, path=p) for p in (mm.PATH_GENERIC, mm.PATH_MFMA, mm.PATH_DECODE)]
    for o in outs[1:]:
        assert oracle.rel_max_err(o, outs[0]) < BF16_TOL / 2


# ------------------------------------------------------------------ edge cases
def test_edge_cases(mm):
    import torch
    args = list(small_bf16_case(3, 20, 64, [0, 1024, 2048], [1, 1]))
    x, Wg, Wu, Wd, off, alpha, mask = args
    dev = tuple(to_dev(a) for a in (x, Wg, Wu, Wd))
    # nothing active: exact zeros on every path
    none = np.zeros(2, np.uint8)
    for p in (None, mm.PATH_GENERIC, mm.PATH_MFMA):
        assert np.all(run_gpu(x, Wg, Wu, Wd, off, alpha, none, path=p, dev=dev) == 0)
    # T == 0: accepted, nothing written
    out = torch.zeros((0, 64), dtype=torch.float32, device="cuda")
    mm.mlpmoe_forward_bf16(dev[0][:0], dev[1], dev[2], dev[3], off, alpha, mask, out=out)
    # d_inter == 0 (one empty branch)
    e_off = np.array([0, 0], np.int32)
    got = run_gpu(x, Wg[:0], Wu[:0], np.ascontiguousarray(Wd[:, :0]), e_off, alpha[:1], mask[:1])
    assert np.all(got == 0)
    # non-finite weights inside a pruned branch must not leak, on any path
    Wg2, Wu2, Wd2 = Wg.copy(), Wu.copy(), Wd.copy()
    Wg2[1024:] = 0x7FC0     # bf16 NaN
    Wu2[1024:] = 0x7F80     # +inf
    Wd2[:, 1024:] = 0x7FC0
    m2 = np.array([1, 0], np.uint8)
    ref = oracle_out(x, Wg, Wu, Wd, off, alpha, m2, "contract")
    for p in (mm.PATH_GENERIC, mm.PATH_MFMA):
        got = run_gpu(x, Wg2, Wu2, Wd2, off, alpha, m2, path=p)
        assert np.all(np.isfinite(got)) and oracle.rel_max_err(got, ref) < BF16_TOL
    got = run_gpu(x[:16], Wg2, Wu2, Wd2, off, alpha, m2, path=mm.PATH_DECODE)
    assert np.all(np.isfinite(got)) and oracle.rel_max_err(got, ref[:16]) < BF16_TOL
    # alpha == 0 with the mask set is computed (gives zeros on finite data), mask == 0 is skipped
    a0 = alpha.copy()
    a0[1] = 0
    got_a0 = run_gpu(x, Wg, Wu, Wd, off, a0, mask, path=mm.PATH_MFMA, dev=dev)
    assert oracle.rel_max_err(got_a0, ref) < BF16_TOL
    # caller-owned workspace that is too small is refused
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(mm.MlpMoeError) as ei:
        mm.mlpmoe_forward_bf16_ws(dev[0], dev[1], dev[2], dev[3], off, alpha, mask, ws)
    assert ei.value.status == mm.ERR_WORKSPACE


def test_max_branches_and_single_neuron_runs(mm):
    """B = 64 with alternating pruned branches of 40 neurons: 32 separate runs, none tile aligned."""
    B = 64
    off = (np.arange(B + 1) * 40).astype(np.int32)
    mask = (np.arange(B) % 2 == 0).astype(np.uint8)
    rng = np.random.default_rng(64)
    x, Wg, Wu, Wd = synth.random_layer(rng, 33, 64, 2560, dtype="bf16", w_scale=0.1)
    alpha = rng.uniform(0.9, 1.2, size=B).astype(np.float32)
    args = (x, Wg, Wu, Wd, off, alpha, mask)
    for p in (mm.PATH_GENERIC, mm.PATH_MFMA):
        check_bf16(run_gpu(*args, path=p), args)
    a16 = (x[:16],) + args[1:]
    check_bf16(run_gpu(*a16, path=mm.PATH_DECODE), a16)


# ------------------------------------------------------------------ compaction (fade) end to end
def test_slice_compact_forward_equals_zeroed_rows(mm):
    """Neuron removal + compaction + padding on the device == the uncompacted layer with those
    neurons' up-projection rows set to zero, evaluated by the oracle."""
    L = synth.make_layer("llama8b_fade", 48, seed=2, d_model=128, d_inter=16 * 112)
    B = L.workload.B
    off, alpha1, mask, gather = mm.mlpmoe_slice(16 * 112, B, 0, L.neuron_keep, pad_to=8)
    dev = tuple(to_dev(a) for a in (L.W_gate, L.W_up, L.W_down))
    Wg_c, Wu_c, Wd_c = mm.mlpmoe_compact(dev[0], dev[1], dev[2], gather)
    # data movement is bit exact against the oracle's gather
    o_off, _, _, o_gather = oracle.slice_plan(16 * 112, B, 0, L.neuron_keep, 8)
    rWg, rWu, rWd = oracle.compact_layer(L.W_gate, L.W_up, L.W_down, o_gather)
    import torch
    for t, r in ((Wg_c, rWg), (Wu_c, rWu), (Wd_c, rWd)):
        assert np.array_equal(t.view(torch.int16).cpu().numpy().view(np.uint16), r)
    alpha = L.alpha_draw
    Wu_z = L.W_up.copy()
    Wu_z[L.neuron_keep == 0] = 0
    full_off = equal_offsets(16 * 112, B)
    ref_args = (L.x, L.W_gate, Wu_z, L.W_down, full_off, alpha, mask)
    x_d = to_dev(L.x)
    for path in (mm.PATH_MFMA, mm.PATH_GENERIC):
        ws = mm.new_workspace(48, 128, int(off[-1]), B)
        out = mm.mlpmoe_forward_bf16_ws(x_d, Wg_c, Wu_c, Wd_c, off, alpha, mask, ws, path=path)
        check_bf16(out.cpu().numpy(), ref_args)
    # unpadded compaction has odd widths and takes the generic kernels
    off1, _, _, gather1 = mm.mlpmoe_slice(16 * 112, B, 0, L.neuron_keep, pad_to=1)
    c1 = mm.mlpmoe_compact(dev[0], dev[1], dev[2], gather1)
    out = mm.mlpmoe_forward_bf16(x_d, c1[0], c1[1], c1[2], off1, alpha, mask)
    check_bf16(out.cpu().numpy(), ref_args)


def test_compensated_pruning_first_k(mm):
    """Sec. 3.3 exactly: keep the first K of B branches with alpha = sqrt(B/K)."""
    L = synth.make_layer("qwen05b", 40, seed=4, d_model=128, d_inter=8 * 192)
    off, alpha, mask, _ = mm.mlpmoe_slice(8 * 192, 8, K_keep=6)
    args = (L.x, L.W_gate, L.W_up, L.W_down, off, alpha, mask)
    check_bf16(run_gpu(*args, path=mm.PATH_MFMA), args)
    a16 = (L.x[:16],) + args[1:]
    check_bf16(run_gpu(*a16, path=mm.PATH_DECODE), a16)


# ------------------------------------------------------------------ other branch counts and uneven splits
@pytest.mark.parametrize("B,pruned", [(4, [2]), (32, [0, 5, 6, 7, 31])])
def test_branch_counts_4_and_32(mm, B, pruned):
    """The 0.5B-shaped layer cut into B = 4 and B = 32 branches (the other branch counts of Sec. 4)."""
    L = synth.make_layer("qwen05b", 300, seed=B, B=B)
    off, _, mask, _ = mm.mlpmoe_slice(4864, B)
    mask[pruned] = 0
    alpha = np.random.default_rng(B).uniform(0.9, 1.2, size=B).astype(np.float32)
    args = (L.x, L.W_gate, L.W_up, L.W_down, off, alpha, mask)
    check_bf16(run_gpu(*args), args)                       # T = 300: MFMA kernels
    a7 = (L.x[:7],) + args[1:]
    check_bf16(run_gpu(*a7), a7)                           # T = 7: decode kernels


def test_d_inter_not_divisible_by_B(mm):
    """d_inter = 4870 over B = 8: the first 6 branches are one neuron wider (609, 608).  The raw table
    has unaligned boundaries (generic kernels); padded to multiples of 8 and compacted it takes the
    MFMA and decode kernels.  All three must match the oracle on the original layer."""
    d_inter, B = 4870, 8
    L = synth.make_layer("qwen05b", 130, seed=9, d_inter=d_inter)
    off, _, mask, _ = mm.mlpmoe_slice(d_inter, B)
    assert list(np.diff(off)) == [609] * 6 + [608] * 2
    mask[3] = 0
    alpha = L.alpha_draw
    args = (L.x, L.W_gate, L.W_up, L.W_down, off, alpha, mask)
    check_bf16(run_gpu(*args), args)                       # unaligned: generic kernels
    keep = np.ones(d_inter, np.uint8)
    off8, _, _, gather = mm.mlpmoe_slice(d_inter, B, 0, keep, pad_to=8)
    assert all(int(o) % 8 == 0 for o in off8) and int(off8[-1]) == 6 * 616 + 2 * 608
    dev = tuple(to_dev(a) for a in (L.W_gate, L.W_up, L.W_down))
    Wc = mm.mlpmoe_compact(dev[0], dev[1], dev[2], gather)
    x_d = to_dev(L.x)
    out = mm.mlpmoe_forward_bf16(x_d, Wc[0], Wc[1], Wc[2], off8, alpha, mask)
    check_bf16(out.cpu().numpy(), args)                    # T = 130: MFMA kernels
    out = mm.mlpmoe_forward_bf16(x_d[:16], Wc[0], Wc[1], Wc[2], off8, alpha, mask)
    check_bf16(out.cpu().numpy(), (L.x[:16],) + args[1:])  # decode kernels


@pytest.mark.parametrize("K", [1, 3, 8])
def test_first_k_sweep(mm, K):
    """Sec. 3.3 for several K on the 0.5B-shaped layer: alpha = sqrt(B / K), branches K.. skipped."""
    L = synth.make_layer("qwen05b", 64, seed=20 + K)
    off, alpha, mask, _ = mm.mlpmoe_slice(4864, 8, K_keep=K)
    assert np.allclose(alpha[:K], np.sqrt(8.0 / K)) and mask.sum() == K
    args = (L.x, L.W_gate, L.W_up, L.W_down, off, alpha, mask)
    if K * 608 >= 1000:                                    # see check_bf16: enough active neurons
        check_bf16(run_gpu(*args), args)
    got, H = run_gpu_with_hidden(*args)                    # any K: H itself and both oracle modes, flips accounted for
    check_bf16_flip_aware(got, H, *args, label="first-K K=%d T=64:" % K)
    assert np.array_equal(got, run_gpu(*args))
    a1 = (L.x[:1],) + args[1:]
    got, H = run_gpu_with_hidden(*a1)
    check_bf16_flip_aware(got, H, *a1, label="first-K K=%d T=1:" % K)


def test_bf16_mfma_mixed_tile_widths(mm):
    """More than one round of 256 wide tiles with a small remainder: the gate+up launch runs the full round
    with 256 x (128 + 128) tiles and the remainder (54 wide tiles, less than a quarter of a round) as quarters of
    128 tokens x 64 neurons.  Ten token tiles (the last ragged: its second half holds no token), three runs of
    active branches whose last wide tiles are 104, 88 and exactly 64 neurons wide (a second half that is partly
    filled, and one that is empty)."""
    widths = [1000, 200, 1640, 1008, 8, 192]
    off = np.concatenate([[0], np.cumsum(widths)]).astype(np.int32)
    mask = [1, 0, 1, 1, 0, 1]
    args = small_bf16_case(77, 2304 + 77, 64, off.tolist(), mask)
    got, H = run_gpu_with_hidden(*args, path=mm.PATH_MFMA_MIXED)
    e_c, _, _ = check_bf16_flip_aware(got, H, *args, label="mixed tile widths:")
    assert e_c <= BF16_TOL                                 # the plain gate as well (3840 active neurons)
    # every output element adds up the same products in the same order whatever the tile width
    wide, Hw = run_gpu_with_hidden(*args, path=mm.PATH_MFMA_WIDE)
    act = np.repeat(np.array(mask, bool), widths)
    assert np.array_equal(H[:, act], Hw[:, act])
    assert np.array_equal(got, run_gpu(*args, path=mm.PATH_MFMA_MIXED))
    # a remainder of more than a quarter of a round (4 x 89 = 356 wide tiles: 100 left over) runs as halves
    w2 = [5000, 304, 6200]
    off2 = np.concatenate([[0], np.cumsum(w2)]).astype(np.int32)
    args2 = small_bf16_case(79, 3 * 256 + 40, 64, off2.tolist(), [1, 0, 1])
    got2, H2 = run_gpu_with_hidden(*args2, path=mm.PATH_MFMA_MIXED)
    check_bf16_flip_aware(got2, H2, *args2, label="mixed tile widths, halves:")
    wide2, Hw2 = run_gpu_with_hidden(*args2, path=mm.PATH_MFMA_WIDE)
    act2 = np.repeat(np.array([1, 0, 1], bool), w2)
    assert np.array_equal(H2[:, act2], Hw2[:, act2])
    # where the tile count leaves no such remainder the selector falls back to wide tiles
    small = small_bf16_case(78, 300, 64, [0, 1024], [1])
    assert np.array_equal(run_gpu(*small, path=mm.PATH_MFMA_MIXED), run_gpu(*small, path=mm.PATH_MFMA_WIDE))


THIN_CASES = [
    # active neurons from 8 to 512: one thin branch of a faded or pruned layer.  T, d_model, offsets, mask
    (300, 136, [0, 8], [1]),
    (300, 256, [0, 64, 128, 136], [0, 1, 1]),              # 72 active
    (257, 264, [0, 200, 456, 1000], [1, 0, 0]),            # 200 active, run ends mid tile
    (64, 512, [0, 384], [1]),                              # the shape of the first failure of a plain 1e-2 gate
    (600, 128, [0, 256, 512, 768], [1, 1, 0]),             # 512 active, three token tiles, K split
    (16, 136, [0, 8, 16, 48], [1, 0, 1]),                  # decode-sized batches on every path
    (3, 512, [0, 384], [1]),
]


@pytest.mark.parametrize("T,dm,off,mask", THIN_CASES)
def test_bf16_thin_layers_every_path(mm, T, dm, off, mask):
    """Layers with 8 .. 512 active neurons in contract AND exact mode on the generic, MFMA and decode kernels:
    the stored intermediate is compared element by element, and the outputs with the flips accounted for."""
    args = small_bf16_case(500 + T + dm, T, dm, off, mask)
    paths = [mm.PATH_GENERIC, mm.PATH_MFMA, mm.PATH_MFMA_WIDE, mm.PATH_MFMA_NARROW, mm.PATH_MFMA_SMALL, mm.PATH_MFMA_DEEP,
             mm.PATH_MFMA_SLIM] + (
        [mm.PATH_DECODE] if T <= 16 else [])
    for p in paths:
        got, H = run_gpu_with_hidden(*args, path=p)
        check_bf16_flip_aware(got, H, *args, label="thin T=%d d_model=%d path=%d:" % (T, dm, p))
    assert np.array_equal(run_gpu(*args), run_gpu_with_hidden(*args, path=mm.PATH_AUTO)[0])


@pytest.mark.parametrize("d_model", [3072, 328])
def test_decode_is_reproducible_and_clears_out(mm, d_model):
    """Float result at T <= 16: the down projection splits K over two workgroups and adds the halves with float
    atomics into an `out` the gate+up kernel has cleared (two row tiles per workgroup for d_model >= 3072, one
    below).  The bits must not depend on the order of the two atomics (30 repetitions), nor on what `out` held
    before, and the result must match the oracle."""
    import torch
    d_inter, B = 1536, 6
    for T in (1, 11, 16):
        L = synth.make_layer("qwen05b", T, seed=80 + T, d_model=d_model, d_inter=d_inter, B=B)
        off, _, mask, _ = mm.mlpmoe_slice(d_inter, B)
        mask[4] = 0
        x, Wg, Wu, Wd = (to_dev(a) for a in (L.x, L.W_gate, L.W_up, L.W_down))
        first = None
        for rep in range(30):
            out = torch.full((T, d_model), float("nan") if rep % 2 else 1e30, dtype=torch.float32, device="cuda")
            mm.mlpmoe_forward_bf16(x, Wg, Wu, Wd, off, L.alpha_draw, mask, out=out)
            if first is None:
                first = out.clone()
            else:
                assert torch.equal(out, first), rep
        got = first.cpu().numpy()
        for mode in ("contract", "exact"):
            ref = oracle_out(L.x, L.W_gate, L.W_up, L.W_down, off, L.alpha_draw, mask, mode)
            assert oracle.rel_max_err(got, ref) <= BF16_TOL, (T, mode)
