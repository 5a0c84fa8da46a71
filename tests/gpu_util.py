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


# --------------------------------------------------------------------------- the bf16 rounding point, looked at directly
# The bf16 paths round alpha_b * SiLU(g) * u once to bf16.  The GPU forms that value in fp32 from fp32 sums,
# the contract oracle in float from double sums; where the value lies very close to a bf16 rounding boundary
# the two may pick different neighbours ("flip").  Each flip moves one output by up to one bf16 unit of
# that h times |W_down|, which on a layer with few active neurons can exceed 1e-2 of rms(out) although
# both sides are correct.  The checks below therefore look at H itself and account for the flips they see,
# instead of needing many neurons to drown them.
U24 = 2.0 ** -24          # unit roundoff of fp32
C_SUM = 16.0              # fp32 sum of n products (exact in fp32 for bf16 inputs), any order: the error behaves
                          # like a random walk of the partial sums, standard deviation ~ 0.64 * U24 * sum|terms|
                          # (terms ~ product of two normals); 16 * U24 * sum|terms| is 25 standard deviations
                          # and still below the worst-case bound (n - 1) * U24 * sum|terms| for n > 17


def hidden_bounds(x, Wg, Wu, off, alpha, mask):
    """Oracle side of the H check: (h_contract, h_exact, lo, hi, act) with lo <= H <= hi the bf16 values
    a correct fp32 evaluation may store (both bounds bf16 values), act the [d_inter] column mask of
    active branches."""
    xw, Wgw, Wuw = widen(x), widen(Wg), widen(Wu)
    h_c = oracle.mlpmoe_hidden(xw, Wgw, Wuw, off, alpha, mask, "contract")
    h_e, g, u, ag, au = oracle.mlpmoe_hidden(xw, Wgw, Wuw, off, alpha, mask, "exact", details=True)
    B = len(alpha)
    act = np.zeros(int(off[-1]), dtype=bool)
    a_col = np.zeros(int(off[-1]))
    for b in range(B):
        if mask[b]:
            act[off[b]:off[b + 1]] = True
        a_col[off[b]:off[b + 1]] = float(alpha[b])
    # first-order error of h = a * silu(g) * u under errors eg, eu of the two sums, plus a few fp32
    # roundings of h itself (exp and reciprocal about 1 ulp each, three multiplications)
    sig = 1.0 / (1.0 + np.exp(-g))
    silu = g * sig
    dsilu = sig * (1.0 + g * (1.0 - sig))
    eg, eu = C_SUM * U24 * ag, C_SUM * U24 * au
    delta = np.abs(a_col) * (np.abs(dsilu * u) * eg + np.abs(silu) * eu + eg * eu) + C_SUM * U24 * np.abs(h_e)
    # rounding is monotone: every value within delta of the exact one rounds into [lo, hi]
    lo = oracle.round_to_bf16(h_e - delta)
    hi = oracle.round_to_bf16(h_e + delta)
    return h_c, h_e, lo, hi, act


def flip_terms(H_gpu, x, Wg, Wu, Wd, off, alpha, mask, route=None, label=""):
    """Step 1 of check_bf16_flip_aware (asserts that every stored h is one fp32 could have rounded to) and the
    quantities the output checks need: H (stored values, 0 where not taken), h_c / h_e (oracle, contract /
    exact), flips, ref_c / ref_e (oracle results = h W_down^T), rms_c / rms_e, allow_c (what the flips may
    move an output by), sum_err (fp32 summation error bound of the down projection of H)."""
    h_c, h_e, lo, hi, act = hidden_bounds(x, Wg, Wu, off, alpha, mask)
    T, d_inter = h_c.shape
    B = len(alpha)
    take = np.broadcast_to(act, (T, d_inter)).copy()
    if route is not None:
        for b in range(B):
            take[:, off[b]:off[b + 1]] &= (np.asarray(route)[:, b:b + 1] != 0)
        h_c = np.where(take, h_c, 0.0)
        h_e = np.where(take, h_e, 0.0)
    H = np.where(take, np.asarray(H_gpu, dtype=np.float64), 0.0)
    assert np.all(np.isfinite(H)), (label, "unwritten or non-finite h")
    bad = take & ((H < lo) | (H > hi))
    assert not bad.any(), (label, "stored h outside what fp32 can round to", int(bad.sum()),
                           np.argwhere(bad)[:4].tolist())
    flips = take & (H != h_c)
    Wdw = widen(Wd).astype(np.float64)
    aWd = np.abs(Wdw)
    ref_c = h_c @ Wdw.T          # the contract oracle's forward (pinned: forward(contract) == hidden(contract) W_down^T)
    ref_e = h_e @ Wdw.T
    return dict(H=H, h_c=h_c, h_e=h_e, flips=flips, take=take, Wd=Wdw, aWd=aWd, ref_c=ref_c, ref_e=ref_e,
                rms_c=float(np.sqrt(np.mean(ref_c * ref_c))) if ref_c.size else 0.0,
                rms_e=float(np.sqrt(np.mean(ref_e * ref_e))) if ref_e.size else 0.0,
                allow_c=np.abs(np.where(flips, H - h_c, 0.0)) @ aWd.T,
                sum_err=C_SUM * U24 * (np.abs(H) @ aWd.T))


def check_bf16_flip_aware(got, H_gpu, x, Wg, Wu, Wd, off, alpha, mask, route=None, tol=BF16_TOL, label=""):
    """Parity of a bf16 path that holds for ANY number of active neurons.

    got [T, d_model] float result, H_gpu [T, d_inter] the bf16 intermediate the kernels stored (as float64;
    columns of inactive branches are ignored).  route (optional [T, B]): per-token routing; entries of H a
    token does not take are ignored here (the output checks below catch anything they would do).
      1. every stored h is a bf16 value a correct fp32 evaluation could have produced (hidden_bounds);
      2. the result is the down projection of the stored H (fp64 product of H_gpu and W_down) up to fp32
         summation error;
      3. against the contract oracle: |got - ref| <= tol * rms(ref) + sum over flipped h of |dh| |W_down|;
      4. against the exact oracle: |got - ref| <= sum_j |H_gpu - h_exact| |W_down| + the summation error of 2
         (the bound that 1 and 2 imply; with many active neurons the plain tol * rms(ref) holds as well and
         the callers that have them assert it).
    Returns (err_contract, err_exact, flip_fraction) with the errors as max|.|/rms."""
    f = flip_terms(H_gpu, x, Wg, Wu, Wd, off, alpha, mask, route, label)
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), label
    own = f["H"] @ f["Wd"].T
    assert np.all(np.abs(got - own) <= f["sum_err"] + 1e-30), (
        label, "result is not the down projection of the stored H", float(np.max(np.abs(got - own) - f["sum_err"])))
    assert np.all(np.abs(got - f["ref_c"]) <= tol * f["rms_c"] + f["allow_c"]), (label, "contract")
    allow_e = np.abs(f["H"] - f["h_e"]) @ f["aWd"].T + f["sum_err"]
    assert np.all(np.abs(got - f["ref_e"]) <= allow_e + 1e-30), (label, "exact")
    e_c = float(np.max(np.abs(got - f["ref_c"]))) / f["rms_c"] if f["rms_c"] > 0 else 0.0
    e_e = float(np.max(np.abs(got - f["ref_e"]))) / f["rms_e"] if f["rms_e"] > 0 else 0.0
    n_flips = int(f["flips"].sum())
    frac = n_flips / max(int(f["take"].sum()), 1)
    print("%s err(contract)=%.2e err(exact)=%.2e flips=%d (%.4f%%)" % (label, e_c, e_e, n_flips, 100 * frac), flush=True)
    return e_c, e_e, frac


def run_gpu_with_hidden(x, Wg, Wu, Wd, off, alpha, mask, path=0, route=None, out_bf16=False):
    """bf16 forward through the caller-workspace entry point; returns (out [T, d_model] numpy (float32, or the
    bf16 result widened to float64 with out_bf16), H [T, d_inter] float64 numpy: the intermediate the kernels
    left at the start of the workspace)."""
    import torch
    from paper_2511_21089_amd import binding as mm
    d = tuple(to_dev(a) for a in (x, Wg, Wu, Wd))
    T, d_model = x.shape
    d_inter, B = Wg.shape[0], len(alpha)
    out = torch.full((T, d_model), float("nan"), dtype=torch.bfloat16 if out_bf16 else torch.float32, device="cuda")
    ws = mm.new_workspace(T, d_model, d_inter, B, 2)
    ws.fill_(0xFF)                                   # bf16 NaN everywhere: unwritten h shows
    if out_bf16:
        mm.mlpmoe_forward_bf16_out_bf16_ws(d[0], d[1], d[2], d[3], off, alpha, mask, ws, path=path, out=out)
    elif route is None:
        mm.mlpmoe_forward_bf16_ws(d[0], d[1], d[2], d[3], off, alpha, mask, ws, path=path, out=out)
    else:
        r = torch.from_numpy(np.ascontiguousarray(route)).cuda()
        mm.mlpmoe_forward_routed_bf16(d[0], d[1], d[2], d[3], off, alpha, mask, r, out=out, workspace=ws)
    torch.cuda.synchronize()
    ld = mm.mlpmoe_hidden_ld(d_inter)
    Hb = ws[: T * ld * 2].view(torch.int16).view(T, ld)[:, :d_inter].cpu().numpy().view(np.uint16)
    res = out.to(torch.float64).cpu().numpy() if out_bf16 else out.cpu().numpy()
    return res, synth.bf16_bits_to_f32(Hb).astype(np.float64)
