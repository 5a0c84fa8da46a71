#!/usr/bin/env python3
"""Benchmark of the branched SwiGLU MLP forward (MLPMoE, Sec. 3.1) on one MI355X.

A step is one call of the whole hot path (gate+up projection with the fused SiLU*up
epilogue, down projection with the sum over branches) on one batch of T synthetic tokens
that is already resident in HBM.  The headline workload is the Llama-8B-shaped layer
(d_model 4096, d_inter 14336, B=16 branches of 896) at T=4096; the same layer is then timed
at T=16 and T=1 through the decode kernels, rotating over several weight copies so that the
weights come from HBM and not from the last-level cache.

Prints ONE JSON line: tokens/s, the roofline of the dominant kernel (per-kernel durations come
from HIP events the library records on the stream it launches on) and the CPU oracle timed on
the host cores for context.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2516.6    # MI355X dense bf16: 256 CU x 2.4 GHz x 4096 flop/clk/CU
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E

# HBM traffic per launch of the dominant kernel, from two rocprofv3 --pmc runs of this script
# (FETCH_SIZE, then WRITE_SIZE), scaled by what the same counters read for the elementwise pass of
# --copy-mib.  Valid only for the kernel source it was measured on: keyed by that file's SHA-256,
# and reported as null when the source has changed since.
TRAFFIC = {
    # (workload, kernel): (sha256 of the kernel's source file, bytes per launch = read + written, summary file)
    # gate_up_mfma at T=4096: 1409.5 MB read (x is re-read once per group of 4 neuron tiles and the
    # weights once per XCD that needs them: 5.3x the 268 MB the kernel has to read) + 117.5 MB written
    ("llama8b_T4096", "gate_up_mfma"): ("74cf58c3161623bf36554d18cbcebfc1f69733b1bbae9467c73cc306b07d3fac", 1527.0e6,
                                        "profiles/bench_llama8b_T4096_hbm_counters.md"),
    # decode gate+up at T=1: 235.8 MB read (the weights, once) + 0.1 MB written
    ("llama8b_T1", "decode_gate_up"): ("86003e6bc49cbb5e7a657b5889afe067ff945beef544ca3f06cde8ec9f871dcf", 235.9e6,
                                       "profiles/bench_llama8b_T1_hbm_counters.md"),
}
PREWARM_S = 0.1          # untimed repetitions of the step before the warm-up steps (see time_steps)
KERNEL_SOURCE = {"gate_up_mfma": "kernels_mfma.hip", "down_mfma": "kernels_mfma.hip",
                 "decode_gate_up": "kernels_decode.hip", "decode_down": "kernels_decode.hip"}


def traffic_of(workload, kernel):
    """(bytes per launch, where the figure comes from), or (None, None) when there is none for the kernel source
    as it stands: the counters are not read by this run, they were taken by the rocprofv3 runs whose summary the
    second element names."""
    ent = TRAFFIC.get((workload, kernel))
    src = KERNEL_SOURCE.get(kernel)
    if ent is None or src is None:
        return None, None
    path = os.path.join(ROOT, "paper_2511_21089_amd", "csrc", src)
    with open(path, "rb") as f:
        if hashlib.sha256(f.read()).hexdigest() != ent[0]:
            return None, None
    return ent[1], ent[2]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama8b",
                    choices=["qwen05b", "qwen05b_pruned", "llama8b", "llama8b_fade"])
    ap.add_argument("--T", type=int, default=4096)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short runs of the other workloads (0.5B-shaped layer, pruned and faded layers)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="before the timed steps, run one elementwise pass that reads and writes this many "
                         "MiB (calibrates the HBM byte counters under rocprofv3 --pmc)")
    return ap.parse_args()


def build_layer(mm, synth, name, T, seed):
    """Synthetic layer -> device tensors + branch table (+ host copies for the oracle)."""
    L = synth.make_layer(name, T, seed=seed)
    w = L.workload
    off, _, mask, gather = mm.mlpmoe_slice(w.d_inter, w.B, 0, L.neuron_keep, 8, 64)
    mask = mask.copy()
    mask[L.inactive] = 0
    alpha = L.alpha_draw
    dev = [mm.bf16_tensor(a) for a in (L.W_gate, L.W_up, L.W_down)]
    host = (L.W_gate, L.W_up, L.W_down)
    d_eff_alg = int(sum(off[b + 1] - off[b] for b in range(w.B) if mask[b]))
    if L.neuron_keep is not None:
        dev = list(mm.mlpmoe_compact(dev[0], dev[1], dev[2], gather))
        # algorithmic width counts kept neurons only, not the zero rows that pad branches to 8
        kept = L.neuron_keep.reshape(w.B, -1).sum(axis=1)
        d_eff_alg = int(sum(int(kept[b]) for b in range(w.B) if mask[b]))
        import torch
        host = tuple(t.view(torch.int16).cpu().numpy().view(np.uint16) for t in dev)
    x = mm.bf16_tensor(L.x)
    return L, x, dev, host, off, alpha, mask, d_eff_alg


def time_steps(mm, torch, call, steps, warmup, events=False):
    """Warm up, then time exactly `steps` calls; returns (ms_per_step, {kernel: [ms...]}).

    With events=False (the default) the timed steps run bare, and the per-kernel durations come from
    a second pass of the same steps in which the library brackets every kernel with HIP events on
    the stream it launches on.  The brackets keep a kernel from starting while the previous one
    drains, which costs a millisecond step several per cent and a decode step a tenth, so they stay
    out of the timed region.  With events=True the timed steps themselves carry the brackets.

    Before the warm-up steps the same call is repeated for PREWARM_S seconds, untimed: after an idle
    spell (the host-side set-up) the GPU needs some 30 ms of work to settle at its sustained clocks
    (measured on this layer: 1255, 1095, 1049, then 1025 us per step for successive groups of ten
    steps), and a handful of warm-up steps would leave the timed steps on that ramp.
    """
    t_end = time.perf_counter() + PREWARM_S
    n = 0
    while time.perf_counter() < t_end:
        for _ in range(4):
            call(n)
            n += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    cap = steps * 4
    if events:
        mm.mlpmoe_profile_enable(cap)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        call(warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if not events:
        mm.mlpmoe_profile_enable(cap)
        for i in range(steps):
            call(warmup + i)
        torch.cuda.synchronize()
    per_kernel = {}
    for name, ms in mm.mlpmoe_profile_collect(cap):
        per_kernel.setdefault(name, []).append(ms)
    mm.mlpmoe_profile_disable()
    return (t1 - t0) * 1e3 / steps, per_kernel


def roofline_of(per_kernel, T, d_model, d_eff, decode, workload=None):
    """Roofline of the kernel with the largest total time."""
    if not per_kernel:
        return None
    dom = max(per_kernel, key=lambda k: sum(per_kernel[k]))
    avg_ms = sum(per_kernel[dom]) / len(per_kernel[dom])
    gate_up = "gate_up" in dom
    if decode:
        # weights of the kernel's projection(s) read once + activations in and out
        wbytes = (2 if gate_up else 1) * d_model * d_eff * 2
        io = T * d_model * 2 + T * d_eff * 2 if gate_up else T * d_eff * 2 + T * d_model * 4
        ach = (wbytes + io) / (avg_ms * 1e-3) / 1e9
        traffic, source = traffic_of(workload, dom)
        return {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": source,
                "avg_kernel_us": round(avg_ms * 1e3, 2)}
    flops = (4.0 if gate_up else 2.0) * T * d_model * d_eff
    ach = flops / (avg_ms * 1e-3) / 1e12
    traffic, source = traffic_of(workload, dom)
    return {"kernel": dom, "bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": round(ach / MFMA_PEAK_TFLOPS, 4), "traffic": traffic, "traffic_source": source,
            "avg_kernel_us": round(avg_ms * 1e3, 2)}


def cpu_baseline(synth, L, host, off, alpha, mask, seconds):
    """The oracle as it stands (exact mode, OpenMP over tokens) on a bounded sample of the batch."""
    import oracle
    Wg, Wu, Wd = (synth.bf16_bits_to_f32(a) for a in host)
    x = synth.bf16_bits_to_f32(L.x)
    threads = oracle.num_threads()
    n0 = min(L.T, threads)
    t0 = time.perf_counter()
    oracle.mlpmoe_forward(x[:n0], Wg, Wu, Wd, off, alpha, mask, mode="exact")
    probe = time.perf_counter() - t0
    n = int(max(n0, min(L.T, (seconds / max(probe, 1e-6)) * n0)))
    n = max(threads, n // threads * threads) if L.T >= threads else L.T
    n = min(n, L.T)
    t0 = time.perf_counter()
    oracle.mlpmoe_forward(x[:n], Wg, Wu, Wd, off, alpha, mask, mode="exact")
    dt = time.perf_counter() - t0
    return {"value": round(n / dt, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "first %d of %d tokens of the same batch, exact fp64 mode, %.1f s" % (n, L.T, dt)}


def library_gemms(torch, Wgu, Wd, T):
    """x @ [W_gate; W_up]^T and h @ W_down^T as two torch.mm calls, per-call time from events."""
    d_model, d_inter = Wd.shape
    x = torch.randn(T, d_model, device="cuda").to(torch.bfloat16)
    h = (torch.randn(T, d_inter, device="cuda") * 0.5).to(torch.bfloat16)
    o1 = torch.empty(T, 2 * d_inter, device="cuda", dtype=torch.bfloat16)
    o2 = torch.empty(T, d_model, device="cuda", dtype=torch.bfloat16)
    t_end = time.perf_counter() + PREWARM_S
    while time.perf_counter() < t_end:
        for _ in range(4):
            torch.mm(x, Wgu.t(), out=o1)
            torch.mm(h, Wd.t(), out=o2)
        torch.cuda.synchronize()
    n = 20
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * n)]
    for k in range(n):
        ev[3 * k].record()
        torch.mm(x, Wgu.t(), out=o1)
        ev[3 * k + 1].record()
        torch.mm(h, Wd.t(), out=o2)
        ev[3 * k + 2].record()
    torch.cuda.synchronize()
    return {"gate_up_us": round(sum(ev[3 * k].elapsed_time(ev[3 * k + 1]) for k in range(n)) / n * 1e3, 1),
            "down_us": round(sum(ev[3 * k + 1].elapsed_time(ev[3 * k + 2]) for k in range(n)) / n * 1e3, 1),
            "what": "torch.mm x2 on the same layer (plain GEMMs, context only)"}


def others(mm, synth, torch, seed):
    """Short runs of the remaining workloads: tokens/s and the fraction of the roofline that bounds them."""
    res = {}
    for name, Ts in (("qwen05b", (2048, 1)), ("qwen05b_pruned", (2048, 16, 8, 1)), ("llama8b_fade", (4096, 16, 1)),
                     ("llama8b", (512, 256, 128, 64))):
        Tmax = max(Ts)
        L, x, dev, _, off, alpha, mask, d_eff = build_layer(mm, synth, name, Tmax, seed)
        w = L.workload
        wbytes = 3 * w.d_model * int(off[-1]) * 2
        for T in Ts:
            decode = T <= 16
            n_sets = max(2, int(np.ceil(2 * 256e6 / wbytes))) if decode else 1
            sets = [dev] + [[t.clone() for t in dev] for _ in range(n_sets - 1)]
            xT = x[:T].contiguous()
            out = torch.empty((T, w.d_model), dtype=torch.float32, device="cuda")

            def call(i, xT=xT, out=out, sets=sets):
                Wg, Wu, Wd = sets[i % len(sets)]
                mm.mlpmoe_forward_bf16(xT, Wg, Wu, Wd, off, alpha, mask, out=out)

            ms, pk = time_steps(mm, torch, call, 50 if decode else 20, 10 if decode else 5, events=False)
            ent = {"tokens_per_s": round(T / (ms * 1e-3), 1), "us_per_step": round(ms * 1e3, 2), "d_eff": d_eff,
                   "kernels_us": {k: round(1e3 * sum(v) / len(v), 2) for k, v in pk.items()}}
            if decode:
                byts = 3 * w.d_model * d_eff * 2 + T * w.d_model * 6
                ent["hbm_frac"] = round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                ent["weight_sets"] = len(sets)
            else:
                ent["mfma_frac"] = round(6.0 * T * w.d_model * d_eff / (ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4)
                if T < 512:      # between the two rooflines: the weight stream matters as much as the flops
                    byts = 3 * w.d_model * d_eff * 2 + T * w.d_model * 6
                    ent["hbm_frac"] = round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
            res["%s_T%d" % (name, T)] = ent
            del sets, out
        if name == "llama8b":
            # Sec. 3.3 swept over K on the same weights: keep the first K of 16 branches, alpha = sqrt(16/K)
            sweep = {}
            xs = mm.bf16_tensor(synth.make_layer(name, 4096, seed=seed).x)
            sets = [dev, [t.clone() for t in dev]]
            for K in (4, 8, 12, 16):
                offk, alphak, maskk, _ = mm.mlpmoe_slice(w.d_inter, w.B, K)
                row = {}
                for T in (4096, 1):
                    xT = xs[:T].contiguous()
                    out = torch.empty((T, w.d_model), dtype=torch.float32, device="cuda")

                    def callk(i, xT=xT, out=out):
                        Wg, Wu, Wd = sets[i % 2]
                        mm.mlpmoe_forward_bf16(xT, Wg, Wu, Wd, offk, alphak, maskk, out=out)

                    ms, _ = time_steps(mm, torch, callk, 20 if T > 16 else 50, 5, events=False)
                    row["T%d_us" % T] = round(ms * 1e3, 2)
                sweep["K%d" % K] = row
            res["llama8b_first_k_sweep"] = sweep
            # the same forward with the result stored as bf16 (T = 4096 and T = 1)
            o16 = {}
            for T in (4096, 1):
                xT = xs[:T].contiguous()
                out = torch.empty((T, w.d_model), dtype=torch.bfloat16, device="cuda")

                def call16(i, xT=xT, out=out):
                    Wg, Wu, Wd = sets[i % 2]
                    mm.mlpmoe_forward_bf16_out_bf16(xT, Wg, Wu, Wd, off, alpha, mask, out=out)

                ms, _ = time_steps(mm, torch, call16, 20 if T > 16 else 50, 5, events=False)
                o16["T%d_us" % T] = round(ms * 1e3, 2)
            res["llama8b_out_bf16"] = o16
            del sets, xs
            # per-token routing, 4 of 16 branches per token: tokens grouped by route (each tile of 256
            # tokens shares its 4 branches), random routes, and decode
            rt = {}
            xs = mm.bf16_tensor(synth.make_layer(name, 4096, seed=seed).x)
            off16, _, mask16, _ = mm.mlpmoe_slice(w.d_inter, w.B)
            rng = np.random.default_rng(seed)
            grouped = np.zeros((4096, w.B), np.uint8)
            for g in range(16):
                for j in range(4):
                    grouped[g * 256:(g + 1) * 256, (g + 3 * j) % w.B] = 1
            rand = np.zeros((4096, w.B), np.uint8)
            for t in range(4096):
                rand[t, rng.choice(w.B, size=4, replace=False)] = 1
            sets = [dev, [t.clone() for t in dev]]
            for tag, route, T in (("grouped_T4096", grouped, 4096), ("random_T4096", rand, 4096),
                                  ("top4_T1", rand, 1), ("top4_T16_same", grouped, 16)):
                r = torch.from_numpy(np.ascontiguousarray(route[:T])).cuda()
                xT = xs[:T].contiguous()
                out = torch.empty((T, w.d_model), dtype=torch.float32, device="cuda")

                def callr(i, xT=xT, out=out, r=r):
                    Wg, Wu, Wd = sets[i % 2]
                    mm.mlpmoe_forward_routed_bf16(xT, Wg, Wu, Wd, off16, alpha, mask16, r, out=out)

                ms, _ = time_steps(mm, torch, callr, 20 if T > 16 else 50, 5, events=False)
                rt[tag] = {"us_per_step": round(ms * 1e3, 2), "branches_per_token": 4}
            res["llama8b_routed_4_of_16"] = rt
            del sets, xs
            # Fractal Fade weight preparation (Sec. 3.2 schedule) on the same layer: the call is
            # synchronous (it returns thresholds), so wall-clock time around it is the cost
            best = None
            for _ in range(3):
                Wg, Wu = dev[0].clone(), dev[1].clone()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                mm.mlpmoe_fade(Wg, Wu, off)
                dt = time.perf_counter() - t0
                best = dt if best is None or dt < best else best
            touched = 2 * (w.d_inter - int(off[1])) * w.d_model * 2      # bytes of the faded blocks
            res["llama8b_fade_prep"] = {"ms": round(best * 1e3, 3), "bound": "hbm",
                                        "algorithmic_bytes": 3 * touched,   # read, read again, write
                                        "gbs": round(3 * touched / best / 1e9, 1),
                                        "hbm_frac": round(3 * touched / best / 1e9 / HBM_PEAK_GBS, 4)}
            # Context only, not part of the path: the two plain GEMMs of this layer (no SiLU*up pass, no branch
            # table, bf16 results) through the vendor library as PyTorch calls it, timed with events in the same
            # process on the same weights at the prefill sizes timed above; boxes differ by more than the
            # margin between the two, so the comparison is only meaningful inside one run.
            Wgu = torch.cat([dev[0], dev[1]])
            for Tl in (4096, 512, 256, 64):
                res["llama8b_T%d_library_gemms" % Tl] = library_gemms(torch, Wgu, dev[2], Tl)
            del Wgu
        del x, dev
        torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (tokens are independent, so more GPUs would just "
              "split the batch); --gpus %d is not supported." % args.gpus, file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback.", file=sys.stderr)
        return 3
    from paper_2511_21089_amd import binding as mm
    from paper_2511_21089_amd import synth

    L, x, dev, host, off, alpha, mask, d_eff = build_layer(mm, synth, args.workload, args.T, args.seed)
    w = L.workload
    T, d_model = args.T, w.d_model
    decode = T <= 16
    out = torch.empty((T, d_model), dtype=torch.float32, device="cuda")

    # decode-sized batches cycle through copies of the weights so that every pass is cold
    wbytes = 3 * d_model * int(off[-1]) * 2
    n_sets = max(1, int(np.ceil(2 * 256e6 / wbytes))) if decode else 1
    sets = [dev] + [[t.clone() for t in dev] for _ in range(n_sets - 1)]

    def call(i):
        Wg, Wu, Wd = sets[i % len(sets)]
        mm.mlpmoe_forward_bf16(x, Wg, Wu, Wd, off, alpha, mask, out=out)

    if args.copy_mib > 0:
        src = torch.ones(args.copy_mib * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)              # reads copy_mib MiB, writes copy_mib MiB
        torch.cuda.synchronize()
        del src, dst

    ms, per_kernel = time_steps(mm, torch, call, args.steps, args.warmup)
    result = {
        "metric": "MLP-layer tokens/s",
        "value": round(T / (ms * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s_T%d" % (args.workload, T), "d_model": d_model,
                   "d_inter": w.d_inter, "B": w.B, "d_eff": d_eff, "T": T,
                   "active_branches": int(mask.sum()), "weight_sets": len(sets)},
        "roofline": roofline_of(per_kernel, T, d_model, d_eff, decode, "%s_T%d" % (args.workload, T)),
        "kernels_us": {k: round(1e3 * sum(v) / len(v), 2) for k, v in per_kernel.items()},
        "kernel_timing": "HIP events around every kernel launch, in a second pass of the same %d steps" % args.steps,
    }
    flops = 6.0 * T * d_model * d_eff
    result["whole_path"] = {
        "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
        "mfma_frac": round(flops / (ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4),
        "gbs": round((3 * d_model * d_eff * 2 + T * d_model * 6) / (ms * 1e-3) / 1e9, 1),
    }
    result["whole_path"]["hbm_frac"] = round(result["whole_path"]["gbs"] / HBM_PEAK_GBS, 4)

    if not decode and not args.no_decode:
        # the second half of the metric: the same layer through the decode kernels
        n_sets = max(2, int(np.ceil(2 * 256e6 / wbytes)))
        sets = [dev] + [[t.clone() for t in dev] for _ in range(n_sets - 1)]
        dec = {}
        for Td in (16, 1):
            xd = x[:Td].contiguous()
            outd = torch.empty((Td, d_model), dtype=torch.float32, device="cuda")

            def calld(i, xd=xd, outd=outd):
                Wg, Wu, Wd = sets[i % len(sets)]
                mm.mlpmoe_forward_bf16(xd, Wg, Wu, Wd, off, alpha, mask, out=outd)

            msd, pk = time_steps(mm, torch, calld, 50, 10, events=False)
            byts = 3 * d_model * d_eff * 2 + Td * d_model * 6
            dec["T%d" % Td] = {"tokens_per_s": round(Td / (msd * 1e-3), 1), "us_per_step": round(msd * 1e3, 2),
                               "gbs": round(byts / (msd * 1e-3) / 1e9, 1),
                               "hbm_frac": round(byts / (msd * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                               "roofline": roofline_of(pk, Td, d_model, d_eff, True, "%s_T%d" % (args.workload, Td)),
                               "kernels_us": {k: round(1e3 * sum(v) / len(v), 2) for k, v in pk.items()}}
        dec["weight_sets"] = len(sets)
        result["decode"] = dec
        del sets

    if not args.no_others and args.workload == "llama8b" and T == 4096:
        # context: the other configurations, a few steps each (same code path, same timing rules)
        del x, dev, out
        result["other_workloads"] = others(mm, synth, torch, args.seed)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(synth, L, host, off, alpha, mask, args.cpu_seconds)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
