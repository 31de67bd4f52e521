#!/usr/bin/env python3
"""Benchmark of the LoQT hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input for one
transformer block: loqt_linear_fwd + loqt_linear_bwd for each of the 7 projections, then the
merge + NF4 requantisation of all 7 weights (loqt_merge_requant_batched).  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line (see README / DESIGN for the fields).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b_block] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E

METRIC = "LoQT NF4 linear fwd+bwd TFLOP/s at 7B shapes; merge+requant GB/s"

# HBM-side traffic of the dominant kernel per launch, from profiles/bench_7b_block_hbm_traffic.md
# per gemm_y launch slot: 256x256 kernel fetch 674.9 MB + write 98.3 MB, plus 2/7 of the 128x128 tail
# launch of the gate and up projections (117.6 + 12.6 MB); null for workloads that were not profiled.
TRAFFIC_BYTES_PER_LAUNCH = {"7b_block": 810.4e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b_block")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--mode", choices=["saved", "plain"], default="saved",
                    help="saved: forward of all projections with loqt_linear_fwd_save, then backward in reverse order "
                         "with loqt_linear_bwd_saved (the transient bf16 weight of each layer is kept in between, "
                         "one fold per layer and step); plain: loqt_linear_fwd + loqt_linear_bwd layer by layer "
                         "(nothing kept, the weight is folded in both passes).  The other mode is timed too and "
                         "reported beside the headline.")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the supplementary timings (codec streams, small-rank merges, the Alg. 2 loop)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of 1 GiB (reference dispatch for HBM byte counters)")
    return ap.parse_args()


def cpu_baseline(wl, seed, sample_T):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload:
    forward + backward of every projection of the block on `sample_T` tokens (each output row
    depends only on its own token, so a token subset is the same arithmetic per token)."""
    from oracle import loqt_oracle as O
    from paper_2405_16528_amd import synth
    picks = range(len(wl.projections))
    secs, flops, names = 0.0, 0, []
    for pi in picks:
        name, out, inp = wl.projections[pi]
        lay = synth.make_layer(wl.name, name, out, inp, wl.r, sample_T, seed)
        Wq, Pq = O.nf4_quantize(lay.W), O.nf4_quantize(lay.P)
        t0 = time.perf_counter()
        O.loqt_linear_fwd(lay.x, Wq, Pq, lay.B, 1.0)
        O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, 1.0)
        secs += time.perf_counter() - t0
        flops += synth.flops_fwd(sample_T, out, inp, wl.r) + synth.flops_bwd(sample_T, out, inp, wl.r)
        names.append(f"{name}:{out}x{inp}")
        del lay, Wq, Pq
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        cores = min(cores, int(env))
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"fwd+bwd of projections {', '.join(names)} (r={wl.r}) of {wl.name} on {sample_T} of "
                      f"{wl.T} tokens, numpy float64, {secs:.1f} s of oracle time",
            "seconds": secs}


def extras(L, synth, torch, wl, full_precision, layers):
    """Supplementary timings outside the K timed steps (not part of `value`): the HBM-bound codec
    streams, the merge at ranks where the product no longer binds, and the error-compensated
    initialisation loop (Alg. 2), per distinct projection shape.  HIP events around 10 back-to-back calls."""
    dev = "cuda"

    def timed_us(fn, reps=10, warm=2):
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    res = {"codec": [], "absmax_dq": [], "merge_small_rank": [], "init_compensate": []}
    for (out, inp), (Wd, Pd) in full_precision.items():
        n = out * inp
        Wq = L.nf4_quantize(Wd)
        Wb = torch.empty((out, (inp + 7) // 8 * 8), dtype=torch.bfloat16, device=dev)[:, :inp]
        t_q = timed_us(lambda: L.nf4_quantize(Wd, out=Wq))
        t_d = timed_us(lambda: L.nf4_dequantize(Wq, Wb))
        res["codec"].append({"shape": f"{out}x{inp}", "quantize_us": t_q, "quantize_GBs": n * 4.5625 / t_q / 1e3,
                             "quantize_frac_hbm": n * 4.5625 / t_q / 1e3 / PEAK_HBM_GBS,
                             "dequantize_bf16_us": t_d, "dequantize_bf16_GBs": n * 2.5625 / t_d / 1e3,
                             "dequantize_frac_hbm": n * 2.5625 / t_d / 1e3 / PEAK_HBM_GBS})
        del Wb
        # double-quantised block scales (sec. 2.4): three launches over n / 64 scales (launch-sized), the storage
        # they buy, and what the 8-bit scales do to the dequantised weight
        a = Wq.absmax.reshape(-1)
        dq = L.loqt_absmax_dq_compress(a)
        a2 = L.loqt_absmax_dq_expand(*dq)
        t_c = timed_us(lambda: L.loqt_absmax_dq_compress(a))
        t_e = timed_us(lambda: L.loqt_absmax_dq_expand(*dq, out=a2))
        res["absmax_dq"].append({"shape": f"{out}x{inp}", "scales": a.numel(), "compress_us": t_c, "expand_us": t_e,
                                 "bytes_per_weight": 0.5 + (a.numel() + 4 * dq[1].numel() + 4) / n,
                                 "bytes_per_weight_fp32_scales": 0.5 + 4 * a.numel() / n,
                                 "rms_rel_change_of_scales": float(((a2 - a).double().pow(2).mean().sqrt()
                                                                   / a.double().pow(2).mean().sqrt()).item())})
        Wq_out = L.NF4Tensor.empty(out, inp)
        for r in (64, 128):
            Pq = L.nf4_quantize(Pd[:, :r].contiguous())
            B = (torch.randn((r, inp), device=dev, generator=gen) * 1e-3).to(torch.bfloat16)
            ws = L.workspace(L.OP_MERGE, 0, out, inp, r)
            t = timed_us(lambda: L.loqt_merge_requant(Wq, Pq, B, 1.0, out=Wq_out, ws=ws))
            byts, fl = synth.bytes_merge(out, inp, r), synth.flops_merge(out, inp, r)
            res["merge_small_rank"].append({"shape": f"{out}x{inp}", "rank": r, "us": t, "algorithmic_GBs": byts / t / 1e3,
                                            "frac_of_hbm_peak": byts / t / 1e3 / PEAK_HBM_GBS,
                                            "tflops": fl / t / 1e6})
        # Alg. 2 loop, five steps from B = 0: step c costs two rank-r products of 2 out in r flop (the first
        # step has no W - s P B product) and streams W (4 B), Q_c (0.5625 B) and the residual (2 + 2 B) per element
        r, iters = wl.r, 5
        B = torch.empty((r, (inp + 7) // 8 * 8), dtype=torch.bfloat16, device=dev)[:, :inp]
        ws = L.workspace(L.OP_INIT, 0, out, inp, r)
        t = timed_us(lambda: L.loqt_init_compensate(Wd, Pd, 1.0, iters, B, out=Wq_out, ws=ws), reps=3, warm=1)
        fl = (2 * iters - 1) * 2.0 * out * inp * r
        res["init_compensate"].append({"shape": f"{out}x{inp}", "rank": r, "iters": iters, "us": t,
                                       "tflops": fl / t / 1e6, "frac_of_bf16_peak": fl / t / 1e6 / PEAK_BF16_TFLOPS})
    # Merge sweep over a whole 13B model (40 blocks x 7 projections, 280 distinct NF4 weights = 7.1 GB
    # resident, far beyond the 256 MB Infinity Cache): the streaming figure of record for the merge.
    w13 = synth.WORKLOADS["13b_block"]
    shapes = {}
    sweep = []
    for (name, out, inp) in w13.projections:
        if (out, inp) not in shapes:
            Pq = L.nf4_quantize(torch.randn((out, w13.r), device=dev, generator=gen) / out ** 0.5)
            B = (torch.randn((w13.r, inp), device=dev, generator=gen) * 1e-3).to(torch.bfloat16)
            shapes[(out, inp)] = (Pq, B)
    for _ in range(w13.n_blocks):
        for (name, out, inp) in w13.projections:
            W = torch.empty((out, inp), device=dev, dtype=torch.float32).normal_(0.0, 0.02, generator=gen)
            Wq = L.nf4_quantize(W)
            del W
            Pq, B = shapes[(out, inp)]
            sweep.append((Wq, None, Pq, B, 1.0))  # in place
    descs = L.make_merge_descs(sweep)
    ws = torch.empty(L.merge_descs_workspace_bytes(descs), dtype=torch.uint8, device=dev)
    t = timed_us(lambda: L.loqt_merge_requant_batched(descs, ws), reps=2, warm=1)
    byts = w13.n_blocks * sum(synth.bytes_merge(o, i, w13.r) for (_, o, i) in w13.projections)
    fl = w13.n_blocks * sum(synth.flops_merge(o, i, w13.r) for (_, o, i) in w13.projections)
    t_hbm, t_mfma = byts / (PEAK_HBM_GBS * 1e9) * 1e6, fl / (PEAK_BF16_TFLOPS * 1e12) * 1e6
    res["merge_sweep_13b"] = {"layers": len(sweep), "rank": w13.r, "ms": t / 1e3, "algorithmic_GBs": byts / t / 1e3,
                              "frac_of_hbm_peak": t_hbm / t, "tflops": fl / t / 1e6,
                              "frac_of_binding_roof": max(t_hbm, t_mfma) / t}
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (got --gpus {args.gpus}); "
              "there is no multi-GPU path to time.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2405_16528_amd import binding as L
    from paper_2405_16528_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    T, r = wl.T, wl.r
    dev = "cuda"
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)

    def pitch8(n):
        return (n + 7) // 8 * 8

    def randn_bf16(rows, cols, sigma):
        buf = torch.empty((rows, pitch8(cols)), dtype=torch.float32, device=dev)
        buf.normal_(0.0, sigma, generator=gen)
        return buf.to(torch.bfloat16)[:, :cols]

    layers = []
    full_precision = {}
    ws_bytes = 256
    for (name, out, inp) in wl.projections:
        # W and P are drawn on the host by the seeded generator (P needs a QR), x / dy / B on the device
        W = synth.normal_f32(synth.rng_for(args.seed, wl.name, 0, name, "W"), (out, inp), 0.02)
        P = synth.orthonormal_f32(synth.rng_for(args.seed, wl.name, 0, name, "P"), out, r)
        Wd = torch.from_numpy(W).to(dev)
        if inp % 4:
            Wp = torch.zeros((out, (inp + 3) // 4 * 4), dtype=torch.float32, device=dev)
            Wp[:, :inp] = Wd
            Wd = Wp[:, :inp]
        Wq = L.nf4_quantize(Wd)
        Pd = torch.from_numpy(P).to(dev)
        Pq = L.nf4_quantize(Pd)
        if not args.no_extras and (out, inp) not in full_precision:
            full_precision[(out, inp)] = (Wd, Pd)  # one fp32 W and P per distinct shape, for the extras
        del Wd, Pd
        lay = dict(name=name, out=out, inp=inp, Wq=Wq, Pq=Pq,
                   Wq_out=L.NF4Tensor.empty(out, inp),
                   B=randn_bf16(r, inp, 1e-3), x=randn_bf16(T, inp, 1.0), dy=randn_bf16(T, out, 1e-2),
                   y=torch.empty((T, pitch8(out)), dtype=torch.bfloat16, device=dev)[:, :out],
                   dx=torch.empty((T, pitch8(inp)), dtype=torch.bfloat16, device=dev)[:, :inp],
                   dB=torch.empty((r, inp), dtype=torch.float32, device=dev))
        layers.append(lay)
        ws_bytes = max(ws_bytes, L.loqt_workspace_bytes(L.OP_BWD, T, out, inp, r),
                       L.loqt_workspace_bytes(L.OP_FWD, T, out, inp, r),
                       L.loqt_workspace_bytes(L.OP_MERGE, T, out, inp, r))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    for l in layers:  # the transient bf16 weight of the saved mode: out x in per layer (0.4 GB for the 7B block)
        l["w_eff"] = torch.empty((l["out"], pitch8(l["inp"])), dtype=torch.bfloat16, device=dev)[:, :l["inp"]]
    descs = L.make_merge_descs([(l["Wq"], l["Wq_out"], l["Pq"], l["B"], 1.0) for l in layers])
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    phase_events = []

    mode = args.mode

    def step(record=False):
        if record:
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
        if mode == "saved":
            for l in layers:
                L.loqt_linear_fwd_save(l["x"], l["Wq"], l["Pq"], l["B"], 1.0, l["y"], l["w_eff"], ws)
            for l in reversed(layers):
                L.loqt_linear_bwd_saved(l["dy"], l["x"], l["Pq"], 1.0, l["w_eff"], l["dx"], l["dB"], False, ws)
        else:
            for l in layers:
                L.loqt_linear_fwd(l["x"], l["Wq"], l["Pq"], l["B"], 1.0, l["y"], ws)
                L.loqt_linear_bwd(l["dy"], l["x"], l["Wq"], l["Pq"], l["B"], 1.0, l["dx"], l["dB"], False, ws)
        if record:
            e1.record()
        L.loqt_merge_requant_batched(descs, ws)
        if record:
            e2.record()
            phase_events.append((e0, e1, e2))

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: K steps, three events per step (start, after fwd+bwd, after merge), nothing else
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(record=True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # a second pass of K steps with the library's per-launch HIP events on the launch stream (the kernel
    # breakdown and the roofline object come from here; the events cost about 2 % of the step, so they
    # stay out of the region `value` is measured on)
    timed_events = list(phase_events)
    L.timing_enable(True)
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    L.timing_enable(False)
    kt = L.timing_read()
    # the other mode, timed the same way as the headline (reported beside it, not part of `value`)
    other = "plain" if args.mode == "saved" else "saved"
    mode, phase_events = other, []
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    for _ in range(args.steps):
        step(record=True)
    torch.cuda.synchronize()
    t5 = time.perf_counter()
    other_events, mode = phase_events, args.mode
    phase_events = timed_events
    ms_step_instrumented = (t3 - t2) * 1e3 / args.steps

    ms_step = (t1 - t0) * 1e3 / args.steps
    f_fb = sum(synth.flops_fwd(T, o, i, r) + synth.flops_bwd(T, o, i, r) for (_, o, i) in wl.projections)
    f_mg = sum(synth.flops_merge(o, i, r) for (_, o, i) in wl.projections)
    b_mg = sum(synth.bytes_merge(o, i, r) for (_, o, i) in wl.projections)
    ms_fb = sum(a.elapsed_time(b) for (a, b, _) in phase_events) / args.steps
    ms_mg = sum(b.elapsed_time(c) for (_, b, c) in phase_events) / args.steps

    # flops each kernel actually executes over one step (depends on the implementation the library picks)
    saved = args.mode == "saved"
    folded = {n: saved or L.resolved_path(L.OP_FWD, T, o, i) == L.PATH_FOLDED for (n, o, i) in wl.projections}
    kflops = {
        "gemm_u": sum(2 * T * i * r for (n, o, i) in wl.projections if not folded[n]),
        "gemm_y": sum(2 * T * o * (i + (0 if folded[n] else r)) for (n, o, i) in wl.projections),
        # folded: Z may ride along with dx ([dx | Z] = dy [W_eff | s deq(P)]); its flops are then in gemm_dx
        "gemm_z+dx": sum(2 * T * o * (i + r) if folded[n] else 2 * T * (o * r + i * (o + r))
                         for (n, o, i) in wl.projections),
        "gemm_db": sum(2 * T * r * i for (n, o, i) in wl.projections),
        "fold_weight": sum((1 if saved else 2) * 2 * o * i * r for (n, o, i) in wl.projections if folded[n]),
        "merge_requant": f_mg,
    }
    f_exec = sum(v for k, v in kflops.items() if k != "merge_requant")
    kernels = {}
    if "gemm_z" in kt or "gemm_dx" in kt:
        nz, mz = kt.pop("gemm_z", (0, 0.0))
        nd, md = kt.pop("gemm_dx", (0, 0.0))
        kt["gemm_z+dx"] = (nz + nd, mz + md)
    for name, (n, ms) in kt.items():
        if n == 0:
            continue
        ent = {"launches_per_step": n / args.steps, "ms_per_step": ms / args.steps, "avg_ms": ms / n}
        if name in kflops:
            ent["tflops"] = kflops[name] * args.steps / (ms * 1e-3) / 1e12
        kernels[name] = ent
    # dominant kernel: the K-contiguous 256x256 bf16-epilogue instantiation, i.e. the gemm_y launches
    dom_slots = [k for k in ("gemm_y",) if k in kernels]
    dom_ms = sum(kernels[k]["ms_per_step"] for k in dom_slots)
    dom_launches = sum(kernels[k]["launches_per_step"] for k in dom_slots)
    dom_flops = sum(kflops[k] for k in dom_slots)
    dom_tflops = dom_flops / (dom_ms * 1e-3) / 1e12
    roofline = {
        "kernel": "nt_gemm_kernel<256,256,EPI_BF16,false,false> (the gemm_y launches: y = x W_eff^T; for 11008 "
                  "output columns the last 768 run as a 128x128-tile launch inside the same timed slot)",
        "bound": "mfma",
        "achieved": dom_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": dom_tflops / PEAK_BF16_TFLOPS,
        "flops_per_launch": dom_flops / dom_launches, "avg_launch_ms": dom_ms / dom_launches,
        # HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE, rocprofv3 --pmc, scaled by a plain copy):
        # see profiles/bench_7b_block_hbm_traffic.md; not measurable from inside this process
        "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(wl.name),
    }
    # the merge is bound by max(HBM stream, rank-r bf16 product); report both views.  Time: the whole
    # loqt_merge_requant_batched call of the timed region (pre-pass of P included), not the kernel slot alone
    t_hbm = b_mg / (PEAK_HBM_GBS * 1e9) * 1e3
    t_mfma = f_mg / (PEAK_BF16_TFLOPS * 1e12) * 1e3
    merge = {"ms_per_step": ms_mg, "algorithmic_GBs": b_mg / (ms_mg * 1e-3) / 1e9,
             "tflops": f_mg / (ms_mg * 1e-3) / 1e12, "t_hbm_ms": t_hbm, "t_mfma_ms": t_mfma,
             "frac_of_binding_roof": max(t_hbm, t_mfma) / ms_mg, "frac_of_hbm_peak": t_hbm / ms_mg}

    out = {
        "metric": METRIC,
        "value": (f_fb + f_mg) / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "tokens": T, "rank": r,
                   "projections": [f"{n}:{o}x{i}" for (n, o, i) in wl.projections],
                   "mode": args.mode,
                   "step": ("loqt_linear_fwd_save of the 7 projections, loqt_linear_bwd_saved of the 7 in reverse order "
                            "(W_eff bf16 kept per layer in between: %.2f GB), batched merge/requant of the block"
                            % (sum(o * pitch8(i) for (_, o, i) in wl.projections) * 2 / 1e9)) if saved else
                           "7x(loqt_linear_fwd + loqt_linear_bwd) + batched merge/requant of the block"},
        "fwd_bwd": {"tflops": f_fb / (ms_fb * 1e-3) / 1e12, "ms_per_step": ms_fb,
                    "flop_model": "algorithmic, factored form: fwd 2T(out*in + in*r + r*out), bwd 2T(out*in + out*r + 2*r*in)",
                    "executed_tflops": f_exec / (ms_fb * 1e-3) / 1e12,
                    "paths": ["folded"] if saved else
                             sorted({["auto", "fused", "prepass", "folded"][L.resolved_path(L.OP_FWD, T, o, i)]
                                     for (_, o, i) in wl.projections}),
                    "frac_of_bf16_peak": f_fb / (ms_fb * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "merge": merge,
        "other_mode": {"mode": other, "ms_per_step": (t5 - t4) * 1e3 / args.steps,
                       "value": (f_fb + f_mg) / ((t5 - t4) / args.steps) / 1e12,
                       "fwd_bwd_ms_per_step": sum(a.elapsed_time(b) for (a, b, _) in other_events) / args.steps,
                       "fwd_bwd_tflops": f_fb / (sum(a.elapsed_time(b) for (a, b, _) in other_events) / args.steps
                                                 * 1e-3) / 1e12},
        "kernels": kernels,
        "kernels_pass": {"steps": args.steps, "ms_per_step": ms_step_instrumented,
                         "note": "per-kernel figures and the roofline object: a second pass of the same K steps "
                                 "with a HIP event pair around every launch"},
        "roofline": roofline,
    }
    if not args.no_extras:
        out["extras"] = extras(L, synth, torch, wl, full_precision, layers)
        # the same step captured once as a HIP graph and replayed (the library allocates nothing and keeps no
        # state, so the capture holds only its kernels): what the gaps between the launches of a step cost
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t6 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t7 = time.perf_counter()
        out["extras"]["graph_replay"] = {"mode": args.mode, "ms_per_step": (t7 - t6) * 1e3 / args.steps,
                                         "value": (f_fb + f_mg) / ((t7 - t6) / args.steps) / 1e12}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.seed, min(args.cpu_sample_tokens, T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
