#!/usr/bin/env python3
"""Benchmark of the LoQT hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input for one
transformer block: loqt_linear_fwd + loqt_linear_bwd for each of the 7 projections (nothing kept
between the two calls), then the merge + NF4 requantisation of all 7 weights
(loqt_merge_requant_batched).  Inputs are resident in HBM before the timed region.  Prints ONE
JSON line: the whole-step rate (`value`), forward + backward alone (`fwd_bwd`, algorithmic and executed flops), the
merge against its roofs (`merge`), the other mode (`other_mode`), per-kernel timings (`kernels`), the roofline of
the dominant kernel (`roofline`, `roofline_dx`), supplementary timings (`extras`), the oracle timed on the host
(`cpu_baseline`) and the parity of the library against it on all five workloads (`parity`).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b_block] [--mode plain|saved]
                    [--no-extras] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E

METRIC = "LoQT NF4 linear fwd+bwd TFLOP/s at 7B shapes; merge+requant GB/s"
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_7b_block_hbm_traffic.md")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b_block")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--mode", choices=["plain", "saved"], default="plain",
                    help="plain (the headline): loqt_linear_fwd + loqt_linear_bwd layer by layer, nothing kept between "
                         "the two calls (the 16-bit weight is rebuilt from the 4-bit codes in both passes); saved: "
                         "loqt_linear_fwd_save for all projections, then loqt_linear_bwd_saved in reverse order (the "
                         "transient bf16 weight of every layer is kept in between).  The other mode is timed too and "
                         "reported beside the headline.")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle leg (cpu_baseline and the parity numbers, which need the oracle)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the supplementary timings (codec streams, small-rank merges, the Alg. 2 loop, the other "
                         "workloads, the 13B merge sweep)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of 1 GiB (reference dispatch for HBM byte counters)")
    return ap.parse_args()


def traffic_from_profile(workload):
    """HBM-side bytes per gemm_y timing slot (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc, scaled by a plain copy)
    from the committed counter summary, or None when the file does not cover the workload or the kernels it names
    no longer exist under those names.  A slot is one launch of the 256x256 kernel plus, for the gate and up
    projections (2 of 7 launches), the tail launch on 256x128 tiles."""
    if workload != "7b_block" or not os.path.exists(TRAFFIC_PROFILE):
        return None
    big = small = None
    for line in open(TRAFFIC_PROFILE):
        cells = [c.strip() for c in line.split("|")]
        if len(cells) < 7 or "nt_gemm_kernel" not in cells[1]:
            continue
        try:
            mb = float(cells[4]) + float(cells[6])
        except ValueError:
            continue
        if "<256, 256, 0, false, false, 2, true>" in cells[1]:
            big = mb
        elif "<256, 128, 0, false, false, 2, true>" in cells[1]:
            small = mb
    if big is None or small is None:
        return None
    return (big + small * 2.0 / 7.0) * 1e6


def bf16_bits_host(t):
    import numpy as np
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def oracle_leg(L, torch, synth, seed, sample_T):
    """Everything that needs the CPU oracle: (1) cpu_baseline, the oracle as it stands timed on the host cores on
    forward + backward of every projection of the 7B block; (2) parity numbers of the library against it, on the
    same seeded inputs, in the launch configuration the bench times (plain calls, implementation chosen from the
    sizes), for all five workloads.  Inputs are quantised by the oracle and uploaded: nothing the oracle sees comes
    from the HIP path."""
    import numpy as np
    from oracle import loqt_oracle as O
    dev = "cuda"

    def up_bf16(bits):
        rows, cols = bits.shape
        ld = (cols + 7) // 8 * 8
        buf = np.zeros((rows, ld), dtype=np.uint16)
        buf[:, :cols] = bits
        return torch.from_numpy(buf.view(np.int16)).to(dev).view(torch.bfloat16)[:, :cols]

    def up_nf4(q):
        codes, absmax = q
        rows, cols = codes.shape
        ld = (cols + 63) // 64 * 64
        packed, am = O.pack_nf4(codes, absmax, ld)
        return L.NF4Tensor(torch.from_numpy(packed).to(dev), torch.from_numpy(am).to(dev), rows, cols, ld)

    def empty_bf16(rows, cols):
        return torch.empty((rows, (cols + 7) // 8 * 8), dtype=torch.bfloat16, device=dev)[:, :cols]

    def err(got, ref):
        return float(np.abs(got - ref).max() / np.sqrt(np.mean(ref ** 2)))

    def floor(ref):
        """max |err| / RMS of the oracle's own values rounded to bf16: what the output format allows at all (over
        ~10^8 outputs it comes close to the 2e-2 bound by itself)"""
        return err(O.bf16_to_f64(O.f32_to_bf16_rne(ref.astype(np.float32))), ref)

    def worse(acc, ey, ex, eb, fy, fx):
        return {"y": max(acc["y"], ey), "dx": max(acc["dx"], ex), "dB": max(acc["dB"], eb),
                "y_bf16_format_floor": max(acc["y_bf16_format_floor"], fy),
                "dx_bf16_format_floor": max(acc["dx_bf16_format_floor"], fx)}

    zero = {"y": 0.0, "dx": 0.0, "dB": 0.0, "y_bf16_format_floor": 0.0, "dx_bf16_format_floor": 0.0}

    def gpu_layer(lay, Wq, Pq, T, s):
        out, inp, r = lay.out, lay.inp, lay.r
        x, dy, B = up_bf16(lay.x), up_bf16(lay.dy), up_bf16(lay.B)
        Wd, Pd = up_nf4(Wq), up_nf4(Pq)
        y, dx = empty_bf16(T, out), empty_bf16(T, inp)
        dB = torch.empty((r, inp), dtype=torch.float32, device=dev)
        ws = torch.empty(max(L.loqt_workspace_bytes(L.OP_FWD, T, out, inp, r),
                             L.loqt_workspace_bytes(L.OP_BWD, T, out, inp, r),
                             L.loqt_workspace_bytes(L.OP_MERGE, T, out, inp, r), 256), dtype=torch.uint8, device=dev)
        L.loqt_linear_fwd(x, Wd, Pd, B, s, y, ws)
        L.loqt_linear_bwd(dy, x, Wd, Pd, B, s, dx, dB, False, ws)
        merged = L.loqt_merge_requant(Wd, Pd, B, s, out=L.NF4Tensor.empty(out, inp), ws=ws)
        torch.cuda.synchronize()
        return y, dx, dB, merged

    def merge_numbers(merged, Wq, Pq, B, s, rows):
        """Code mismatches against the oracle's merge on `rows` rows of the weight (blocks run along rows, so a
        row subset is the same arithmetic)."""
        cols = Wq[0].shape[1]
        c, a = O.unpack_nf4(merged.codes[torch.from_numpy(rows).to(dev)].cpu().numpy(),
                            merged.absmax[torch.from_numpy(rows).to(dev)].cpu().numpy(), cols)
        c_ref, a_ref = O.loqt_merge_requant((Wq[0][rows], Wq[1][rows]), (Pq[0][rows], Pq[1][rows]), B, s)
        diff = c.astype(np.int32) - c_ref.astype(np.int32)
        rel = np.abs(a.astype(np.float64) - a_ref) / np.maximum(np.abs(a_ref.astype(np.float64)), 1e-300)
        return {"codes_compared": int(diff.size), "code_mismatches": int(np.count_nonzero(diff)),
                "mismatches_by_more_than_one_level": int(np.count_nonzero(np.abs(diff) > 1)),
                "absmax_max_rel_err": float(rel.max())}

    parity = []
    # ---- the 7B block in full: timed oracle (cpu_baseline) + every element of y, dx, dB of every projection
    wl = synth.WORKLOADS["7b_block"]
    T = min(sample_T, wl.T)
    secs, flops, names = 0.0, 0, []
    s = 1.0
    worst = dict(zero)
    mg = {"codes_compared": 0, "code_mismatches": 0, "mismatches_by_more_than_one_level": 0, "absmax_max_rel_err": 0.0}
    for (name, out, inp) in wl.projections:
        lay = synth.make_layer(wl.name, name, out, inp, wl.r, T, seed)
        Wq, Pq = O.nf4_quantize(lay.W), O.nf4_quantize(lay.P)
        t0 = time.perf_counter()
        y_ref = O.loqt_linear_fwd(lay.x, Wq, Pq, lay.B, s)
        dx_ref, dB_ref = O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, s)
        secs += time.perf_counter() - t0
        flops += synth.flops_fwd(T, out, inp, wl.r) + synth.flops_bwd(T, out, inp, wl.r)
        names.append(f"{name}:{out}x{inp}")
        y, dx, dB, merged = gpu_layer(lay, Wq, Pq, T, s)
        worst = worse(worst, err(O.bf16_to_f64(bf16_bits_host(y)), y_ref), err(O.bf16_to_f64(bf16_bits_host(dx)), dx_ref),
                      err(dB.cpu().numpy().astype(np.float64), dB_ref), floor(y_ref), floor(dx_ref))
        rows = np.unique(np.linspace(0, out - 1, 64).astype(np.int64))
        m = merge_numbers(merged, Wq, Pq, lay.B, s, rows)
        for k in ("codes_compared", "code_mismatches", "mismatches_by_more_than_one_level"):
            mg[k] += m[k]
        mg["absmax_max_rel_err"] = max(mg["absmax_max_rel_err"], m["absmax_max_rel_err"])
        del lay, Wq, Pq, y_ref, dx_ref, dB_ref, y, dx, dB, merged
        torch.cuda.empty_cache()
    parity.append({"workload": wl.name, "tokens": T, "projections": "all 7", "compared": "every element of y, dx, dB",
                   "max_abs_err_over_rms": worst, "merge": dict(mg, rows_per_projection=64)})
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        cores = min(cores, int(env))
    baseline = {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                "sample": f"fwd+bwd of projections {', '.join(names)} (r={wl.r}) of {wl.name} on {T} of "
                          f"{wl.T} tokens, numpy float64, {secs:.1f} s of oracle time",
                "seconds": secs}

    # ---- the other four workloads: every element for the small ones, sampled token rows / dB patches for 13B
    plan = [("60m_layer", None, False), ("130m_block", None, False), ("1b_block", ("q", "up", "down"), False),
            ("13b_block", ("o", "down"), True)]
    for wname, pick, sampled in plan:
        wl = synth.WORKLOADS[wname]
        T = wl.T
        worst = dict(zero)
        mg = {"codes_compared": 0, "code_mismatches": 0, "mismatches_by_more_than_one_level": 0,
              "absmax_max_rel_err": 0.0}
        used = []
        for (name, out, inp) in wl.projections:
            if pick is not None and name not in pick:
                continue
            used.append(name)
            lay = synth.make_layer(wl.name, name, out, inp, wl.r, T, seed)
            Wq, Pq = O.nf4_quantize(lay.W), O.nf4_quantize(lay.P)
            y, dx, dB, merged = gpu_layer(lay, Wq, Pq, T, 0.5)
            if sampled:
                I = np.unique(np.linspace(0, T - 1, 512).astype(np.int64))
                Id = torch.from_numpy(I).to(dev)
                y_ref = O.loqt_linear_fwd(lay.x[I], Wq, Pq, lay.B, 0.5)
                dx_ref, _ = O.loqt_linear_bwd(lay.dy[I], lay.x[I], Wq, Pq, lay.B, 0.5)
                ey = err(O.bf16_to_f64(bf16_bits_host(y[Id])), y_ref)
                ex = err(O.bf16_to_f64(bf16_bits_host(dx[Id])), dx_ref)
                # dB on (rank block x column block) patches over all tokens
                Rb = np.unique(np.linspace(0, (wl.r - 1) // 64, 3).astype(np.int64))
                Jb = np.unique(np.linspace(0, (inp - 1) // 64, 4).astype(np.int64))
                R = np.concatenate([np.arange(64 * b, min(64 * b + 64, wl.r)) for b in Rb])
                J = np.concatenate([np.arange(64 * b, min(64 * b + 64, inp)) for b in Jb])
                _, dB_ref = O.loqt_linear_bwd(lay.dy, np.ascontiguousarray(lay.x[:, J]),
                                              (np.ascontiguousarray(Wq[0][:, J]), np.ascontiguousarray(Wq[1][:, Jb])),
                                              (np.ascontiguousarray(Pq[0][:, R]), np.ascontiguousarray(Pq[1][:, Rb])),
                                              np.ascontiguousarray(lay.B[R][:, J]), 0.5)
                got = dB[torch.from_numpy(R).to(dev)][:, torch.from_numpy(J).to(dev)].cpu().numpy().astype(np.float64)
                eb = err(got, dB_ref)
            else:
                y_ref = O.loqt_linear_fwd(lay.x, Wq, Pq, lay.B, 0.5)
                dx_ref, dB_ref = O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, 0.5)
                ey = err(O.bf16_to_f64(bf16_bits_host(y)), y_ref)
                ex = err(O.bf16_to_f64(bf16_bits_host(dx)), dx_ref)
                eb = err(dB.cpu().numpy().astype(np.float64), dB_ref)
            worst = worse(worst, ey, ex, eb, floor(y_ref), floor(dx_ref))
            rows = np.unique(np.linspace(0, out - 1, 64).astype(np.int64))
            m = merge_numbers(merged, Wq, Pq, lay.B, 0.5, rows)
            for k in ("codes_compared", "code_mismatches", "mismatches_by_more_than_one_level"):
                mg[k] += m[k]
            mg["absmax_max_rel_err"] = max(mg["absmax_max_rel_err"], m["absmax_max_rel_err"])
            del lay, Wq, Pq, y, dx, dB, merged
            torch.cuda.empty_cache()
        parity.append({"workload": wl.name, "tokens": T, "projections": ",".join(used),
                       "compared": ("512 token rows of y and dx, (rank block x column block) patches of dB over all "
                                    "tokens") if sampled else "every element of y, dx, dB",
                       "max_abs_err_over_rms": worst, "merge": dict(mg, rows_per_projection=64)})
    return baseline, parity


class BlockBench:
    """Buffers and the step of one workload (one transformer block): forward + backward of every projection, then
    the batched merge of the block."""

    def __init__(self, L, synth, torch, wl, seed, keep_full_precision=False):
        self.L, self.torch, self.wl = L, torch, wl
        dev = "cuda"
        gen = torch.Generator(device=dev)
        gen.manual_seed(seed)
        T, r = wl.T, wl.r

        def pitch8(n):
            return (n + 7) // 8 * 8

        def randn_bf16(rows, cols, sigma):
            buf = torch.empty((rows, pitch8(cols)), dtype=torch.float32, device=dev)
            buf.normal_(0.0, sigma, generator=gen)
            return buf.to(torch.bfloat16)[:, :cols]

        self.layers, self.full_precision = [], {}
        ws_bytes = 256
        for (name, out, inp) in wl.projections:
            # W and P are drawn on the host by the seeded generator (P needs a QR), x / dy / B on the device
            W = synth.normal_f32(synth.rng_for(seed, wl.name, 0, name, "W"), (out, inp), 0.02)
            P = synth.orthonormal_f32(synth.rng_for(seed, wl.name, 0, name, "P"), out, r)
            Wd = torch.from_numpy(W).to(dev)
            if inp % 4:
                Wp = torch.zeros((out, (inp + 3) // 4 * 4), dtype=torch.float32, device=dev)
                Wp[:, :inp] = Wd
                Wd = Wp[:, :inp]
            Wq = L.nf4_quantize(Wd)
            Pd = torch.from_numpy(P).to(dev)
            Pq = L.nf4_quantize(Pd)
            if keep_full_precision and (out, inp) not in self.full_precision:
                self.full_precision[(out, inp)] = (Wd, Pd)  # one fp32 W and P per distinct shape, for the extras
            del Wd, Pd
            self.layers.append(dict(
                name=name, out=out, inp=inp, Wq=Wq, Pq=Pq, Wq_out=L.NF4Tensor.empty(out, inp),
                B=randn_bf16(r, inp, 1e-3), x=randn_bf16(T, inp, 1.0), dy=randn_bf16(T, out, 1e-2),
                y=torch.empty((T, pitch8(out)), dtype=torch.bfloat16, device=dev)[:, :out],
                dx=torch.empty((T, pitch8(inp)), dtype=torch.bfloat16, device=dev)[:, :inp],
                dB=torch.empty((r, inp), dtype=torch.float32, device=dev)))
            ws_bytes = max(ws_bytes, L.loqt_workspace_bytes(L.OP_BWD, T, out, inp, r),
                           L.loqt_workspace_bytes(L.OP_FWD, T, out, inp, r),
                           L.loqt_workspace_bytes(L.OP_MERGE, T, out, inp, r))
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.w_eff_bytes = sum(l["out"] * pitch8(l["inp"]) * 2 for l in self.layers)
        self.descs = L.make_merge_descs([(l["Wq"], l["Wq_out"], l["Pq"], l["B"], 1.0) for l in self.layers])
        self._saved_ready = False
        torch.cuda.synchronize()

    def _ensure_saved(self):
        if not self._saved_ready:  # the transient bf16 weight of the saved mode: out x in per layer
            for l in self.layers:
                l["w_eff"] = self.torch.empty((l["out"], (l["inp"] + 7) // 8 * 8), dtype=self.torch.bfloat16,
                                              device="cuda")[:, :l["inp"]]
            self._saved_ready = True

    def fwd_bwd(self, mode):
        L, ws = self.L, self.ws
        if mode == "saved":
            self._ensure_saved()
            for l in self.layers:
                L.loqt_linear_fwd_save(l["x"], l["Wq"], l["Pq"], l["B"], 1.0, l["y"], l["w_eff"], ws)
            for l in reversed(self.layers):
                L.loqt_linear_bwd_saved(l["dy"], l["x"], l["Pq"], 1.0, l["w_eff"], l["dx"], l["dB"], False, ws)
        else:
            for l in self.layers:
                L.loqt_linear_fwd(l["x"], l["Wq"], l["Pq"], l["B"], 1.0, l["y"], ws)
                L.loqt_linear_bwd(l["dy"], l["x"], l["Wq"], l["Pq"], l["B"], 1.0, l["dx"], l["dB"], False, ws)

    def merge(self):
        self.L.loqt_merge_requant_batched(self.descs, self.ws)

    def timed(self, mode, steps, warmup, with_merge=True):
        """(wall ms per step, fwd+bwd ms per step, merge ms per step) over `steps` steps after `warmup` untimed ones;
        three events per step, nothing else, inside the timed region."""
        torch = self.torch
        ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
        for _ in range(warmup):
            self.fwd_bwd(mode)
            if with_merge:
                self.merge()
        torch.cuda.synchronize()
        events = []
        t0 = time.perf_counter()
        for _ in range(steps):
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
            self.fwd_bwd(mode)
            e1.record()
            if with_merge:
                self.merge()
            e2.record()
            events.append((e0, e1, e2))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return ((t1 - t0) * 1e3 / steps, sum(a.elapsed_time(b) for (a, b, _) in events) / steps,
                sum(b.elapsed_time(c) for (_, b, c) in events) / steps)


def flop_counts(synth, L, wl, mode):
    """Algorithmic flops (the metric's model) and the flops the chosen implementation executes, per step."""
    T, r = wl.T, wl.r
    f_fb = sum(synth.flops_fwd(T, o, i, r) + synth.flops_bwd(T, o, i, r) for (_, o, i) in wl.projections)
    saved = mode == "saved"
    # the forward and the backward call choose separately (the backward one has Z at hand anyway)
    folded = {n: saved or L.resolved_path(L.OP_FWD, T, o, i) == L.PATH_FOLDED for (n, o, i) in wl.projections}
    folded_b = {n: saved or L.resolved_path(L.OP_BWD, T, o, i) == L.PATH_FOLDED for (n, o, i) in wl.projections}
    k = {
        "gemm_u": sum(2 * T * i * r for (n, o, i) in wl.projections if not folded[n]),
        "gemm_y": sum(2 * T * o * (i + (0 if folded[n] else r)) for (n, o, i) in wl.projections),
        # folded: Z may ride along with dx ([dx | Z] = dy [W_eff | s deq(P)]); its flops are then in gemm_dx
        "gemm_z+dx": sum(2 * T * o * (i + r) if folded_b[n] else 2 * T * (o * r + i * (o + r))
                         for (n, o, i) in wl.projections),
        "gemm_db": sum(2 * T * r * i for (n, o, i) in wl.projections),
        "fold_weight": sum(2 * o * i * r * ((1 if folded[n] else 0) + (1 if folded_b[n] and not saved else 0))
                           for (n, o, i) in wl.projections),
    }
    return f_fb, k, folded


def extras(L, synth, torch, bench, steps, warmup):
    """Supplementary timings outside the K timed steps (not part of `value`).  Streams that are meant as HBM figures
    rotate over enough distinct buffer sets (> 512 MB in all) that nothing is served by the 256 MB Infinity Cache."""
    dev = "cuda"
    wl = bench.wl

    def timed_us(fn, reps=10, warm=2):
        for i in range(warm):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    res = {"codec": [], "absmax_dq": [], "merge_small_rank": [], "init_compensate": []}
    for (out, inp), (Wd, Pd) in bench.full_precision.items():
        n = out * inp
        # distinct buffer sets: the fp32 source alone is 4 B per weight
        nsets = max(4, -(-(640 << 20) // (n * 4)))
        Ws = [Wd] + [torch.empty_like(Wd).normal_(0.0, 0.02, generator=gen) for _ in range(nsets - 1)]
        Wqs = [L.nf4_quantize(w) for w in Ws]
        Wbs = [torch.empty((out, (inp + 7) // 8 * 8), dtype=torch.bfloat16, device=dev)[:, :inp] for _ in range(nsets)]
        t_q = timed_us(lambda i: L.nf4_quantize(Ws[i % nsets], out=Wqs[i % nsets]), reps=2 * nsets)
        t_d = timed_us(lambda i: L.nf4_dequantize(Wqs[i % nsets], Wbs[i % nsets]), reps=2 * nsets)
        res["codec"].append({"shape": f"{out}x{inp}", "buffer_sets": nsets, "rotated_MB": nsets * n * 4 / 1e6,
                             "quantize_us": t_q, "quantize_GBs": n * 4.5625 / t_q / 1e3,
                             "quantize_frac_hbm": n * 4.5625 / t_q / 1e3 / PEAK_HBM_GBS,
                             "dequantize_bf16_us": t_d, "dequantize_bf16_GBs": n * 2.5625 / t_d / 1e3,
                             "dequantize_frac_hbm": n * 2.5625 / t_d / 1e3 / PEAK_HBM_GBS})
        del Ws, Wbs
        Wq = Wqs[0]
        # double-quantised block scales (sec. 2.4): three launches over n / 64 scales (launch-sized), the storage
        # they buy, and what the 8-bit scales do to the dequantised weight
        a = Wq.absmax.reshape(-1)
        dq = L.loqt_absmax_dq_compress(a)
        a2 = L.loqt_absmax_dq_expand(*dq)
        t_c = timed_us(lambda i: L.loqt_absmax_dq_compress(a))
        t_e = timed_us(lambda i: L.loqt_absmax_dq_expand(*dq, out=a2))
        res["absmax_dq"].append({"shape": f"{out}x{inp}", "scales": a.numel(), "compress_us": t_c, "expand_us": t_e,
                                 "bytes_per_weight": 0.5 + (a.numel() + 4 * dq[1].numel() + 4) / n,
                                 "bytes_per_weight_fp32_scales": 0.5 + 4 * a.numel() / n,
                                 "rms_rel_change_of_scales": float(((a2 - a).double().pow(2).mean().sqrt()
                                                                   / a.double().pow(2).mean().sqrt()).item())})
        # merge at the ranks where the rank-r product no longer binds (the paper's fine-tuning ranks), in place,
        # rotating over the NF4 sets above (codes + scales: 0.5625 B per weight and set) -- cache-assisted unless the
        # sets exceed the Infinity Cache, which `rotated_MB` tells; the 13B sweep below is the HBM figure of record
        for r in (64, 128):
            Pq = L.nf4_quantize(Pd[:, :r].contiguous())
            B = (torch.randn((r, inp), device=dev, generator=gen) * 1e-3).to(torch.bfloat16)
            ws = L.workspace(L.OP_MERGE, 0, out, inp, r)
            t = timed_us(lambda i: L.loqt_merge_requant(Wqs[i % nsets], Pq, B, 1.0, ws=ws), reps=2 * nsets)
            byts, fl = synth.bytes_merge(out, inp, r), synth.flops_merge(out, inp, r)
            res["merge_small_rank"].append({"shape": f"{out}x{inp}", "rank": r, "us": t,
                                            "rotated_MB": nsets * n * 0.5625 / 1e6,
                                            "algorithmic_GBs": byts / t / 1e3,
                                            "frac_of_hbm_peak": byts / t / 1e3 / PEAK_HBM_GBS,
                                            "tflops": fl / t / 1e6})
        # Alg. 2 loop, five steps from B = 0: step c costs two rank-r products of 2 out in r flop (the first
        # step has no W - s P B product) and streams W (4 B), Q_c (0.5625 B) and the residual (2 + 2 B) per element
        r, iters = wl.r, 5
        B = torch.empty((r, (inp + 7) // 8 * 8), dtype=torch.bfloat16, device=dev)[:, :inp]
        ws = L.workspace(L.OP_INIT, 0, out, inp, r)
        Wq_out = L.NF4Tensor.empty(out, inp)
        t = timed_us(lambda i: L.loqt_init_compensate(Wd, Pd, 1.0, iters, B, out=Wq_out, ws=ws), reps=3, warm=1)
        fl = (2 * iters - 1) * 2.0 * out * inp * r
        res["init_compensate"].append({"shape": f"{out}x{inp}", "rank": r, "iters": iters, "us": t,
                                       "tflops": fl / t / 1e6, "frac_of_bf16_peak": fl / t / 1e6 / PEAK_BF16_TFLOPS})
        del Wqs, Wq, Wq_out
    torch.cuda.empty_cache()

    # forward + backward of the other workloads, both modes (same calls, same flop model)
    res["fwd_bwd_other_workloads"] = []
    for name in ("60m_layer", "130m_block", "1b_block", "13b_block"):
        if name == wl.name:
            continue
        w = synth.WORKLOADS[name]
        b = BlockBench(L, synth, torch, w, seed=0)
        row = {"workload": name, "tokens": w.T, "rank": w.r}
        for mode in ("plain", "saved"):
            _, ms_fb, _ = b.timed(mode, steps, warmup, with_merge=False)
            f_fb, kfl, folded = flop_counts(synth, L, w, mode)
            f_exec = sum(kfl.values())
            row[mode] = {"ms": ms_fb, "tflops": f_fb / ms_fb / 1e9, "frac_of_bf16_peak": f_fb / ms_fb / 1e9 / PEAK_BF16_TFLOPS,
                         "executed_tflops": f_exec / ms_fb / 1e9,
                         "frac_of_bf16_peak_executed": f_exec / ms_fb / 1e9 / PEAK_BF16_TFLOPS}
        _, _, ms_mg = b.timed("plain", max(2, steps // 2), 1, with_merge=True)
        f_mg = sum(synth.flops_merge(o, i, w.r) for (_, o, i) in w.projections)
        b_mg = sum(synth.bytes_merge(o, i, w.r) for (_, o, i) in w.projections)
        t_hbm, t_mfma = b_mg / (PEAK_HBM_GBS * 1e9) * 1e3, f_mg / (PEAK_BF16_TFLOPS * 1e12) * 1e3
        row["merge_block"] = {"ms": ms_mg, "algorithmic_GBs": b_mg / ms_mg / 1e6,
                              "frac_of_binding_roof": max(t_hbm, t_mfma) / ms_mg}
        row["saved_mode_extra_bytes"] = b.w_eff_bytes
        res["fwd_bwd_other_workloads"].append(row)
        del b
        torch.cuda.empty_cache()

    # Merge sweep over a whole 13B model (40 blocks x 7 projections, 280 distinct NF4 weights = 7.1 GB
    # resident, far beyond the 256 MB Infinity Cache): the streaming figure of record for the merge, at the
    # workload's rank (the rank-r product binds) and at rank 64 (it does not)
    w13 = synth.WORKLOADS["13b_block"]
    Wqs13 = []
    for _ in range(w13.n_blocks):
        for (name, out, inp) in w13.projections:
            W = torch.empty((out, inp), device=dev, dtype=torch.float32).normal_(0.0, 0.02, generator=gen)
            Wqs13.append(L.nf4_quantize(W))
            del W
    res["merge_sweep_13b"] = []
    for r in (w13.r, 64):
        shapes = {}
        for (name, out, inp) in w13.projections:
            if (out, inp) not in shapes:
                Pq = L.nf4_quantize(torch.randn((out, r), device=dev, generator=gen) / out ** 0.5)
                B = (torch.randn((r, inp), device=dev, generator=gen) * 1e-3).to(torch.bfloat16)
                shapes[(out, inp)] = (Pq, B)
        sweep = [(Wq, None, *shapes[(Wq.rows, Wq.cols)], 1.0) for Wq in Wqs13]  # in place
        descs = L.make_merge_descs(sweep)
        ws = torch.empty(L.merge_descs_workspace_bytes(descs), dtype=torch.uint8, device=dev)
        t = timed_us(lambda i: L.loqt_merge_requant_batched(descs, ws), reps=2, warm=1)
        byts = w13.n_blocks * sum(synth.bytes_merge(o, i, r) for (_, o, i) in w13.projections)
        fl = w13.n_blocks * sum(synth.flops_merge(o, i, r) for (_, o, i) in w13.projections)
        t_hbm, t_mfma = byts / (PEAK_HBM_GBS * 1e9) * 1e6, fl / (PEAK_BF16_TFLOPS * 1e12) * 1e6
        res["merge_sweep_13b"].append({"layers": len(sweep), "rank": r, "resident_GB": len(sweep) and sum(
            q.codes.numel() + 4 * q.absmax.numel() for q in Wqs13) / 1e9, "ms": t / 1e3,
            "algorithmic_GBs": byts / t / 1e3, "frac_of_hbm_peak": t_hbm / t, "tflops": fl / t / 1e6,
            "binding_roof": "mfma" if t_mfma > t_hbm else "hbm", "frac_of_binding_roof": max(t_hbm, t_mfma) / t})
        del descs, sweep, shapes
    del Wqs13
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (got --gpus {args.gpus}); "
              "there is no multi-GPU path to time.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2405_16528_amd import binding as L
    from paper_2405_16528_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    T, r = wl.T, wl.r
    bench = BlockBench(L, synth, torch, wl, args.seed, keep_full_precision=not args.no_extras)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    mode = args.mode
    other = "saved" if mode == "plain" else "plain"
    # the timed region: K steps of the headline mode
    ms_step, ms_fb, ms_mg = bench.timed(mode, args.steps, args.warmup)
    # a second pass of K steps with the library's per-launch HIP events on the launch stream (the kernel
    # breakdown and the roofline object come from here; the event pairs cost a few per cent of the step, so they
    # stay out of the region `value` is measured on)
    L.timing_enable(True)
    t2 = time.perf_counter()
    for _ in range(args.steps):
        bench.fwd_bwd(mode)
        bench.merge()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    L.timing_enable(False)
    kt = L.timing_read()
    ms_step_instrumented = (t3 - t2) * 1e3 / args.steps
    # the other mode, timed the same way as the headline (reported beside it, not part of `value`)
    o_step, o_fb, _ = bench.timed(other, args.steps, args.warmup)

    f_fb, kflops, folded = flop_counts(synth, L, wl, mode)
    f_fb_o, kflops_o, _ = flop_counts(synth, L, wl, other)
    f_mg = sum(synth.flops_merge(o, i, r) for (_, o, i) in wl.projections)
    b_mg = sum(synth.bytes_merge(o, i, r) for (_, o, i) in wl.projections)
    kflops["merge_requant"] = f_mg
    f_exec = sum(v for k, v in kflops.items() if k != "merge_requant")
    f_exec_o = sum(kflops_o.values())

    kernels = {}
    if "gemm_z" in kt or "gemm_dx" in kt:
        nz, mz = kt.pop("gemm_z", (0, 0.0))
        nd, md = kt.pop("gemm_dx", (0, 0.0))
        kt["gemm_z+dx"] = (nz + nd, mz + md)
    for name, (n, ms) in kt.items():
        if n == 0:
            continue
        ent = {"launches_per_step": n / args.steps, "ms_per_step": ms / args.steps, "avg_ms": ms / n}
        if name in kflops and kflops[name]:
            ent["tflops"] = kflops[name] * args.steps / (ms * 1e-3) / 1e12
        kernels[name] = ent

    def roof(slot, label):
        if slot not in kernels or "tflops" not in kernels[slot]:
            return None
        k = kernels[slot]
        return {"kernel": label, "bound": "mfma", "achieved": k["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": k["tflops"] / PEAK_BF16_TFLOPS,
                "flops_per_launch": kflops[slot] / k["launches_per_step"], "avg_launch_ms": k["avg_ms"]}

    # dominant kernel: the 256x256 bf16-epilogue product with both operands K-contiguous, i.e. the gemm_y launches
    roofline = roof("gemm_y", "nt_gemm_kernel<256,256,EPI_BF16,false,false> (the gemm_y launches: y = x W_eff^T; for "
                              "11008 output columns the last 768 run as a 256x128-tile launch inside the same timed slot)")
    if roofline is not None:
        # HBM-side bytes per launch slot (FETCH_SIZE + WRITE_SIZE, rocprofv3 --pmc, scaled by a plain copy), read from
        # the committed summary of those counter runs; not measurable from inside this process
        roofline["traffic"] = traffic_from_profile(wl.name)
    roofline_dx = roof("gemm_z+dx", "nt_gemm_kernel<256,256,EPI_BF16,false,true> (dx = dy W_eff, B operand stored K x "
                                    "rows; the slot also holds the stand-alone Z = s dy deq(P) launches on 128x128 tiles)")

    # the merge is bound by max(HBM stream, rank-r bf16 product); report both views.  Time: the whole
    # loqt_merge_requant_batched call of the timed region, not the kernel slot alone
    t_hbm = b_mg / (PEAK_HBM_GBS * 1e9) * 1e3
    t_mfma = f_mg / (PEAK_BF16_TFLOPS * 1e12) * 1e3
    merge = {"ms_per_step": ms_mg, "algorithmic_GBs": b_mg / (ms_mg * 1e-3) / 1e9,
             "tflops": f_mg / (ms_mg * 1e-3) / 1e12, "t_hbm_ms": t_hbm, "t_mfma_ms": t_mfma,
             "binding_roof": "mfma" if t_mfma > t_hbm else "hbm",
             "frac_of_binding_roof": max(t_hbm, t_mfma) / ms_mg, "frac_of_hbm_peak": t_hbm / ms_mg}

    def fb_entry(ms, f_alg, f_ex):
        return {"ms_per_step": ms, "tflops": f_alg / (ms * 1e-3) / 1e12,
                "frac_of_bf16_peak": f_alg / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                "executed_tflops": f_ex / (ms * 1e-3) / 1e12,
                "frac_of_bf16_peak_executed": f_ex / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}

    step_text = {
        "plain": "7x(loqt_linear_fwd + loqt_linear_bwd), nothing kept between the two calls, + batched merge/requant "
                 "of the block",
        "saved": "loqt_linear_fwd_save of the 7 projections, loqt_linear_bwd_saved of the 7 in reverse order (W_eff "
                 "bf16 kept per layer in between: %.2f GB for this block), + batched merge/requant of the block"
                 % (bench.w_eff_bytes / 1e9)}
    out = {
        "metric": METRIC,
        "value": (f_fb + f_mg) / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "tokens": T, "rank": r,
                   "projections": [f"{n}:{o}x{i}" for (n, o, i) in wl.projections],
                   "mode": mode, "step": step_text[mode]},
        "fwd_bwd": dict(fb_entry(ms_fb, f_fb, f_exec),
                        flop_model="tflops / frac_of_bf16_peak: the metric's algorithmic model, factored form: fwd "
                                   "2T(out*in + in*r + r*out), bwd 2T(out*in + out*r + 2*r*in).  executed_*: the flops "
                                   "the chosen implementation runs (folded: 2*out*in*r per fold instead of the "
                                   "rank-r products through every token)",
                        paths=["folded"] if mode == "saved" else
                        {"fwd": sorted({["auto", "fused", "prepass", "folded"][L.resolved_path(L.OP_FWD, T, o, i)]
                                        for (_, o, i) in wl.projections}),
                         "bwd": sorted({["auto", "fused", "prepass", "folded"][L.resolved_path(L.OP_BWD, T, o, i)]
                                        for (_, o, i) in wl.projections})}),
        "merge": merge,
        "other_mode": dict(fb_entry(o_fb, f_fb_o, f_exec_o), mode=other, step=step_text[other],
                           ms_per_whole_step=o_step, value=(f_fb + f_mg) / (o_step * 1e-3) / 1e12,
                           extra_bytes_kept_per_block=bench.w_eff_bytes if other == "saved" else 0),
        "kernels": kernels,
        "kernels_pass": {"steps": args.steps, "ms_per_step": ms_step_instrumented,
                         "note": "per-kernel figures and the roofline objects: a second pass of the same K steps "
                                 "with a HIP event pair around every launch"},
        "roofline": roofline,
        "roofline_dx": roofline_dx,
    }
    if not args.no_extras:
        out["extras"] = extras(L, synth, torch, bench, max(3, args.steps // 2), 2)
        # the same step captured once as a HIP graph and replayed (the library allocates nothing and keeps no
        # state, so the capture holds only its kernels): what the gaps between the launches of a step cost
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            bench.fwd_bwd(mode)
            bench.merge()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            bench.fwd_bwd(mode)
            bench.merge()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t6 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t7 = time.perf_counter()
        out["extras"]["graph_replay"] = {"mode": mode, "ms_per_step": (t7 - t6) * 1e3 / args.steps,
                                         "value": (f_fb + f_mg) / ((t7 - t6) / args.steps) / 1e12}
    if not args.no_cpu_baseline:
        del bench
        torch.cuda.empty_cache()
        out["cpu_baseline"], out["parity"] = oracle_leg(L, torch, synth, args.seed, min(args.cpu_sample_tokens, T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
