#!/usr/bin/env python3
"""Benchmark of the Quaff quantized-linear hot path on one MI355X.

A "step" is one pass of the whole path - scale update, scale+quantize, INT8 forward with fused dequant+LoRA
epilogue, and the dX backward - over every projection of the workload for one synthetic batch, with all inputs
already resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0   # MI355X dense INT8 MFMA peak, TOP/s
HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload (BASELINE.json configs, 1-based)")
    ap.add_argument("--batches", type=int, default=4, help="distinct input batches rotated through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-calls", action="store_true",
                    help="forward as scale_update + quant_act + linear_fwd instead of the one-call forward step")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path is built and measured on ONE GPU only (no collectives, no sharding); "
                 "run with --gpus 1")

    import numpy as np
    import torch
    from paper_2505_14742_amd import binding as q
    from paper_2505_14742_amd import synth
    q.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    i8, f32 = torch.int8, torch.float32

    projs = synth.CONFIGS[args.config]
    if args.config in (4, 5):   # distinct shapes only, to bound set-up time
        seen, keep = set(), []
        for p in projs:
            if (p.c_in, p.c_out) not in seen:
                seen.add((p.c_in, p.c_out))
                keep.append(p)
        projs = keep

    def bf16_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev)

    layers = []
    for p in projs:
        W, O = synth.weight(p), synth.outlier_indices(p)
        A, B = synth.lora(p)
        n, r = int(O.size), p.lora_rank
        n_pad = q.padded_outliers(n)
        L = dict(p=p, n=n, r=r, n_pad=n_pad)
        L["O"] = torch.from_numpy(O).to(dev) if n else None
        L["A"] = bf16_dev(A) if r else None
        L["B"] = bf16_dev(B) if r else None
        Wd = torch.from_numpy(W).to(dev)
        L["Wq"] = torch.empty(q.packed_weight_bytes(p.c_in, p.c_out), dtype=i8, device=dev)
        L["dw"] = torch.empty(p.c_out, dtype=f32, device=dev)
        L["W_O"] = torch.empty((max(n, 1), p.c_out), dtype=f32, device=dev)
        L["wmax"] = torch.empty(max(n, 1), dtype=f32, device=dev)
        ws = torch.empty(q.prepare_workspace_bytes(p.c_in, p.c_out), dtype=i8, device=dev)
        q.prepare_weight(Wd, L["O"], L["Wq"], L["dw"], L["W_O"] if n else None, L["wmax"] if n else None, None, ws)
        del Wd, ws
        L["s"] = torch.ones(max(n, 1), dtype=f32, device=dev)
        L["cs"] = torch.ones(p.c_in, dtype=f32, device=dev)
        L["what"] = torch.zeros((p.c_out, max(n_pad, 1)), dtype=i8, device=dev)
        L["dwh"] = torch.zeros(p.c_out, dtype=f32, device=dev)
        L["ws"] = torch.empty(max(q.workspace_bytes(p.t, p.c_in, p.c_out, n, r),
                                  q.fwd_step_workspace_bytes(p.t, p.c_in, p.c_out, n, r)), dtype=i8, device=dev)
        L["X"] = [bf16_dev(synth.activations(p, s)) for s in range(args.batches)]
        L["dY"] = [bf16_dev(synth.out_grad(p, s)) for s in range(args.batches)] if p.backward else None
        L["Xq"] = torch.empty((p.t, p.c_in), dtype=i8, device=dev)
        L["dx"] = torch.empty(p.t, dtype=f32, device=dev)
        L["xo"] = torch.zeros((p.t, max(n_pad, 1)), dtype=i8, device=dev)
        L["Y"] = [torch.empty((p.t, p.c_out), dtype=f32, device=dev) for _ in range(args.batches)]
        L["dX"] = [torch.empty((p.t, p.c_in), dtype=f32, device=dev) for _ in range(args.batches)]
        L["fwd_ops"] = 2.0 * p.t * p.c_out * (p.c_in + n)
        L["bwd_ops"] = 2.0 * p.t * p.c_out * p.c_in if p.backward else 0.0
        layers.append(L)

    def step(i, separate=None):
        separate = args.separate_calls if separate is None else separate
        b = i % args.batches
        for L in layers:
            p, n, r = L["p"], L["n"], L["r"]
            X = L["X"][b]
            if separate:
                q.scale_update(X, L["O"], L["W_O"], L["wmax"], p.c_out, p.gamma, L["s"], L["cs"], L["what"], L["dwh"],
                               None, L["ws"])
                q.quant_act(X, L["cs"], L["O"], L["Xq"], L["dx"], L["xo"] if n else None)
                q.linear_fwd(L["Xq"], L["dx"], L["xo"] if n else None, L["Wq"], L["dw"], p.c_in, p.c_out,
                             L["what"] if n else None, L["dwh"] if n else None, n, X if r else None, L["A"], L["B"], r,
                             p.lora_scale, L["Y"][b], L["ws"])
            else:
                q.linear_fwd_step(X, L["O"], L["W_O"] if n else None, L["wmax"] if n else None, p.c_out, p.gamma,
                                  L["s"], L["cs"], L["what"], L["dwh"], None, L["Xq"], L["dx"], L["xo"] if n else None,
                                  L["Wq"], L["dw"], L["A"], L["B"], r, p.lora_scale, L["Y"][b], L["ws"])
            if p.backward:
                q.linear_bwd_dx(L["dY"][b], L["Wq"], L["dw"], p.c_in, p.c_out, L["A"], L["B"], r, p.lora_scale,
                                L["dX"][b], L["ws"])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = max(e0.elapsed_time(e1), 0.0) / args.steps
    ms_per_step = max(ms_per_step, 0.0)
    total_ops = sum(L["fwd_ops"] + L["bwd_ops"] for L in layers)
    tops = total_ops / (ms_per_step * 1e-3) / 1e12

    # "warm" variant for comparison: the same batch every step (inputs and outputs may stay in the Infinity Cache);
    # the headline figures above are the rotated ("cold") ones
    e0.record()
    for i in range(args.steps):
        step(0)
    e1.record()
    torch.cuda.synchronize()
    warm_ms_per_step = e0.elapsed_time(e1) / args.steps

    # ---- per-kernel durations with HIP events on the launch stream (separate pass: the events perturb the step)
    q.profile_enable(True)
    prof_steps = min(args.steps, 20)
    for i in range(prof_steps):
        step(i)
    torch.cuda.synchronize()
    launches = q.profile_launches()
    q.profile_enable(False)
    per_step = len(launches) // prof_steps
    kinds = {}
    for name, ms in launches:
        k = kinds.setdefault(name, [0.0, 0])
        k[0] += ms
        k[1] += 1
    gemm_ms = [ms for name, ms in launches if name == "gemm_i8"]
    gemm_ops = sum(L["fwd_ops"] + L["bwd_ops"] for L in layers) * prof_steps
    gemm_total_ms = sum(gemm_ms)
    gemm_tops = gemm_ops / (gemm_total_ms * 1e-3) / 1e12
    # per-shape GEMM figures, launches come in call order: for each layer fwd then bwd
    seq = [(name, ms) for name, ms in launches]
    shape_stats = {}
    gi = 0
    order = []
    for L in layers:
        order.append((L["p"].name + ".fwd", L["fwd_ops"]))
        if L["p"].backward:
            order.append((L["p"].name + ".bwd_dx", L["bwd_ops"]))
    for idx, ms in enumerate(gemm_ms):
        nm, ops = order[idx % len(order)]
        st = shape_stats.setdefault(nm, [0.0, 0, ops])
        st[0] += ms
        st[1] += 1
    gemm_shapes = {nm: {"avg_us": round(st[0] / st[1] * 1e3, 2), "tops": round(st[2] / (st[0] / st[1] * 1e-3) / 1e12, 1),
                        "frac_peak": round(st[2] / (st[0] / st[1] * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)}
                   for nm, st in shape_stats.items()}
    # HBM traffic of the GEMM launches: operands once, output once (algorithmic), against the PMC figure recorded
    # for this workload (counters cannot be read from inside the process)
    gemm_bytes = 0.0
    for L in layers:
        p = L["p"]
        gemm_bytes += p.t * p.c_in + p.c_in * p.c_out + (p.t + p.c_out) * L["n_pad"] + 4.0 * p.t * p.c_out
        if p.backward:
            gemm_bytes += p.t * p.c_out + p.c_in * p.c_out + 4.0 * p.t * p.c_in
    gemm_traffic = None
    prof_file = os.path.join(ROOT, "profiles", "gemm_i8_hbm_traffic_phi3_attention.md")
    if args.config == 2 and os.path.exists(prof_file):
        for ln in open(prof_file):
            if ln.strip().startswith("gemm_traffic_bytes_per_launch"):
                gemm_traffic = int(ln.split("=")[1])
    def kernel_stats(kinds, launches, prof_steps):
        # HBM-bound kernels: algorithmic bytes / measured time
        # forward quantizer: 2 B read + 1 B written per element; backward: one launch quantizes dY and forms dY B^T
        quant_bytes = fused_bytes = lora_bytes = 0.0
        for L in layers:
            p, r = L["p"], L["r"]
            quant_bytes += 3.0 * p.t * p.c_in + 4.0 * p.t + p.t * L["n_pad"]
            if r:
                lora_bytes += 2.0 * p.t * p.c_in + 2.0 * p.c_in * r + 8.0 * p.t * r + 4.0 * p.c_out * r
            if p.backward:
                fused_bytes += 3.0 * p.t * p.c_out + 4.0 * p.t + (2.0 * p.c_out * r + 8.0 * p.t * r if r else 0.0)
        kernels = {name: {"avg_us": round(v[0] / v[1] * 1e3, 2), "launches_per_step": v[1] // prof_steps,
                          "us_per_step": round(v[0] / prof_steps * 1e3, 2)} for name, v in kinds.items()}

        def hbm(name, nbytes):
            if name in kernels and nbytes:
                ms = kinds[name][0] / prof_steps
                kernels[name]["achieved_GBs"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
                kernels[name]["frac_hbm_peak"] = round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        if "quant_rows+lora_down" in kernels:
            hbm("quant_rows", quant_bytes)
            hbm("quant_rows+lora_down", fused_bytes)
            hbm("lora_down", lora_bytes)
            hbm("colmax_outlier+lora_down", lora_bytes)   # the abs-max gather adds about a third of X's bytes
            what_bytes = sum(4.0 * L["n"] * L["p"].c_out + L["n_pad"] * L["p"].c_out + 4.0 * L["p"].c_out for L in layers)
            hbm("momentum_what+quant_rows", quant_bytes + what_bytes)
        else:   # rank 0 or shapes the combined launch does not cover: separate launches in the backward pass too
            hbm("quant_rows", quant_bytes + fused_bytes)
            hbm("lora_down", lora_bytes)
        # column abs-max: useful bytes are the 2-byte outlier entries; what the memory system must fetch is one
        # 64-byte segment per (row, distinct segment touched by O) - counted here from the outlier positions
        for col_kind in ("colmax_outlier",):
            if col_kind not in kernels:
                continue
            useful = fetched = 0.0
            for L in layers:
                if L["n"]:
                    seg = len(set(int(o) // 32 for o in L["O"].cpu().tolist()))
                    useful += 2.0 * L["p"].t * L["n"]
                    # the library streams whole rows when the outliers touch most segments anyway (n * 64 >= c_in)
                    fetched += 2.0 * L["p"].t * L["p"].c_in if L["n"] * 64 >= L["p"].c_in else 64.0 * L["p"].t * seg
            col_ms = kinds["colmax_outlier"][0] / prof_steps
            kernels["colmax_outlier"]["useful_GBs"] = round(useful / (col_ms * 1e-3) / 1e9, 1)
            kernels["colmax_outlier"]["fetched_GBs"] = round(fetched / (col_ms * 1e-3) / 1e9, 1)
            kernels["colmax_outlier"]["frac_hbm_peak_fetched"] = round(fetched / (col_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        for name, v in kinds.items():
            ds = sorted(ms for nm, ms in launches if nm == name)
            kernels[name]["min_us"] = round(ds[0] * 1e3, 2)
            kernels[name]["median_us"] = round(ds[len(ds) // 2] * 1e3, 2)
        return kernels

    kernels = kernel_stats(kinds, launches, prof_steps)
    kernels_separate = None
    if not args.separate_calls:
        # the same step through the four separate calls, for the stand-alone figures of the abs-max, momentum,
        # quantizer and down-projection kernels
        for i in range(3):              # untimed: the first launch of a kernel pays for loading its code
            step(i, separate=True)
        torch.cuda.synchronize()
        q.profile_enable(True)
        sep_steps = min(args.steps, 10)
        for i in range(sep_steps):
            step(i, separate=True)
        torch.cuda.synchronize()
        sep_launches = q.profile_launches()
        q.profile_enable(False)
        sep_kinds = {}
        for name, ms in sep_launches:
            k = sep_kinds.setdefault(name, [0.0, 0])
            k[0] += ms
            k[1] += 1
        kernels_separate = kernel_stats(sep_kinds, sep_launches, sep_steps)
        kernels_separate.pop("gemm_i8", None)

    out = {
        "metric": "INT8 quantized-linear TOPS fwd+bwd_dx at Phi-3 shapes; % INT8 MFMA peak",
        "value": round(tops, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "configs[%d]: %s" % (args.config - 1, ", ".join(
            "%s t=%d %d->%d |O|=%d r=%d" % (L["p"].name, L["p"].t, L["p"].c_in, L["p"].c_out, L["n"], L["r"])
            for L in layers)), "batches_rotated": args.batches, "calls_per_step":
            ("scale_update, quant_act, linear_fwd, linear_bwd_dx per projection" if args.separate_calls else
             "linear_fwd_step (= scale_update + quant_act + linear_fwd), linear_bwd_dx per projection")},
        "frac_int8_peak_whole_step": round(tops / INT8_PEAK_TOPS, 4),
        "wall_ms_per_step": round(wall_ms / args.steps, 5),
        "warm_same_batch_ms_per_step": round(warm_ms_per_step, 5),
        "roofline": {"bound": "mfma", "kernel": "gemm_i8 (all launches of the step)", "achieved": round(gemm_tops, 2),
                     "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": round(gemm_tops / INT8_PEAK_TOPS, 4),
                     "traffic": gemm_traffic, "traffic_unit": "bytes per GEMM launch (rocprofv3 FETCH_SIZE + "
                     "WRITE_SIZE, scaled by the copy kernel; profiles/gemm_i8_hbm_traffic_phi3_attention.md)",
                     "algorithmic_bytes_per_launch": round(gemm_bytes / len(order)), "per_shape": gemm_shapes,
                     "note": "priced against the INT8 MFMA peak as a contraction; the 128x192-tile launches (2048 x 3072 "
                             "outputs: one tile per compute unit) are held back by operand delivery from L2 into LDS, "
                             "the 256x288-tile launch by the power-limited MFMA clock (measured_ceilings)"},
        "kernels": kernels,
        "kernels_with_separate_calls": kernels_separate,
    }

    # ---- rows beyond the headline metric, timed on their own (not part of `value`)
    extra = {}
    if all(L["r"] for L in layers) and all(L["p"].backward for L in layers):
        for L in layers:
            p, r = L["p"], L["r"]
            L["dA"] = torch.empty((p.c_in, r), dtype=f32, device=dev)
            L["dB"] = torch.empty((r, p.c_out), dtype=f32, device=dev)
            L["gws"] = torch.empty(q.lora_bwd_workspace_bytes(p.t, p.c_in, p.c_out, r), dtype=i8, device=dev)

        def grads(i):
            b = i % args.batches
            for L in layers:
                q.lora_bwd_weights(L["X"][b], L["dY"][b], L["A"], L["B"], L["r"], L["p"].lora_scale, L["dA"], L["dB"],
                                   L["gws"])
        for i in range(3):
            grads(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            grads(i)
        e1.record()
        torch.cuda.synchronize()
        g_ms = e0.elapsed_time(e1) / args.steps
        g_bytes = sum(2.0 * L["p"].t * (L["p"].c_in + L["p"].c_out) for L in layers)
        extra["lora_weight_grads"] = {
            "ms_per_step": round(g_ms, 5), "calls_per_step": "quaff_lora_bwd_weights per projection (dA, dB)",
            "algorithmic_GBs": round(g_bytes / (g_ms * 1e-3) / 1e9, 1),
            "frac_hbm_peak": round(g_bytes / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "algorithmic_bytes": "X and dY read once (2 t (c_in + c_out)); the implementation reads each twice"}
        # the whole fine-tuning step of the layers: one forward call and one backward call (dX, dA, dB) per projection
        for L in layers:
            p = L["p"]
            L["bws"] = torch.empty(q.bwd_step_workspace_bytes(p.t, p.c_in, p.c_out, L["r"]), dtype=i8, device=dev)

        def two_call_step(i):
            b = i % args.batches
            for L in layers:
                p, n, r = L["p"], L["n"], L["r"]
                q.linear_fwd_step(L["X"][b], L["O"], L["W_O"] if n else None, L["wmax"] if n else None, p.c_out,
                                  p.gamma, L["s"], L["cs"], L["what"], L["dwh"], None, L["Xq"], L["dx"],
                                  L["xo"] if n else None, L["Wq"], L["dw"], L["A"], L["B"], r, p.lora_scale, L["Y"][b],
                                  L["ws"])
                q.linear_bwd_step(L["dY"][b], L["X"][b], L["Wq"], L["dw"], p.c_in, p.c_out, L["A"], L["B"], r,
                                  p.lora_scale, L["dX"][b], L["dA"], L["dB"], L["bws"])
        for i in range(3):
            two_call_step(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            two_call_step(i)
        e1.record()
        torch.cuda.synchronize()
        f_ms = e0.elapsed_time(e1) / args.steps
        extra["full_step_with_lora_grads"] = {
            "ms_per_step": round(f_ms, 5),
            "calls_per_step": "quaff_linear_fwd_step + quaff_linear_bwd_step (dX, dA, dB) per projection",
            "tops": round(total_ops / (f_ms * 1e-3) / 1e12, 2),
            "through_separate_calls_ms": round(ms_per_step + g_ms, 5)}
    if all(L["n"] for L in layers) and all(L["p"].backward for L in layers):
        for L in layers:
            L["ows"] = torch.empty(q.bwd_dx_outlier_workspace_bytes(L["p"].t, L["p"].c_out), dtype=i8, device=dev)

        def exact_cols(i):
            b = i % args.batches
            for L in layers:
                q.bwd_dx_outlier_exact(L["dY"][b], L["p"].c_in, L["O"], L["W_O"], L["A"], L["B"], L["r"],
                                       L["p"].lora_scale, L["dX"][b], L["ows"])
        for i in range(3):
            exact_cols(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            exact_cols(i)
        e1.record()
        torch.cuda.synchronize()
        extra["exact_dx_on_outlier_channels"] = {
            "ms_per_step": round(e0.elapsed_time(e1) / args.steps, 5),
            "calls_per_step": "quaff_bwd_dx_outlier_exact per projection (after quaff_linear_bwd_dx)"}
    # bf16-output variant of the two products (four separate calls; compare with --separate-calls)
    if all(L["p"].backward and L["p"].c_in % 64 == 0 and L["p"].c_out % 64 == 0 and L["n"] <= 128 for L in layers):
        for L in layers:
            L["Y16"] = torch.empty((L["p"].t, L["p"].c_out), dtype=torch.int16, device=dev)
            L["dX16"] = torch.empty((L["p"].t, L["p"].c_in), dtype=torch.int16, device=dev)

        def step16(i):
            b = i % args.batches
            for L in layers:
                p, n, r = L["p"], L["n"], L["r"]
                X = L["X"][b]
                q.scale_update(X, L["O"], L["W_O"], L["wmax"], p.c_out, p.gamma, L["s"], L["cs"], L["what"], L["dwh"],
                               None, L["ws"])
                q.quant_act(X, L["cs"], L["O"], L["Xq"], L["dx"], L["xo"] if n else None)
                q.linear_fwd(L["Xq"], L["dx"], L["xo"] if n else None, L["Wq"], L["dw"], p.c_in, p.c_out,
                             L["what"] if n else None, L["dwh"] if n else None, n, X if r else None, L["A"], L["B"], r,
                             p.lora_scale, L["Y16"], L["ws"], bf16_out=True)
                q.linear_bwd_dx(L["dY"][b], L["Wq"], L["dw"], p.c_in, p.c_out, L["A"], L["B"], r, p.lora_scale,
                                L["dX16"], L["ws"], bf16_out=True)
        for i in range(3):
            step16(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            step16(i)
        e1.record()
        torch.cuda.synchronize()
        ms16 = e0.elapsed_time(e1) / args.steps
        extra["bf16_outputs"] = {"ms_per_step": round(ms16, 5), "tops": round(total_ops / (ms16 * 1e-3) / 1e12, 2),
                                 "calls_per_step": "scale_update, quant_act, linear_fwd_bf16, linear_bwd_dx_bf16"}
    # outlier identification (Eq. 6) on 32 calibration samples of 512 tokens of the first projection's recipe
    p0 = layers[0]["p"]
    ns, rows = 32, 512
    Xc = torch.cat([layers[0]["X"][b % args.batches][:rows] for b in range(ns)]).contiguous()
    offs = torch.arange(ns + 1, dtype=torch.int64, device=dev) * rows
    xi = torch.empty(p0.c_in, dtype=torch.int32, device=dev)
    Oc = torch.empty(max(layers[0]["n"], 1), dtype=torch.int32, device=dev)
    nc = torch.empty(1, dtype=torch.int32, device=dev)
    cws = torch.empty(q.calibrate_workspace_bytes(p0.c_in, ns), dtype=i8, device=dev)
    for i in range(3):
        q.calibrate_outliers(Xc, offs, 100.0, Oc.numel(), xi, Oc, nc, cws)
    torch.cuda.synchronize()
    e0.record()
    for i in range(10):
        q.calibrate_outliers(Xc, offs, 100.0, Oc.numel(), xi, Oc, nc, cws)
    e1.record()
    torch.cuda.synchronize()
    c_ms = e0.elapsed_time(e1) / 10
    extra["outlier_identification"] = {
        "ms_per_call": round(c_ms, 5), "workload": "%d samples x %d tokens x %d channels, budget %d" % (
            ns, rows, p0.c_in, Oc.numel()),
        "algorithmic_GBs": round(2.0 * ns * rows * p0.c_in / (c_ms * 1e-3) / 1e9, 1),
        "channels_selected": int(nc.item())}
    out["beyond_headline"] = extra

    # measured ceilings next to the published peaks (register-only MFMA loop, streaming copy)
    mf_const, clk_const = q.microbench_mfma_i8(False)
    mf_rand, clk_rand = q.microbench_mfma_i8(True)
    out["measured_ceilings"] = {
        "mfma_i8_register_loop_constant_operands": {"tops": round(mf_const, 1), "clock_mhz": round(clk_const)},
        "mfma_i8_register_loop_random_operands": {"tops": round(mf_rand, 1), "clock_mhz": round(clk_rand)},
        "stream_copy_GBs_read_plus_write": round(q.microbench_copy(1 << 30), 1),
        "gemm_frac_of_random_operand_mfma_rate": round(gemm_tops / mf_rand, 4)}

    if not args.no_cpu_baseline:
        # the oracle as it stands on the host cores: whole steps of the same workload (all projections, all rows),
        # repeated on successive batches until about 10 s of CPU work have been timed
        from oracle import api as orc
        nthreads = min(orc.max_threads(), 16)
        orc.set_threads(nthreads)
        state = []
        for L in layers:
            p = L["p"]
            W, O = synth.weight(p), synth.outlier_indices(p)
            A, B = synth.lora(p)
            Wq, dw = orc.weight_quantize(W)
            W_O, wmax = orc.outlier_rows(W, O)
            state.append(dict(p=p, O=O, A=A if p.lora_rank else None, B=B if p.lora_rank else None, Wq=Wq, dw=dw,
                              W_O=W_O, wmax=wmax, s=np.ones(O.size, np.float32), cs=np.ones(p.c_in, np.float32)))
        batches = [[(synth.activations(S["p"], b), synth.out_grad(S["p"], b) if S["p"].backward else None)
                    for S in state] for b in range(min(args.batches, 2))]
        secs, ops, nsteps = 0.0, 0.0, 0
        while secs < 10.0 and nsteps < 8:
            t0 = time.perf_counter()
            for S, (X, dY) in zip(state, batches[nsteps % len(batches)]):
                p = S["p"]
                S["s"], S["cs"], what, dwh, _ = orc.scale_update(X, S["O"], S["W_O"], S["wmax"], p.gamma, S["s"],
                                                                 S["cs"])
                Xq, dx, xo = orc.quant_act(X, S["cs"], S["O"])
                orc.linear_fwd(Xq, dx, xo, S["Wq"], S["dw"], what, dwh, X, S["A"], S["B"], p.lora_scale)
                ops += 2.0 * p.t * p.c_out * (p.c_in + S["O"].size)
                if p.backward:
                    orc.linear_bwd_dx(dY, S["Wq"], S["dw"], S["A"], S["B"], p.lora_scale)
                    ops += 2.0 * p.t * p.c_out * p.c_in
            secs += time.perf_counter() - t0
            nsteps += 1
        # one thread, first projection's forward only (bounded: the whole step would take about ten times longer)
        orc.set_threads(1)
        S, (X, dY) = state[-1], batches[0][-1]
        p = S["p"]
        t0 = time.perf_counter()
        _s, _cs, what, dwh, _ = orc.scale_update(X, S["O"], S["W_O"], S["wmax"], p.gamma, S["s"].copy(), S["cs"].copy())
        Xq, dx, xo = orc.quant_act(X, _cs, S["O"])
        orc.linear_fwd(Xq, dx, xo, S["Wq"], S["dw"], what, dwh, X, S["A"], S["B"], p.lora_scale)
        one_secs = time.perf_counter() - t0
        one_tops = 2.0 * p.t * p.c_out * (p.c_in + S["O"].size) / one_secs / 1e12
        orc.set_threads(nthreads)
        out["cpu_baseline"] = {"single_thread": {"value": round(one_tops, 5), "unit": "TOPS", "cores": 1,
                                                 "seconds": round(one_secs, 2),
                                                 "sample": "forward of %s (scale update, quantize, forward)" % p.name},
                               "value": round(ops / secs / 1e12, 5), "unit": "TOPS", "cores": nthreads,
                               "kind": "oracle", "seconds": round(secs, 2),
                               "sample": "%d whole step(s) of the same workload (every projection, all %d rows: scale "
                                         "update, quantize, forward, dX)" % (nsteps, layers[0]["p"].t)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
