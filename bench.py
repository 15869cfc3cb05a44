#!/usr/bin/env python3
"""Benchmark of the Quaff quantized-linear hot path on one MI355X.

A "step" is one pass of the whole path - scale update, scale+quantize, INT8 forward with fused dequant+LoRA
epilogue, and the dX backward - over every projection of the workload for one synthetic batch, with all inputs
already resident in HBM.  Prints ONE JSON line.  The headline (`value`, `roofline`, `cpu_baseline`) is the
Phi-3-mini attention workload (configs[1]); `per_config` holds the same measurements for the other workloads.
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
DEV = "cuda:0"
TRAFFIC_PROFILE = os.path.join("profiles", "gemm_i8_hbm_traffic_phi3_attention.md")


def distinct_shapes(projs):
    seen, keep = set(), []
    for p in projs:
        if (p.c_in, p.c_out) not in seen:
            seen.add((p.c_in, p.c_out))
            keep.append(p)
    return keep


def build_layers(cfg, batches, generated_batches):
    """Device-side state of every projection of workload `cfg`.  `generated_batches` input batches are drawn from the
    seeded generator; further batches are the first one with its token rows rotated (distinct memory, the same
    columns and distribution), which bounds the host time of the long-sequence workloads."""
    import numpy as np
    import torch
    from paper_2505_14742_amd import binding as q
    from paper_2505_14742_amd import synth
    i8, f32 = torch.int8, torch.float32

    def bf16_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)

    projs = synth.CONFIGS[cfg]
    if cfg in (4, 5):   # the distinct shapes of the decoder layer (q = k = v = o, gate = up)
        projs = distinct_shapes(projs)
    layers = []
    for p in projs:
        W, O = synth.weight(p), synth.outlier_indices(p)
        A, B = synth.lora(p)
        n, r = int(O.size), p.lora_rank
        n_pad = q.padded_outliers(n)
        L = dict(p=p, n=n, r=r, n_pad=n_pad)
        L["O"] = torch.from_numpy(O).to(DEV) if n else None
        L["A"] = bf16_dev(A) if r else None
        L["B"] = bf16_dev(B) if r else None
        Wd = torch.from_numpy(W).to(DEV)
        L["Wq"] = torch.empty(q.packed_weight_bytes(p.c_in, p.c_out), dtype=i8, device=DEV)
        L["dw"] = torch.empty(p.c_out, dtype=f32, device=DEV)
        L["W_O"] = torch.empty((max(n, 1), p.c_out), dtype=f32, device=DEV)
        L["wmax"] = torch.empty(max(n, 1), dtype=f32, device=DEV)
        ws = torch.empty(q.prepare_workspace_bytes(p.c_in, p.c_out), dtype=i8, device=DEV)
        q.prepare_weight(Wd, L["O"], L["Wq"], L["dw"], L["W_O"] if n else None, L["wmax"] if n else None, None, ws)
        del Wd, ws, W
        L["s"] = torch.ones(max(n, 1), dtype=f32, device=DEV)
        L["cs"] = torch.ones(p.c_in, dtype=f32, device=DEV)
        L["what"] = torch.zeros((p.c_out, max(n_pad, 1)), dtype=i8, device=DEV)
        L["dwh"] = torch.zeros(p.c_out, dtype=f32, device=DEV)
        L["ws"] = torch.empty(max(q.workspace_bytes(p.t, p.c_in, p.c_out, n, r),
                                  q.fwd_step_workspace_bytes(p.t, p.c_in, p.c_out, n, r)), dtype=i8, device=DEV)
        gen = min(batches, generated_batches)
        L["X"] = [bf16_dev(synth.activations(p, s)) for s in range(gen)]
        L["dY"] = [bf16_dev(synth.out_grad(p, s)) for s in range(gen)] if p.backward else None
        for b in range(gen, batches):
            shift = (b * p.t) // (batches + 1) + 1
            L["X"].append(torch.roll(L["X"][0], shift, 0).contiguous())
            if p.backward:
                L["dY"].append(torch.roll(L["dY"][0], shift, 0).contiguous())
        L["Xq"] = torch.empty((p.t, p.c_in), dtype=i8, device=DEV)
        L["dx"] = torch.empty(p.t, dtype=f32, device=DEV)
        L["xo"] = torch.zeros((p.t, max(n_pad, 1)), dtype=i8, device=DEV)
        L["Y"] = [torch.empty((p.t, p.c_out), dtype=f32, device=DEV) for _ in range(batches)]
        L["dX"] = [torch.empty((p.t, p.c_in), dtype=f32, device=DEV) for _ in range(batches)]
        L["fwd_ops"] = 2.0 * p.t * p.c_out * (p.c_in + n)
        L["bwd_ops"] = 2.0 * p.t * p.c_out * p.c_in if p.backward else 0.0
        layers.append(L)
    return layers


def make_step(layers, batches, separate_default):
    from paper_2505_14742_amd import binding as q

    def step(i, separate=None):
        separate = separate_default if separate is None else separate
        b = i % batches
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
    return step


def time_steps(step, steps):
    """(ms per step by events, ms per step by the host clock) of `steps` steps, bracketed by synchronize on both
    sides.  The events are recorded on torch's current stream, which is the stream every call is enqueued on."""
    import torch
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    return max(e0.elapsed_time(e1), 0.0) / steps, (time.perf_counter() - t0) * 1e3 / steps


def profile_steps(step, nsteps, **kw):
    """Per-launch durations (HIP events recorded by the library around each launch, on the launch stream) of nsteps
    steps, in a pass of their own: the events perturb the step time."""
    import torch
    from paper_2505_14742_amd import binding as q
    q.profile_enable(True)
    for i in range(nsteps):
        step(i, **kw)
    torch.cuda.synchronize()
    launches = q.profile_launches()
    q.profile_enable(False)
    kinds = {}
    for name, ms in launches:
        k = kinds.setdefault(name, [0.0, 0])
        k[0] += ms
        k[1] += 1
    return launches, kinds


def gemm_stats(layers, launches, nsteps):
    """Aggregate and per-shape figures of the GEMM launches (they come in call order: per layer forward, then dX)."""
    gemm_ms = [ms for name, ms in launches if name == "gemm_i8"]
    order = []
    for L in layers:
        order.append((L["p"].name + ".fwd", L["fwd_ops"]))
        if L["p"].backward:
            order.append((L["p"].name + ".bwd_dx", L["bwd_ops"]))
    per_step = len(gemm_ms) // nsteps
    shapes = {}
    if per_step == len(order):     # one launch per product (a wide outlier set adds a launch: aggregate only)
        acc = {}
        for idx, ms in enumerate(gemm_ms):
            nm, ops = order[idx % len(order)]
            st = acc.setdefault(nm, [0.0, 0, ops])
            st[0] += ms
            st[1] += 1
        for nm, st in acc.items():
            avg = st[0] / st[1]
            shapes[nm] = {"avg_us": round(avg * 1e3, 2), "tops": round(st[2] / (avg * 1e-3) / 1e12, 1),
                          "frac_peak": round(st[2] / (avg * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)}
    ops = sum(L["fwd_ops"] + L["bwd_ops"] for L in layers) * nsteps
    total_ms = sum(gemm_ms)
    tops = ops / (total_ms * 1e-3) / 1e12
    return tops, total_ms / max(len(gemm_ms), 1), per_step, shapes


def gemm_algorithmic_bytes(layers):
    """HBM bytes the GEMM launches of one step must move: operands once, output once."""
    nbytes = 0.0
    for L in layers:
        p = L["p"]
        nbytes += p.t * p.c_in + p.c_in * p.c_out + (p.t + p.c_out) * L["n_pad"] + 4.0 * p.t * p.c_out
        if p.backward:
            nbytes += p.t * p.c_out + p.c_in * p.c_out + 4.0 * p.t * p.c_in
    return nbytes


def kernel_stats(layers, kinds, launches, nsteps, copy_gbs):
    """Per kernel kind: average / minimum / median launch duration and, for the memory-bound ones, algorithmic bytes
    over time against the 8 TB/s HBM peak and against the streaming-copy rate measured on this machine."""
    quant_bytes = fused_bytes = lora_bytes = 0.0
    for L in layers:
        p, r = L["p"], L["r"]
        quant_bytes += 3.0 * p.t * p.c_in + 4.0 * p.t + p.t * L["n_pad"]          # 2 B read, 1 B written per element
        if r:
            lora_bytes += 2.0 * p.t * p.c_in + 2.0 * p.c_in * r + 8.0 * p.t * r + 4.0 * p.c_out * r
        if p.backward:   # one launch quantizes dY and forms dY B^T
            fused_bytes += 3.0 * p.t * p.c_out + 4.0 * p.t + (2.0 * p.c_out * r + 8.0 * p.t * r if r else 0.0)
    kernels = {name: {"avg_us": round(v[0] / v[1] * 1e3, 2), "launches_per_step": v[1] // nsteps,
                      "us_per_step": round(v[0] / nsteps * 1e3, 2)} for name, v in kinds.items()}

    def hbm(name, nbytes):
        if name in kernels and nbytes:
            ms = kinds[name][0] / nsteps
            gbs = nbytes / (ms * 1e-3) / 1e9
            kernels[name]["achieved_GBs"] = round(gbs, 1)
            kernels[name]["frac_hbm_peak"] = round(gbs / HBM_PEAK_GBS, 4)
            if copy_gbs:
                kernels[name]["frac_measured_copy_rate"] = round(gbs / copy_gbs, 4)
    what_bytes = sum(4.0 * L["n"] * L["p"].c_out + L["n_pad"] * L["p"].c_out + 4.0 * L["p"].c_out for L in layers)
    # one-launch forward preparation: X read once, codes + compact outlier codes + steps written, what requantized,
    # the LoRA factors read and T (hi / lo pair of both parts) and the transposed B written
    prep_bytes = quant_bytes + what_bytes + sum(
        (2.0 * L["p"].c_in * L["r"] + 8.0 * L["p"].t * L["r"] + 4.0 * L["p"].c_out * L["r"]) if L["r"] else 0.0
        for L in layers)
    hbm("fwd_prep", prep_bytes)
    if "quant_rows+lora_down" in kernels:
        hbm("quant_rows", quant_bytes)
        hbm("quant_rows+lora_down", fused_bytes)
        hbm("lora_down", lora_bytes)
        hbm("colmax_outlier+lora_down", lora_bytes)   # the abs-max gather adds about a third of X's bytes
        hbm("momentum_what+quant_rows", quant_bytes + what_bytes)
    else:   # rank 0 or shapes the combined launches do not cover: separate launches in the backward pass too
        hbm("quant_rows", quant_bytes + fused_bytes)
        hbm("lora_down", lora_bytes)
    # column abs-max: useful bytes are the 2-byte outlier entries; what the memory system must fetch is one 64-byte
    # segment per (row, distinct segment touched by O) - counted here from the outlier positions
    if "colmax_outlier" in kernels:
        useful = fetched = 0.0
        for L in layers:
            if L["n"]:
                seg = len(set(int(o) // 32 for o in L["O"].cpu().tolist()))
                useful += 2.0 * L["p"].t * L["n"]
                # the library streams whole rows when the outliers touch most segments anyway (n * 64 >= c_in)
                fetched += 2.0 * L["p"].t * L["p"].c_in if L["n"] * 64 >= L["p"].c_in else 64.0 * L["p"].t * seg
        col_ms = kinds["colmax_outlier"][0] / nsteps
        kernels["colmax_outlier"]["useful_GBs"] = round(useful / (col_ms * 1e-3) / 1e9, 1)
        kernels["colmax_outlier"]["fetched_GBs"] = round(fetched / (col_ms * 1e-3) / 1e9, 1)
        kernels["colmax_outlier"]["frac_hbm_peak_fetched"] = round(fetched / (col_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    for name in kinds:
        ds = sorted(ms for nm, ms in launches if nm == name)
        kernels[name]["min_us"] = round(ds[0] * 1e3, 2)
        kernels[name]["median_us"] = round(ds[len(ds) // 2] * 1e3, 2)
    return kernels


def gemm_cold_vs_warm(layers):
    """GEMM launch times of each projection with its operands cached (one operand set used again and again) and from
    HBM (enough copies of the operand set used in turn, more than 640 MB in all, that none is left in the 256 MB
    Infinity Cache when its turn comes), back to back without idling.  The codes of the weight are copied device to
    device; activations and gradients are random codes."""
    import torch
    from paper_2505_14742_amd import binding as q
    res = {}
    for L in layers:
        p, n, r = L["p"], L["n"], L["r"]
        t, K, N = p.t, p.c_in, p.c_out
        nset = max(2, int(640e6 / (t * K + K * N + 4 * t * N + 2 * t * N + 4 * t * K)) + 1)
        sets = [dict(Xq=torch.randint(-40, 41, (t, K), dtype=torch.int8, device=DEV), Wq=L["Wq"].clone(),
                     dY=L["dY"][0].clone(), Y=torch.empty_like(L["Y"][0]), dX=torch.empty_like(L["dX"][0]))
                for _ in range(nset)]
        row = {}
        for mode in ("cached", "from_hbm"):
            for which in ("fwd", "bwd_dx"):
                def call(i):
                    S = sets[i % nset] if mode == "from_hbm" else sets[0]
                    if which == "fwd":
                        q.linear_fwd(S["Xq"], L["dx"], L["xo"] if n else None, S["Wq"], L["dw"], K, N,
                                     L["what"] if n else None, L["dwh"] if n else None, n, L["X"][0] if r else None,
                                     L["A"], L["B"], r, p.lora_scale, S["Y"], L["ws"])
                    else:
                        q.linear_bwd_dx(S["dY"], S["Wq"], L["dw"], K, N, L["A"], L["B"], r, p.lora_scale, S["dX"], L["ws"])
                for i in range(nset + 2):
                    call(i)
                torch.cuda.synchronize()
                q.profile_enable(True)
                for i in range(2 * nset + 4):
                    call(i)
                torch.cuda.synchronize()
                ts = sorted(x[1] * 1e3 for x in q.profile_launches() if x[0] == "gemm_i8")
                q.profile_enable(False)
                row["%s.%s_us" % (which, mode)] = round(ts[len(ts) // 2], 2)
        row["operand_sets"] = nset
        res[p.name] = row
        del sets
        torch.cuda.empty_cache()
    return res


def workload_name(cfg, layers):
    shapes = ", ".join("%s t=%d %d->%d |O|=%d r=%d" % (L["p"].name, L["p"].t, L["p"].c_in, L["p"].c_out, L["n"], L["r"])
                       for L in layers)
    if cfg <= 5:
        return "configs[%d]: %s" % (cfg - 1, shapes)
    return "paper's outlier budget (4 %% / 10 %% of c_in) at the Phi-3 shapes: %s" % shapes


def oracle_baseline(layers, budget_s):
    """The CPU oracle as it stands, on the host cores, over the same workload.  A workload whose whole step fits the
    budget runs whole steps (all rows).  A larger one runs one step with the scale update and the quantizers on all
    rows and the two products - whose rows are independent (Eq. 9) - on a deterministic row subset (every 16th row
    plus the first and last row of every 256-row block); its whole-step time is the labelled linear extrapolation."""
    import numpy as np
    from oracle import api as orc
    from paper_2505_14742_amd import synth
    nthreads = min(orc.max_threads(), 16)
    orc.set_threads(nthreads)
    total_ops = sum(L["fwd_ops"] + L["bwd_ops"] for L in layers)
    full = total_ops <= 1.5e12        # about 3 s per step at the oracle's usual rate
    state = []
    for L in layers:
        p = L["p"]
        W, O = synth.weight(p), synth.outlier_indices(p)
        A, B = synth.lora(p)
        Wq, dw = orc.weight_quantize(W)
        W_O, wmax = orc.outlier_rows(W, O)
        state.append(dict(p=p, O=O, A=A if p.lora_rank else None, B=B if p.lora_rank else None, Wq=Wq, dw=dw,
                          W_O=W_O, wmax=wmax, s=np.ones(O.size, np.float32), cs=np.ones(p.c_in, np.float32)))
        del W
    secs = ops = 0.0
    if full:
        batches = [[(synth.activations(S["p"], b), synth.out_grad(S["p"], b) if S["p"].backward else None)
                    for S in state] for b in range(2)]
        nsteps = 0
        while secs < budget_s and nsteps < 8:
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
        res = {"value": round(ops / secs / 1e12, 5), "unit": "TOPS", "cores": nthreads, "kind": "oracle",
               "seconds": round(secs, 2),
               "sample": "%d whole step(s) of the same workload (every projection, all %d rows: scale update, "
                         "quantize, forward, dX)" % (nsteps, layers[0]["p"].t)}
        return res, state, batches
    est = 0.0
    used = 0
    for S in state:
        p = S["p"]
        rows = set(range(0, p.t, 16))
        for b0 in range(0, p.t, 256):
            rows.add(b0)
            rows.add(min(p.t, b0 + 256) - 1)
        rows = np.array(sorted(rows), dtype=np.int64)
        X = synth.activations(p, 0)
        dY = synth.out_grad(p, 0) if p.backward else None
        t0 = time.perf_counter()
        S["s"], S["cs"], what, dwh, _ = orc.scale_update(X, S["O"], S["W_O"], S["wmax"], p.gamma, S["s"], S["cs"])
        Xq, dx, xo = orc.quant_act(X, S["cs"], S["O"])
        if p.backward:
            orc.quant_act(dY, S["dw"])             # the dX call's quantizer pass over all rows of dY
        t_all = time.perf_counter() - t0
        Xs, dYs = np.ascontiguousarray(X[rows]), (np.ascontiguousarray(dY[rows]) if p.backward else None)
        Xqs, dxs, xos = np.ascontiguousarray(Xq[rows]), np.ascontiguousarray(dx[rows]), np.ascontiguousarray(xo[rows])
        t0 = time.perf_counter()
        orc.linear_fwd(Xqs, dxs, xos, S["Wq"], S["dw"], what, dwh, Xs, S["A"], S["B"], p.lora_scale)
        if p.backward:
            orc.linear_bwd_dx(dYs, S["Wq"], S["dw"], S["A"], S["B"], p.lora_scale)
        t_rows = time.perf_counter() - t0
        est += t_all + t_rows * (p.t / float(rows.size))
        secs += t_all + t_rows
        used += int(rows.size)
        ops += 2.0 * p.t * p.c_out * (p.c_in + S["O"].size) + (2.0 * p.t * p.c_out * p.c_in if p.backward else 0.0)
        del X, dY, Xq
    res = {"value": round(ops / est / 1e12, 5), "unit": "TOPS", "cores": nthreads, "kind": "oracle",
           "seconds": round(secs, 2), "extrapolated_step_seconds": round(est, 2),
           "sample": "one step: scale update and quantizers on all rows, the two products on every 16th row plus the "
                     "first and last row of every 256-row block (%d rows over %d projections); whole-step time is "
                     "the linear extrapolation over the rows, not a full run" % (used, len(state))}
    return res, state, None


def measure_config(cfg, steps, warmup, batches, generated_batches, copy_gbs, cpu_budget_s):
    """Whole-step time, GEMM and memory-kernel figures of one workload (the per_config entries)."""
    import torch
    layers = build_layers(cfg, batches, generated_batches)
    step = make_step(layers, batches, False)
    for i in range(warmup):
        step(i)
    ms, _wall = time_steps(step, steps)
    total_ops = sum(L["fwd_ops"] + L["bwd_ops"] for L in layers)
    nprof = min(steps, 10)
    launches, kinds = profile_steps(step, nprof)
    gemm_tops, _avg, _n, shapes = gemm_stats(layers, launches, nprof)
    out = {"workload": workload_name(cfg, layers), "ms_per_step": round(ms, 5), "steps": steps, "warmup": warmup,
           "tops": round(total_ops / (ms * 1e-3) / 1e12, 2),
           "frac_int8_peak_whole_step": round(total_ops / (ms * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4),
           "gemm": {"achieved_tops": round(gemm_tops, 2), "frac_peak": round(gemm_tops / INT8_PEAK_TOPS, 4),
                    "per_shape": shapes},
           "kernels": {k: v for k, v in kernel_stats(layers, kinds, launches, nprof, copy_gbs).items()
                       if k != "gemm_i8"},
           "batches_rotated": batches, "batches_generated": min(batches, generated_batches)}
    if cpu_budget_s > 0:
        out["cpu_baseline"] = oracle_baseline(layers, cpu_budget_s)[0]
    del layers, step
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="headline workload (BASELINE.json configs, 1-based)")
    ap.add_argument("--batches", type=int, default=4, help="distinct input batches rotated through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the other workloads (per_config)")
    ap.add_argument("--no-extras", action="store_true", help="skip the rows beyond the headline metric")
    ap.add_argument("--separate-calls", action="store_true",
                    help="forward as scale_update + quant_act + linear_fwd instead of the one-call forward step")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path is built and measured on ONE GPU only (no collectives, no sharding); "
                 "run with --gpus 1")

    import torch
    from paper_2505_14742_amd import binding as q
    q.lib()
    torch.cuda.set_device(0)
    i8, f32 = torch.int8, torch.float32

    layers = build_layers(args.config, args.batches, args.batches if args.config != 5 else 1)
    step = make_step(layers, args.batches, args.separate_calls)

    # Measured ceilings next to the published peaks (register-only MFMA loop, streaming copy) come first: they need
    # nothing from the workload, and the chip has left its idle power state by the time the warm-up steps start (the
    # first steps after an idle period run 5 - 40 % slower than the steady state, which W warm-up steps of 0.3 ms
    # each do not outlast).
    copy_gbs = q.microbench_copy(1 << 30)
    mf_const, clk_const = q.microbench_mfma_i8(False)
    mf_rand, clk_rand = q.microbench_mfma_i8(True)

    for i in range(args.warmup):
        step(i)
    ms_per_step, wall_ms = time_steps(step, args.steps)
    total_ops = sum(L["fwd_ops"] + L["bwd_ops"] for L in layers)
    tops = total_ops / (ms_per_step * 1e-3) / 1e12

    # "warm" variant for comparison: the same batch every step (inputs and outputs may stay in the Infinity Cache);
    # the headline figures above are the rotated ("cold") ones
    warm_ms_per_step, _ = time_steps(lambda i: step(0), args.steps)

    # ---- per-kernel durations with HIP events on the launch stream (separate pass: the events perturb the step)
    prof_steps = min(args.steps, 20)
    launches, kinds = profile_steps(step, prof_steps)
    gemm_tops, gemm_avg_ms, gemm_per_step, gemm_shapes = gemm_stats(layers, launches, prof_steps)
    gemm_bytes = gemm_algorithmic_bytes(layers)
    # HBM traffic of the GEMM launches: counters cannot be read from inside the process, so this is the figure
    # RECORDED under profiles/ by two rocprofv3 --pmc runs of this command (FETCH_SIZE, WRITE_SIZE) together with
    # the commit it was taken at; null for workloads without such a record
    gemm_traffic, traffic_commit = None, None
    prof_file = os.path.join(ROOT, TRAFFIC_PROFILE)
    if args.config == 2 and os.path.exists(prof_file):
        for ln in open(prof_file):
            if ln.strip().startswith("gemm_traffic_bytes_per_launch"):
                gemm_traffic = int(ln.split("=")[1])
            if ln.strip().startswith("measured_at_commit"):
                traffic_commit = ln.split("=")[1].strip()
    kernels = kernel_stats(layers, kinds, launches, prof_steps, copy_gbs)
    kernels_separate = None
    if not args.separate_calls:
        # the same step through the four separate calls, for the stand-alone figures of the abs-max, momentum,
        # quantizer and down-projection kernels
        for i in range(3):              # untimed: the first launch of a kernel pays for loading its code
            step(i, separate=True)
        torch.cuda.synchronize()
        sep_steps = min(args.steps, 10)
        sep_launches, sep_kinds = profile_steps(step, sep_steps, separate=True)
        kernels_separate = kernel_stats(layers, sep_kinds, sep_launches, sep_steps, copy_gbs)
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
        "config": {"workload": workload_name(args.config, layers), "batches_rotated": args.batches, "calls_per_step":
                   ("scale_update, quant_act, linear_fwd, linear_bwd_dx per projection" if args.separate_calls else
                    "linear_fwd_step (= scale_update + quant_act + linear_fwd), linear_bwd_dx per projection")},
        "frac_int8_peak_whole_step": round(tops / INT8_PEAK_TOPS, 4),
        "wall_ms_per_step": round(wall_ms, 5),
        "warm_same_batch_ms_per_step": round(warm_ms_per_step, 5),
        "roofline": {"bound": "mfma", "kernel": "gemm_i8 (all launches of the step)", "achieved": round(gemm_tops, 2),
                     "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": round(gemm_tops / INT8_PEAK_TOPS, 4),
                     "achieved_source": "algorithmic ops of the GEMM launches / their HIP-event durations, recorded by "
                                        "the library on the launch stream during this run (the rocprofv3 kernel-trace "
                                        "summary of the same command under profiles/ agrees)",
                     "avg_launch_us": round(gemm_avg_ms * 1e3, 2),
                     "traffic": gemm_traffic,
                     "traffic_source": "RECORDED, not measured by this run: rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE per "
                                       "average GEMM launch, scaled by the copy kernel, from %s (taken at commit %s)"
                                       % (TRAFFIC_PROFILE, traffic_commit),
                     "algorithmic_bytes_per_launch": round(gemm_bytes / max(gemm_per_step, 1)),
                     "per_shape": gemm_shapes,
                     "note": "priced against the INT8 MFMA peak as a contraction; measured_ceilings holds the "
                             "power-limited MFMA rate of this box"},
        "kernels": kernels,
        "kernels_with_separate_calls": kernels_separate,
    }

    # ---- rows beyond the headline metric, timed on their own (not part of `value`)
    extra = {}
    if not args.no_extras and all(L["r"] for L in layers) and all(L["p"].backward for L in layers):
        for L in layers:
            p, r = L["p"], L["r"]
            L["dA"] = torch.empty((p.c_in, r), dtype=f32, device=DEV)
            L["dB"] = torch.empty((r, p.c_out), dtype=f32, device=DEV)
            L["gws"] = torch.empty(q.lora_bwd_workspace_bytes(p.t, p.c_in, p.c_out, r), dtype=i8, device=DEV)

        def grads(i):
            b = i % args.batches
            for L in layers:
                q.lora_bwd_weights(L["X"][b], L["dY"][b], L["A"], L["B"], L["r"], L["p"].lora_scale, L["dA"], L["dB"],
                                   L["gws"])
        for i in range(3):
            grads(i)
        g_ms, _ = time_steps(grads, args.steps)
        g_bytes = sum(2.0 * L["p"].t * (L["p"].c_in + L["p"].c_out) for L in layers)
        extra["lora_weight_grads"] = {
            "ms_per_step": round(g_ms, 5), "calls_per_step": "quaff_lora_bwd_weights per projection (dA, dB)",
            "algorithmic_GBs": round(g_bytes / (g_ms * 1e-3) / 1e9, 1),
            "frac_hbm_peak": round(g_bytes / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "algorithmic_bytes": "X and dY read once (2 t (c_in + c_out))"}
        # the whole fine-tuning step of the layers: one forward call and one backward call (dX, dA, dB) per projection
        for L in layers:
            p = L["p"]
            L["bws"] = torch.empty(q.bwd_step_workspace_bytes(p.t, p.c_in, p.c_out, L["r"]), dtype=i8, device=DEV)
        side = q.SideStream()   # the caller's second stream for the weight gradients of quaff_linear_bwd_step

        def two_call_step(i):
            b = i % args.batches
            for L in layers:
                p, n, r = L["p"], L["n"], L["r"]
                q.linear_fwd_step(L["X"][b], L["O"], L["W_O"] if n else None, L["wmax"] if n else None, p.c_out,
                                  p.gamma, L["s"], L["cs"], L["what"], L["dwh"], None, L["Xq"], L["dx"],
                                  L["xo"] if n else None, L["Wq"], L["dw"], L["A"], L["B"], r, p.lora_scale, L["Y"][b],
                                  L["ws"])
                q.linear_bwd_step(L["dY"][b], L["X"][b], L["Wq"], L["dw"], p.c_in, p.c_out, L["A"], L["B"], r,
                                  p.lora_scale, L["dX"][b], L["dA"], L["dB"], L["bws"], side=side)
        for i in range(3):
            two_call_step(i)
        f_ms, _ = time_steps(two_call_step, args.steps)
        extra["full_step_with_lora_grads"] = {
            "ms_per_step": round(f_ms, 5),
            "calls_per_step": "quaff_linear_fwd_step + quaff_linear_bwd_step (dX, dA, dB; weight gradients on the "
                              "caller's second stream) per projection",
            "tops": round(total_ops / (f_ms * 1e-3) / 1e12, 2),
            "through_separate_calls_ms": round(ms_per_step + g_ms, 5)}
    if not args.no_extras and all(L["n"] for L in layers) and all(L["p"].backward for L in layers):
        for L in layers:
            L["ows"] = torch.empty(q.bwd_dx_outlier_workspace_bytes(L["p"].t, L["p"].c_out), dtype=i8, device=DEV)

        def exact_cols(i):
            b = i % args.batches
            for L in layers:
                q.bwd_dx_outlier_exact(L["dY"][b], L["p"].c_in, L["O"], L["W_O"], L["A"], L["B"], L["r"],
                                       L["p"].lora_scale, L["dX"][b], L["ows"])
        for i in range(3):
            exact_cols(i)
        x_ms, _ = time_steps(exact_cols, args.steps)
        extra["exact_dx_on_outlier_channels"] = {
            "ms_per_step": round(x_ms, 5),
            "calls_per_step": "quaff_bwd_dx_outlier_exact per projection (after quaff_linear_bwd_dx)"}
    # bf16-output variant of the two products (four separate calls; compare with --separate-calls)
    if not args.no_extras and all(L["p"].backward and L["p"].c_in % 64 == 0 and L["p"].c_out % 64 == 0 and
                                  L["n"] <= 128 for L in layers):
        for L in layers:
            L["Y16"] = torch.empty((L["p"].t, L["p"].c_out), dtype=torch.int16, device=DEV)
            L["dX16"] = torch.empty((L["p"].t, L["p"].c_in), dtype=torch.int16, device=DEV)

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
        ms16, _ = time_steps(step16, args.steps)
        extra["bf16_outputs"] = {"ms_per_step": round(ms16, 5), "tops": round(total_ops / (ms16 * 1e-3) / 1e12, 2),
                                 "calls_per_step": "scale_update, quant_act, linear_fwd_bf16, linear_bwd_dx_bf16"}
    if not args.no_extras:
        # outlier identification (Eq. 6) on 32 calibration samples of 512 tokens of the first projection's recipe
        p0 = layers[0]["p"]
        ns, rows = 32, 512
        Xc = torch.cat([layers[0]["X"][b % args.batches][:rows] for b in range(ns)]).contiguous()
        offs = torch.arange(ns + 1, dtype=torch.int64, device=DEV) * rows
        xi = torch.empty(p0.c_in, dtype=torch.int32, device=DEV)
        Oc = torch.empty(max(layers[0]["n"], 1), dtype=torch.int32, device=DEV)
        nc = torch.empty(1, dtype=torch.int32, device=DEV)
        cws = torch.empty(q.calibrate_workspace_bytes(p0.c_in, ns), dtype=i8, device=DEV)
        for i in range(3):
            q.calibrate_outliers(Xc, offs, 100.0, Oc.numel(), xi, Oc, nc, cws)
        c_ms, _ = time_steps(lambda i: q.calibrate_outliers(Xc, offs, 100.0, Oc.numel(), xi, Oc, nc, cws), 10)
        extra["outlier_identification"] = {
            "ms_per_call": round(c_ms, 5), "workload": "%d samples x %d tokens x %d channels, budget %d" % (
                ns, rows, p0.c_in, Oc.numel()),
            "algorithmic_GBs": round(2.0 * ns * rows * p0.c_in / (c_ms * 1e-3) / 1e9, 1),
            "channels_selected": int(nc.item())}
        extra["gemm_operands_cached_vs_from_hbm"] = gemm_cold_vs_warm(layers)
        out["beyond_headline"] = extra

    out["measured_ceilings"] = {
        "mfma_i8_register_loop_constant_operands": {"tops": round(mf_const, 1), "clock_mhz": round(clk_const)},
        "mfma_i8_register_loop_random_operands": {"tops": round(mf_rand, 1), "clock_mhz": round(clk_rand)},
        "stream_copy_GBs_read_plus_write": round(copy_gbs, 1),
        "gemm_frac_of_random_operand_mfma_rate": round(gemm_tops / mf_rand, 4)}

    if not args.no_extras:
        # Context only, no part of the product: the vendor library's plain int8 product with int32 output (no
        # dequantisation, no outlier correction, no LoRA add) at the headline GEMM shapes, through torch._int_mm.
        vendor = {}
        try:
            for name, (m_, k_, n_) in (("qkv.fwd", (2048, 3072, 9216)), ("qkv.bwd_dx", (2048, 9216, 3072)),
                                        ("o_proj", (2048, 3072, 3072))):
                a8 = torch.randint(-127, 128, (m_, k_), dtype=torch.int8, device=DEV)
                b8 = torch.randint(-127, 128, (k_, n_), dtype=torch.int8, device=DEV)
                for _ in range(3):
                    torch._int_mm(a8, b8)
                v_ms, _ = time_steps(lambda i: torch._int_mm(a8, b8), 20)
                vendor[name] = {"us": round(v_ms * 1e3, 2), "tops": round(2.0 * m_ * k_ * n_ / (v_ms * 1e-3) / 1e12, 1)}
                del a8, b8
            vendor["what"] = "torch._int_mm (vendor library), int32 output, back-to-back launches timed with events"
        except Exception as e:      # not available in this build of the vendor stack: recorded, not fatal
            vendor = {"unavailable": str(e)[:200]}
        out["measured_ceilings"]["vendor_library_int8_gemm"] = vendor

    if not args.no_cpu_baseline:
        # the oracle as it stands on the host cores over the same workload, until about 10 s of CPU work are timed
        from oracle import api as orc
        base, state, batches = oracle_baseline(layers, 10.0)
        if batches is not None:
            # one thread, last projection's forward only (bounded: the whole step would take about ten times longer)
            nthreads = base["cores"]
            orc.set_threads(1)
            S, (X, dY) = state[-1], batches[0][-1]
            p = S["p"]
            t0 = time.perf_counter()
            _s, _cs, what, dwh, _ = orc.scale_update(X, S["O"], S["W_O"], S["wmax"], p.gamma, S["s"].copy(),
                                                     S["cs"].copy())
            Xq, dx, xo = orc.quant_act(X, _cs, S["O"])
            orc.linear_fwd(Xq, dx, xo, S["Wq"], S["dw"], what, dwh, X, S["A"], S["B"], p.lora_scale)
            one_secs = time.perf_counter() - t0
            one_tops = 2.0 * p.t * p.c_out * (p.c_in + S["O"].size) / one_secs / 1e12
            orc.set_threads(nthreads)
            base["single_thread"] = {"value": round(one_tops, 5), "unit": "TOPS", "cores": 1,
                                     "seconds": round(one_secs, 2),
                                     "sample": "forward of %s (scale update, quantize, forward)" % p.name}
        out["cpu_baseline"] = base
        del state, batches

    # ---- the other workloads: the same measurements with fewer steps (the long ones bound the run time)
    del layers, step
    torch.cuda.empty_cache()
    if not args.no_per_config:
        per = {}
        for cfg in (3, 4, 5, 6):
            if cfg == args.config:
                continue
            big = cfg == 5
            key = "configs[%d]" % (cfg - 1) if cfg <= 5 else "paper_outlier_budget"
            per[key] = measure_config(cfg, steps=6 if big else 20, warmup=2 if big else 5, batches=2 if big else 3,
                                      generated_batches=1 if big else 3, copy_gbs=copy_gbs,
                                      cpu_budget_s=0.0 if args.no_cpu_baseline else 4.0)
        out["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
