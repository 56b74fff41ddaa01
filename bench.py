#!/usr/bin/env python3
"""Benchmark of the PTQ4VM W8A8 quantized-linear hot path on one MI355X.

A "step" is one pass of the hot path over one synthetic batch of the Vim-B-shaped stack
(benchmark configs[3]): for each of 24 layers and each of its four linears
(in_proj 768->3072, x_proj 1536->80, dt_proj 48->1536, out_proj 1536->768; M = 256*197 rows)
  ptq4vm_quantize_pts  (fp16 -> int8, per-token static step, smoothing folded in)
  ptq4vm_w8a8_linear   (int8 MFMA GEMM + fused dequantization + bias -> fp16)
or, where an activation element is quantized exactly once anyway (K <= 128 or N <= 128: x_proj,
dt_proj), the single launch ptq4vm_w8a8_linear_fused, which computes the same codes and outputs
bit for bit without writing the codes to memory (--fused off times the two-launch form
everywhere).  Weight folding/quantization is offline (done once in setup, like the paper's stored
INT8 weights) and is not timed.  All inputs are resident in HBM before the
timed region; every layer has its own buffers (~1.1 GB per layer), so the working set of a step
(~27 GB) cannot sit in the 256 MB last-level cache.

After the timed configuration the other four configurations of the benchmark spec are timed the same
way (they take 0.04-4 ms per step) and reported under "configs"; for the two launch-bound ones
(configs 0 and 1) the headline of their record is the step replayed as one HIP graph.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, TOP/s
PEAK_F16_TFLOPS = 2500.0  # dense fp16 MFMA
PEAK_HBM_GBS = 8000.0     # HBM3E

# HBM traffic of the dominant kernel per launch: written by `python -m paper_2412_20386_amd.profile_summary`
# from two rocprofv3 --pmc runs of this script (FETCH_SIZE, WRITE_SIZE, each scaled by the 256 MiB copy that
# this script also issues).  Absent or for another workload: "traffic" is null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "dominant_kernel_traffic.json")
GRAPH_HEADLINE_CONFIGS = (0, 1)  # launch-bound: a step is tens of microseconds of kernels


def dominant_traffic(config: int):
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
        return float(rec["traffic_bytes"]) if int(rec["config"]) == config else None
    except (OSError, ValueError, KeyError):
        return None


def measure_config(args, config: int, full: bool):
    """Builds the buffers of one configuration, times its step and its kernels, frees the buffers.
    full: also the comparison schemes (fp16, per-token dynamic, zero offset, W4A4) and the CPU oracle."""
    import torch

    import paper_2412_20386_amd as ptq
    from paper_2412_20386_amd import synth

    dev = "cuda:0"
    cfg = synth.CONFIGS[config]
    n_layers = (args.layers if full and args.layers else None) or cfg.layers
    B, L, M = cfg.B, cfg.L, cfg.M

    # ------------------------------------------------------------------ setup (untimed)
    t0 = time.time()
    layers = []
    for layer in range(n_layers):
        lin = []
        for li, (name, K, N) in enumerate(cfg.linears):
            c = synth.make_linear_case(config, layer, li, device=dev)
            wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)  # offline weight preparation
            # One fused launch where it beats quantize + linear (measured crossovers: narrow outputs from ~16 k
            # rows, short reductions from ~24 k rows; below that the two small kernels are faster).
            fuse = args.fused == "auto" and ((N <= 128 and M >= 16384) or (K <= 128 and M >= 24576))
            lin.append(dict(name=name, K=K, N=N, fused=fuse,
                            x=c.x, w=c.w, bias=c.bias, s_tok=c.s_tok, wq=wq, s_w=s_w,
                            inv_m=inv_m, xq=torch.empty((M, K), dtype=torch.int8, device=dev),
                            y=torch.empty((M, N), dtype=torch.float16, device=dev)))
        layers.append(lin)
    s_row = torch.empty(M, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def step_w8a8(events=None):
        for lin in layers:
            for d in lin:
                if d["fused"]:
                    ptq.w8a8_linear_fused(d["x"], d["inv_m"], d["s_tok"], d["wq"], d["s_w"], d["bias"], B, L, y=d["y"])
                    continue
                ptq.quantize_pts(d["x"], d["inv_m"], d["s_tok"], B, L, xq=d["xq"])
                if events is not None and d["name"] == events["name"]:
                    a, b = events["pool"][len(events["pairs"])]  # created before the timed region
                    a.record()
                    ptq.w8a8_linear(d["xq"], d["wq"], d["s_tok"], d["s_w"], d["bias"], B, L, y=d["y"])
                    b.record()
                    events["pairs"].append((a, b))
                else:
                    ptq.w8a8_linear(d["xq"], d["wq"], d["s_tok"], d["s_w"], d["bias"], B, L, y=d["y"])

    def step_dynamic():
        """The per-token dynamic comparison scheme (Sec. 4, latency table of Sec. 6.4): steps computed online."""
        for lin in layers:
            for d in lin:
                ptq.quantize_dynamic(d["x"], d["inv_m"], xq=d["xq"], s_row=s_row)
                ptq.w8a8_linear(d["xq"], d["wq"], s_row, d["s_w"], d["bias"], 1, M, y=d["y"])

    def step_f16():
        for lin in layers:
            for d in lin:
                ptq.f16_linear(d["x"], d["w"], d["bias"], y=d["y"])

    # ------------------------------------------------------------------ timed region
    dominant = max(cfg.linears, key=lambda t: t[1] * t[2])  # most MACs: in_proj
    for _ in range(args.warmup):
        step_w8a8()
    torch.cuda.synchronize()
    n_dominant = sum(1 for lin in layers for d in lin if d["name"] == dominant[0] and not d["fused"])
    pool = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps * n_dominant)]
    events = dict(name=dominant[0], pairs=[], pool=pool)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]  # step boundaries, for the median
    gc.collect()
    gc.disable()  # no collector pauses inside the timed region
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for s in range(args.steps):
        step_w8a8(events)
        marks[s + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    gc.enable()
    ms_per_step = elapsed / args.steps * 1e3
    step_ms = sorted(marks[s].elapsed_time(marks[s + 1]) for s in range(args.steps))
    dom_all = sorted(a.elapsed_time(b) * 1e3 for a, b in events["pairs"])
    dom_us = sum(dom_all) / len(dom_all) if dom_all else None

    # ------------------------------------------------------------------ the same step as one HIP graph (extra)
    graph_ms_per_step = None
    if not args.no_graph:
        side = torch.cuda.Stream()  # default priority
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step_w8a8()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step_w8a8()
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
        del graph

    # ------------------------------------------------------------------ per-kernel detail (untimed extras)
    def time_launch(fn, reps=3):
        """Average device time of fn: one HIP-event pair (on the launch stream) around a back-to-back
        sweep over all layers' distinct buffers, so that launch latency is hidden as in the stack."""
        fn(layers[0])
        sweeps = max(1, 24 // len(layers))  # short stacks (config 0 has one layer): repeat the sweep
        tot = 0.0
        for _ in range(reps):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(sweeps):
                for lin in layers:
                    fn(lin)
            b.record()
            b.synchronize()
            tot += a.elapsed_time(b)
        return tot / (reps * sweeps * len(layers)) * 1e3  # us

    kernels = []
    for li, (name, K, N) in enumerate(cfg.linears):
        tq = time_launch(lambda lin: ptq.quantize_pts(lin[li]["x"], lin[li]["inv_m"], lin[li]["s_tok"], B, L,
                                                     xq=lin[li]["xq"]))
        tg = time_launch(lambda lin: ptq.w8a8_linear(lin[li]["xq"], lin[li]["wq"], lin[li]["s_tok"], lin[li]["s_w"],
                                                    lin[li]["bias"], B, L, y=lin[li]["y"]))
        tf = time_launch(lambda lin: ptq.f16_linear(lin[li]["x"], lin[li]["w"], lin[li]["bias"], y=lin[li]["y"]))

        def pair(lin):  # as in the step: the linear reads codes that the quantizer has just written
            ptq.quantize_pts(lin[li]["x"], lin[li]["inv_m"], lin[li]["s_tok"], B, L, xq=lin[li]["xq"])
            ptq.w8a8_linear(lin[li]["xq"], lin[li]["wq"], lin[li]["s_tok"], lin[li]["s_w"], lin[li]["bias"], B, L, y=lin[li]["y"])
        tp = time_launch(pair)
        ops = 2.0 * M * K * N
        q_bytes = 3.0 * M * K + 4 * K + 4 * L
        g_bytes = 1.0 * M * K + N * K + 2.0 * M * N + 4 * L + 6 * N
        rec = dict(
            linear=name, K=K, N=N,
            quantize_us=round(tq, 2), quantize_GBps=round(q_bytes / tq / 1e3, 1),
            quantize_frac_hbm=round(q_bytes / tq / 1e3 / PEAK_HBM_GBS, 4),
            w8a8_us=round(tg, 2), w8a8_TOPS=round(ops / tg / 1e6, 1),
            w8a8_frac_int8_peak=round(ops / tg / 1e6 / PEAK_INT8_TOPS, 4),
            w8a8_GBps=round(g_bytes / tg / 1e3, 1), w8a8_frac_hbm=round(g_bytes / tg / 1e3 / PEAK_HBM_GBS, 4),
            f16_us=round(tf, 2), f16_TFLOPS=round(ops / tf / 1e6, 1),
            quantize_then_w8a8_us=round(tp, 2),  # the two launches back to back (codes still in the memory-side cache)
            speedup_gemm_only=round(tf / tg, 3), speedup_quant_plus_gemm=round(tf / tp, 3))
        if full:
            td = time_launch(lambda lin: ptq.quantize_dynamic(lin[li]["x"], lin[li]["inv_m"], xq=lin[li]["xq"], s_row=s_row))
            # per-token zero offset variant: timing only, offsets drawn at random
            z_tok = torch.randint(-20, 21, (L,), dtype=torch.int32, device=dev)
            rowsums = [ptq.weight_rowsum(lin[li]["wq"]) for lin in layers]
            tzq = time_launch(lambda lin: ptq.quantize_pts_offset(lin[li]["x"], lin[li]["inv_m"], lin[li]["s_tok"], z_tok,
                                                                  B, L, xq=lin[li]["xq"]))
            rs_of = {id(lin): r for lin, r in zip(layers, rowsums)}
            tzg = time_launch(lambda lin: ptq.w8a8_linear_offset(lin[li]["xq"], lin[li]["wq"], lin[li]["s_tok"], z_tok,
                                                                 rs_of[id(lin)], lin[li]["s_w"], lin[li]["bias"], B, L,
                                                                 y=lin[li]["y"]))
            tzf = None
            if layers[0][li]["fused"]:  # one launch: the offset quantizer in the loader
                try:
                    tzf = time_launch(lambda lin: ptq.w8a8_linear_offset_fused(lin[li]["x"], lin[li]["inv_m"], lin[li]["s_tok"],
                                                                               z_tok, lin[li]["wq"], rs_of[id(lin)],
                                                                               lin[li]["s_w"], lin[li]["bias"], B, L,
                                                                               y=lin[li]["y"]))
                except ptq.Ptq4vmError as e:  # a shape outside the two kernels that carry the fused forms
                    if e.status != -2:
                        raise
            # W4A4 (packed 4-bit codes): timing only
            t4q = t4g = t6q = t6g = t4f = None
            s4 = [(lin[li]["s_tok"] * (127.0 / 7.0)).contiguous() for lin in layers]
            idx = {id(lin): i for i, lin in enumerate(layers)}
            blocks6 = ptq.e2m3_blocks(K)
            if blocks6 * 96 <= K:  # the same codes in the FP6 (E2M3) container, where it fits the int8 code buffer (K % 128 == 0)
                w6 = [ptq.fold_smoothing_w4_e2m3(lin[li]["w"], 1.0 / lin[li]["inv_m"]) for lin in layers]
                xq6 = [lin[li]["xq"].view(torch.uint8).view(-1)[: blocks6 * M * 96].view(blocks6, M, 96) for lin in layers]
                t6q = time_launch(lambda lin: ptq.quantize_pts_a4_e2m3(lin[li]["x"], lin[li]["inv_m"], s4[idx[id(lin)]], B, L,
                                                                       xq6=xq6[idx[id(lin)]]))
                t6g = time_launch(lambda lin: ptq.w4a4_linear_e2m3(xq6[idx[id(lin)]], w6[idx[id(lin)]][0], s4[idx[id(lin)]],
                                                                   w6[idx[id(lin)]][1], lin[li]["bias"], B, L, K,
                                                                   y=lin[li]["y"]))
                del w6
            if K % 2 == 0:
                w4 = [ptq.fold_smoothing_w4(lin[li]["w"], 1.0 / lin[li]["inv_m"]) for lin in layers]
                xq4 = [lin[li]["xq"].view(torch.uint8).view(-1)[: M * (K // 2)].view(M, K // 2) for lin in layers]
                t4q = time_launch(lambda lin: ptq.quantize_pts_a4(lin[li]["x"], lin[li]["inv_m"], s4[idx[id(lin)]], B, L,
                                                                  xq4=xq4[idx[id(lin)]]))
                t4g = time_launch(lambda lin: ptq.w4a4_linear(xq4[idx[id(lin)]], w4[idx[id(lin)]][0], s4[idx[id(lin)]],
                                                              w4[idx[id(lin)]][1], lin[li]["bias"], B, L, y=lin[li]["y"]))
                if layers[0][li]["fused"]:  # one launch: quantizer in the loader of the W4A4 kernel
                    try:
                        t4f = time_launch(lambda lin: ptq.w4a4_linear_fused(lin[li]["x"], lin[li]["inv_m"], s4[idx[id(lin)]],
                                                                            w4[idx[id(lin)]][0], w4[idx[id(lin)]][1],
                                                                            lin[li]["bias"], B, L, y=lin[li]["y"]))
                    except ptq.Ptq4vmError as e:  # a shape outside the two kernels that carry the fused 4-bit form
                        if e.status != -2:
                            raise
                del w4
            rec.update(
                w4a4_fused_us=None if t4f is None else round(t4f, 2),
                offset_quantize_us=round(tzq, 2), offset_w8a8_us=round(tzg, 2),
                offset_fused_us=None if tzf is None else round(tzf, 2),
                a4_quantize_us=None if t4q is None else round(t4q, 2),
                a4_quantize_GBps=None if t4q is None else round((2.5 * M * K) / t4q / 1e3, 1),
                w4a4_us=None if t4g is None else round(t4g, 2),
                a4_e2m3_quantize_us=None if t6q is None else round(t6q, 2),
                a4_e2m3_quantize_GBps=None if t6q is None else round((2.75 * M * K) / t6q / 1e3, 1),
                w4a4_e2m3_us=None if t6g is None else round(t6g, 2),
                w4a4_e2m3_TOPS=None if t6g is None else round(ops / t6g / 1e6, 1),
                w4a4_best_us=None if (t4g is None and t6g is None) else round(min(t for t in (t4g, t6g) if t is not None), 2),
                w4a4_best_container=None if (t4g is None and t6g is None)
                else ("e2m3" if (t6g is not None and (t4g is None or t6g < t4g)) else "nibbles"),
                dynamic_quantize_us=round(td, 2), dynamic_quantize_GBps=round((q_bytes + 4.0 * M) / td / 1e3, 1))
        if layers[0][li]["fused"]:  # the form the timed step uses for this linear
            tfu = time_launch(lambda lin: ptq.w8a8_linear_fused(lin[li]["x"], lin[li]["inv_m"], lin[li]["s_tok"],
                                                                lin[li]["wq"], lin[li]["s_w"], lin[li]["bias"], B, L,
                                                                y=lin[li]["y"]))
            f_bytes = 2.0 * M * K + N * K + 2.0 * M * N + 4 * K + 4 * L + 6 * N
            rec.update(in_timed_step="fused", fused_us=round(tfu, 2), fused_GBps=round(f_bytes / tfu / 1e3, 1),
                       fused_frac_hbm=round(f_bytes / tfu / 1e3 / PEAK_HBM_GBS, 4), speedup_fused=round(tf / tfu, 3))
        else:
            rec.update(in_timed_step="quantize + w8a8")
        kernels.append(rec)

    total_ops = sum(2.0 * M * K * N for _, K, N in cfg.linears) * n_layers
    result = dict(config=config, cfg=cfg, n_layers=n_layers, ms_per_step=ms_per_step, step_ms=step_ms,
                  graph_ms_per_step=graph_ms_per_step, kernels=kernels, setup_s=setup_s, total_ops=total_ops,
                  dominant=dominant, dom_all=dom_all, dom_us=dom_us, launches_timed=len(events["pairs"]),
                  fused_linears=[d["name"] for d in layers[0] if d["fused"]])
    if not full:
        del layers, s_row
        torch.cuda.empty_cache()
        return result

    for _ in range(2):
        step_f16()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(max(1, args.steps // 2)):
        step_f16()
    torch.cuda.synchronize()
    result["f16_ms_per_step"] = (time.perf_counter() - t0) / max(1, args.steps // 2) * 1e3
    for _ in range(2):
        step_dynamic()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(max(1, args.steps // 2)):
        step_dynamic()
    torch.cuda.synchronize()
    result["dynamic_ms_per_step"] = (time.perf_counter() - t0) / max(1, args.steps // 2) * 1e3

    # W4A4 stack (the precision of the paper's latency table, Sec. 6.4): per layer and linear PTS-quantize to 4 bits +
    # W4A4 linear, in the form that the per-kernel sweep above found fastest for that linear: one fused launch, or two
    # launches on packed nibbles or on the FP6 (E2M3) container.
    result["w4a4_ms_per_step"] = None
    if all(k.get("w4a4_best_us") is not None for k in kernels):
        choice = []
        for k in kernels:
            nib = (k["a4_quantize_us"] + k["w4a4_us"]) if k.get("w4a4_us") is not None else float("inf")
            e2m3 = (k["a4_e2m3_quantize_us"] + k["w4a4_e2m3_us"]) if k.get("w4a4_e2m3_us") is not None else float("inf")
            fused4 = k["w4a4_fused_us"] if k.get("w4a4_fused_us") is not None else float("inf")
            choice.append("fused" if fused4 < min(nib, e2m3) else ("e2m3" if e2m3 < nib else "nibbles"))
        prepared = []
        for lin in layers:
            row = []
            for li, d in enumerate(lin):
                K = d["K"]
                s4 = (d["s_tok"] * (127.0 / 7.0)).contiguous()
                m = 1.0 / d["inv_m"]
                flat = d["xq"].view(torch.uint8).view(-1)
                if choice[li] == "e2m3":
                    wq6, s_w6, _ = ptq.fold_smoothing_w4_e2m3(d["w"], m)
                    nb = ptq.e2m3_blocks(K)
                    row.append(("e2m3", wq6, s_w6, s4, flat[: nb * M * 96].view(nb, M, 96)))
                else:
                    wq4, s_w4, _ = ptq.fold_smoothing_w4(d["w"], m)
                    row.append((choice[li], wq4, s_w4, s4, flat[: M * (K // 2)].view(M, K // 2)))
            prepared.append(row)

        def step_w4a4():
            for lin, row in zip(layers, prepared):
                for d, (kind, wq_, s_w_, s4, xq_) in zip(lin, row):
                    if kind == "e2m3":
                        ptq.quantize_pts_a4_e2m3(d["x"], d["inv_m"], s4, B, L, xq6=xq_)
                        ptq.w4a4_linear_e2m3(xq_, wq_, s4, s_w_, d["bias"], B, L, d["K"], y=d["y"])
                    elif kind == "fused":
                        ptq.w4a4_linear_fused(d["x"], d["inv_m"], s4, wq_, s_w_, d["bias"], B, L, y=d["y"])
                    else:
                        ptq.quantize_pts_a4(d["x"], d["inv_m"], s4, B, L, xq4=xq_)
                        ptq.w4a4_linear(xq_, wq_, s4, s_w_, d["bias"], B, L, y=d["y"])

        for _ in range(2):
            step_w4a4()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(1, args.steps // 2)):
            step_w4a4()
        torch.cuda.synchronize()
        result["w4a4_ms_per_step"] = (time.perf_counter() - t0) / max(1, args.steps // 2) * 1e3
        result["w4a4_containers"] = {k["linear"]: c for k, c in zip(kernels, choice)}
        del prepared

    # One plain device-to-device copy of known size (untimed): the reference against which the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE counters of the GEMM are scaled in profiles/.
    calib_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()
    del calib_src, calib_dst

    # ------------------------------------------------------------------ CPU oracle baseline (bounded sample)
    result["cpu"] = None
    if not args.no_cpu_baseline:
        import numpy as np

        import oracle

        sb = min(args.cpu_sample_batch, B)
        rows = sb * L
        lin0 = layers[0]
        host = [dict(x=d["x"][:rows].cpu().numpy(), w=d["w"].cpu().numpy(), bias=d["bias"].cpu().numpy(),
                     s_tok=d["s_tok"].cpu().numpy(), inv_m=d["inv_m"].cpu().numpy()) for d in lin0]
        folded = [oracle.fold_smoothing(h["w"], (np.float32(1) / h["inv_m"]).astype(np.float32)) for h in host]
        t0 = time.perf_counter()
        for h, (wq_o, s_w_o, _) in zip(host, folded):
            xq_o = oracle.quantize_pts(h["x"], h["inv_m"], h["s_tok"], sb, L)
            oracle.w8a8_linear(xq_o, wq_o, h["s_tok"], s_w_o, h["bias"], sb, L)
        cpu_s = time.perf_counter() - t0
        result["cpu"] = dict(value=round(rows / (cpu_s * n_layers), 2), unit="tokens/s", cores=oracle.threads(),
                             kind="oracle",
                             sample=f"layer 0, all four linears (quantize + int GEMM + dequantize), first {sb} of {B} "
                                    f"images ({rows} rows) in {cpu_s:.2f} s; extrapolated to {n_layers} layers")
    del layers, s_row
    torch.cuda.empty_cache()
    return result


def workload_text(r, fused_mode: str) -> str:
    cfg = r["cfg"]
    return (f"configs[{r['config']}] {cfg.name}: {r['n_layers']} layers x "
            f"{[f'{n} {k}->{o}' for n, k, o in cfg.linears]}, B={cfg.B}, L={cfg.L}, M={cfg.M}; "
            + (f"step = per layer PTS-quantize + W8A8-linear, one fused quantize+linear launch for {r['fused_linears']} "
               "(same codes and outputs, bit for bit); " if fused_mode == "auto" and r["fused_linears"]
               else "step = one PTS-quantize + one W8A8-linear launch per linear; ")
            + "fold offline")


def config_record(r, fused_mode: str):
    """The compact record of one configuration for the "configs" list."""
    cfg = r["cfg"]
    use_graph = r["config"] in GRAPH_HEADLINE_CONFIGS and r["graph_ms_per_step"] is not None
    head_ms = r["graph_ms_per_step"] if use_graph else r["ms_per_step"]
    keep = ("linear", "K", "N", "in_timed_step", "quantize_us", "quantize_GBps", "quantize_frac_hbm", "w8a8_us",
            "w8a8_TOPS", "w8a8_frac_int8_peak", "w8a8_GBps", "w8a8_frac_hbm", "fused_us", "fused_GBps", "fused_frac_hbm",
            "quantize_then_w8a8_us", "f16_us", "speedup_gemm_only", "speedup_quant_plus_gemm", "speedup_fused")
    return dict(config=r["config"], workload=workload_text(r, fused_mode),
                ms_per_step=round(head_ms, 4), timing="one HIP graph replay per step" if use_graph else "eager launches",
                eager_ms_per_step=round(r["ms_per_step"], 4),
                eager_ms_per_step_median=round(statistics.median(r["step_ms"]), 4),
                graph_ms_per_step=None if r["graph_ms_per_step"] is None else round(r["graph_ms_per_step"], 4),
                tokens_per_s=round(cfg.M / (head_ms * 1e-3), 1), tops=round(r["total_ops"] / (head_ms * 1e-3) / 1e12, 2),
                linears=[{k: rec[k] for k in keep if k in rec} for rec in r["kernels"]])


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="timed workload (BASELINE.json configs index)")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers of the timed workload (debug only)")
    ap.add_argument("--fused", choices=("auto", "off"), default="auto",
                    help="auto: one fused quantize+linear launch for linears with K <= 128 or N <= 128 when there are enough rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the extra timing of the step replayed as one HIP graph")
    ap.add_argument("--no-other-configs", action="store_true", help="time only the workload named by --config")
    ap.add_argument("--cpu-sample-batch", type=int, default=256)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards data-parallel over the batch "
              "with no collectives); run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2412_20386_amd as ptq
    from paper_2412_20386_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ptq.binding.load()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    r = measure_config(args, args.config, full=True)
    M = r["cfg"].M
    ms_per_step = r["ms_per_step"]

    # ------------------------------------------------------------------ roofline of the dominant kernel
    _, dK, dN = r["dominant"]
    dom_ops = 2.0 * M * dK * dN                     # algorithmic int8 ops per launch
    dom_all, dom_us = r["dom_all"], r["dom_us"]
    achieved = dom_ops / dom_us / 1e6               # TOP/s
    roofline = dict(bound="mfma", kernel=f"W8A8 GEMM of {r['dominant'][0]} {dK}->{dN}, M={M}",
                    achieved=round(achieved, 1), peak=PEAK_INT8_TOPS, unit="TOP/s",
                    frac=round(achieved / PEAK_INT8_TOPS, 4), avg_launch_us=round(dom_us, 2),
                    median_launch_us=round(dom_all[len(dom_all) // 2], 2), min_launch_us=round(dom_all[0], 2),
                    p90_launch_us=round(dom_all[min(len(dom_all) - 1, int(0.9 * len(dom_all)))], 2),
                    launches_timed=r["launches_timed"], traffic=dominant_traffic(args.config),
                    algorithmic_bytes=1.0 * M * dK + dN * dK + 2.0 * M * dN)

    configs = [config_record(r, args.fused)]
    if not args.no_other_configs:
        for other in sorted(synth.CONFIGS):
            if other != args.config:
                configs.append(config_record(measure_config(args, other, full=False), args.fused))
        configs.sort(key=lambda c: c["config"])

    tokens_per_s = M / (ms_per_step * 1e-3)
    # W4A4 (the precision of the paper's latency table, Sec. 6.4): sums of the kernel times measured above, per layer
    # quantizer + linear in the faster container of each linear (nibbles or E2M3) against quantizer + W8A8 linear.
    w4a4_sum = w8a8_sum = 0.0
    for k in r["kernels"]:
        pairs = [(k.get("a4_quantize_us"), k.get("w4a4_us")), (k.get("a4_e2m3_quantize_us"), k.get("w4a4_e2m3_us"))]
        pairs = [q + g for q, g in pairs if q is not None and g is not None]
        w4a4_sum = w4a4_sum + min(pairs) if (pairs and w4a4_sum is not None) else None
        w8a8_sum += k["quantize_us"] + k["w8a8_us"]
    out = {
        "metric": "W8A8 linear TOPS + tokens/sec, Vim-B shapes batch 256; speedup vs fp16 GEMM",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(statistics.median(r["step_ms"]), 4),
        "ms_per_step_max": round(max(r["step_ms"]), 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": workload_text(r, args.fused), "fused_linears": r["fused_linears"]},
        "tops": round(r["total_ops"] / (ms_per_step * 1e-3) / 1e12, 1),
        "speedup_vs_f16_stack": round(r["f16_ms_per_step"] / ms_per_step, 3),
        "f16_ms_per_step": round(r["f16_ms_per_step"], 4),
        "graph_ms_per_step": None if r["graph_ms_per_step"] is None else round(r["graph_ms_per_step"], 4),
        "dynamic_ms_per_step": round(r["dynamic_ms_per_step"], 4),
        "speedup_pts_vs_per_token_dynamic": round(r["dynamic_ms_per_step"] / ms_per_step, 3),
        "w4a4_ms_per_step": None if r.get("w4a4_ms_per_step") is None else round(r["w4a4_ms_per_step"], 4),
        "w4a4_containers": r.get("w4a4_containers"),
        "speedup_w4a4_vs_f16_stack": None if r.get("w4a4_ms_per_step") is None else round(r["f16_ms_per_step"] / r["w4a4_ms_per_step"], 3),
        "w4a4_two_launch_us_per_layer": None if w4a4_sum is None else round(w4a4_sum, 1),
        "w8a8_two_launch_us_per_layer": round(w8a8_sum, 1),
        "speedup_w4a4_vs_w8a8_kernel_sums": None if not w4a4_sum else round(w8a8_sum / w4a4_sum, 3),
        "paper_context": "paper: up to 1.83x end-to-end at W4A4 on VMamba-B, batch 32, RTX 3090 (not this metric)",
        "roofline": roofline,
        "cpu_baseline": r["cpu"],
        "kernels": r["kernels"],
        "configs": configs,
        "setup_s": round(r["setup_s"], 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
