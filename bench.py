#!/usr/bin/env python3
"""Throughput of the SnapKV prompt-KV compression step on one MI355X.

A step is one pass of the whole hot path (score -> vote -> pool -> top-k -> gather) over one batch of
synthetic input resident in HBM.  For the configuration the metric is quoted on (long_131k: 32 layers of
32 heads x 131072 tokens, 68.7 GB of K and V) the batch is the whole configuration: all layers resident,
one snapkv_compress_layers call per step.  `--mode single` times one snapkv_compress call per step
instead, cycling over a few resident layers so that no step finds its K/V in a cache left by the previous
one.  Prints ONE JSON line; `roofline.frac` is the whole path's algorithmic bytes over the step's time,
`roofline.kernel_frac` the dominant kernel's own, `configs` the other configurations.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload long_131k] [--mode auto|layers|single]
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_long_131k.txt")
KERNEL_SOURCES = ("snapkv_fused.hip", "snapkv_internal.h")   # what the dominant kernel is built from


def kernel_source_digest() -> str:
    """sha256 over the sources of the scoring kernel, as they are in this tree."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2404_14469_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of the scoring kernel from hardware counters (rocprofv3 --pmc FETCH_SIZE, then
    WRITE_SIZE, each scaled by what the same counter reads for a device copy of known size).  Counters
    cannot be read from inside a timed run: the figure comes from the committed counter summary, which
    names the workload, the kernel, the launch shape and the digest of the kernel sources it was measured
    on.  Anything else than an exact match gives None."""
    try:
        fields = {}
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if line.startswith("bench.") and ":" in line:
                    key, val = line.split(":", 1)
                    fields[key.strip()] = val.strip()
        if fields.get("bench.workload") != workload or fields.get("bench.kernel") != kernel:
            return None, "summary is for another workload or kernel"
        if fields.get("bench.kernel_source_sha256") != kernel_source_digest():
            return None, "kernel sources changed since the counters were read"
        return int(fields["bench.traffic_bytes_per_launch"]), fields.get("bench.launch", "")
    except (OSError, KeyError, ValueError) as e:
        return None, f"no usable counter summary ({e.__class__.__name__})"


def algorithmic_bytes(w):
    """Bytes the method must move per call: K once, the kept K/V rows read and written, the kept
    positions, the window queries.  V is never streamed, only gathered."""
    e = 4 if w.dtype == "f32" else 2
    scan = w.Hkv * w.L * w.D * e + w.Hq * w.W * w.D * e
    gather = w.Hkv * (4 * w.C * w.D * e + 4 * w.C)
    return scan, gather


def bench_decode(args, snapkv, workloads, w, dev) -> int:
    """A separate measurement (not the headline metric): one decoding step of attention over the
    compacted caches of a batch, snapkv_decode_attention.  A step is one layer's call; steps cycle
    over several resident layers.  Every valid K and V row is read once: those bytes over the
    call's duration (HIP events on the launch stream) give the roofline fraction."""
    import numpy as np
    import torch
    nres = max(1, args.resident_layers)
    layers = []
    for l in range(nres):
        c = workloads.generate_decode(dataclasses.replace(w, seed=w.seed + l), device=dev)
        layers.append((c["q"], c["k_cache"], c["v_cache"], c["lens"]))
    out = torch.empty((w.B, w.Hq, w.D), dtype=torch.float32, device=dev)
    lse = torch.empty((w.B, w.Hq), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def step(i):
        q, k, v, lens = layers[i % nres]
        snapkv.snapkv_decode_attention(q, k, v, w.S, out, lse, lens=lens, stream=stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i, (a, b) in enumerate(evs):
        a.record(stream)
        step(i)
        b.record(stream)
    torch.cuda.synchronize()
    call_ms = sorted(a.elapsed_time(b) for a, b in evs)[len(evs) // 2]
    rows = w.B * w.Hkv * w.S
    alg = 2 * rows * w.D * 2 + w.B * w.Hq * w.D * (2 + 4)
    achieved = alg / (call_ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import decode_oracle
        q, k, v, lens = layers[0]
        nb = max(1, min(w.B, int(2.0e9 // (w.Hq * w.S * w.D * 2))))
        qh, kh, vh = (workloads.to_numpy_bits(x[:nb]) for x in (q, k, v))
        c0 = time.perf_counter()
        want, _ = decode_oracle.decode_attention(qh, kh, vh, lens=w.S)
        secs = time.perf_counter() - c0
        step(0)
        torch.cuda.synchronize()
        err = float(np.abs(out[:nb].cpu().numpy() - want).max())
        cpu = {"value": round(nb * w.Hkv * w.S / secs, 1), "unit": "KV-head-rows/s", "cores": 1, "kind": "oracle",
               "sample": f"sequences 0..{nb - 1} of layer 0 ({nb * w.Hkv * w.S} rows), numpy fp64 oracle, {secs:.2f} s wall",
               "max_abs_err_vs_oracle": err}
    print(json.dumps({
        "metric": "decode attention: cached KV rows read/sec per GPU", "value": round(rows / (ms_per_step * 1e-3), 1),
        "unit": "KV-head-rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "S": w.S, "cap": w.cap,
                   "step": "one layer call", "resident_layers": nres},
        "roofline": {"bound": "hbm", "kernel": "decode_attn(+decode_merge)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": alg, "kernel_ms": round(call_ms, 4)},
        "cpu_baseline": cpu}))
    return 0


def bench_varlen(args, snapkv, workloads, dev) -> int:
    """A separate measurement: the batched-varlen configuration (eight prompts of 4K-64K tokens of one GQA
    model) through snapkv_compress_varlen; a step is one batch."""
    import numpy as np
    import torch
    ws = workloads.varlen_prompts()
    cases = [workloads.generate(w, device=dev) for w in ws]
    w0 = ws[0]
    qs, ks, vs = [c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases]
    oks = [torch.empty((w0.Hkv, w0.C, w0.D), dtype=ks[0].dtype, device=dev) for _ in ws]
    ovs = [torch.empty_like(t) for t in oks]
    ois = [torch.empty((w0.Hkv, w0.C), dtype=torch.int32, device=dev) for _ in ws]
    stream = torch.cuda.current_stream()

    def step(_):
        snapkv.snapkv_compress_varlen(qs, ks, vs, w0.pool_kind, w0.p, w0.C, oks, ovs, ois, stream=stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    snapkv.snapkv_profile_start(args.steps)
    for i in range(args.steps):
        step(i)
    stage_ms, _ = snapkv.snapkv_profile_stop()
    stage_ms = {n: v for n, v in stage_ms.items() if v > 0.0}
    positions = sum(w.Hkv * w.L for w in ws)
    e = 2
    scan = sum(w.Hkv * w.L * w.D * e + w.Hq * w.W * w.D * e for w in ws)
    gather = sum(w.Hkv * (4 * w.C * w.D * e + 4 * w.C) for w in ws)
    score_ms = stage_ms.get("score_fused", 0.0)
    kernel_achieved = scan / (score_ms * 1e-3) / 1e9 if score_ms > 0 else 0.0
    achieved = (scan + gather) / (ms_per_step * 1e-3) / 1e9      # the whole path over the step's time
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import c_oracle
        secs, npos, same = 0.0, 0, 0.0
        for i in (1, 2):                                  # two of the shorter prompts: a bounded sample
            w, c = ws[i], cases[i]
            qh, kh, vh = (workloads.to_numpy_bits(x) for x in (c["q_win"], c["k"], c["v"]))
            c0 = time.perf_counter()
            _, _, oidx, _, _ = c_oracle.compress(qh, kh, vh, w.W, w.pool_kind, w.p, w.C)
            secs += time.perf_counter() - c0
            npos += w.Hkv * w.L
            same += float((ois[i].cpu().numpy() == oidx).mean())
        cpu = {"value": round(npos / secs, 1), "unit": "KV-head-positions/s", "cores": c_oracle.threads(), "kind": "oracle",
               "sample": f"prompts 1 and 2 of the batch ({npos} positions), plain-C fp64 oracle, {secs:.2f} s wall",
               "kept_positions_identical_frac": round(same / 2, 6)}
    print(json.dumps({
        "metric": "prompt KV positions compressed/sec per GPU", "value": round(positions / (ms_per_step * 1e-3), 1),
        "unit": "KV-head-positions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w0.dtype, "data": "synthetic",
        "config": {"workload": "varlen", "prompts": len(ws), "L": [w.L for w in ws], "Hq": w0.Hq, "Hkv": w0.Hkv, "D": w0.D,
                   "W": w0.W, "pool": "avg", "p": w0.p, "C": w0.C, "step": "one batch call", "entry": "compress_varlen"},
        "roofline": {"bound": "hbm", "kernel": "score_fused_joint (the prompts share launches of the single-read kernel, longest first)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "path_algorithmic_bytes": scan + gather,
                     "algorithmic_bytes_per_launch": scan, "kernel_ms": round(score_ms, 4),
                     "kernel_achieved": round(kernel_achieved, 1), "kernel_frac": round(kernel_achieved / HBM_PEAK_GBS, 4),
                     "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()}},
        "cpu_baseline": cpu}))
    return 0


def band_parity(np, w, scores, oracle_idx, gpu_idx):
    """The parity bar on kept positions, as a summary: with T the oracle's (C-W)-th largest score of a
    head, every position scoring above T(1+1e-3) must be kept and none below T(1-1e-3) may be; in between
    either is right.  Returns (violations, positions inside the band, share of positions identical)."""
    kc = w.C - w.W
    n = w.L - w.W
    viol = band = 0
    for h in range(scores.shape[0]):
        s = scores[h]
        T = np.partition(s, n - kc)[n - kc]
        keep = s > T * (1 + 1e-3)
        drop = s < T * (1 - 1e-3)
        chosen = np.zeros(n, dtype=bool)
        chosen[gpu_idx[h, :kc]] = True
        viol += int((keep & ~chosen).sum() + (drop & chosen).sum())
        band += int(n - keep.sum() - drop.sum())
    return viol, band, float((gpu_idx == oracle_idx).mean())


def oracle_leg(np, workloads, c_oracle, w, layer_inputs, gpu_idx_of, budget=1.5e11):
    """The plain-C fp64 oracle timed on whole layers of the workload until about `budget` multiply-adds of
    the scoring product are spent; parity of the GPU's kept positions on every layer it ran."""
    per_layer = float(w.Hq) * w.W * w.L * w.D
    nlay = max(1, min(len(layer_inputs), int(budget // per_layer)))
    secs, npos, viol, band, same = 0.0, 0, 0, 0, 0.0
    for l in range(nlay):
        q, k, v = layer_inputs[l]
        qh, kh, vh = (workloads.to_numpy_bits(x) for x in (q, k, v))
        c0 = time.perf_counter()
        _, _, oidx, _, score = c_oracle.compress(qh, kh, vh, w.W, w.pool_kind, w.p, w.C)
        secs += time.perf_counter() - c0
        a, b, c = band_parity(np, w, score, oidx, gpu_idx_of(l))
        viol, band, same = viol + a, band + b, same + c
        npos += w.Hkv * w.L
    return {"value": round(npos / secs, 1), "unit": "KV-head-positions/s", "cores": c_oracle.threads(), "kind": "oracle",
            "sample": f"layers 0..{nlay - 1} of the workload, all {w.Hkv} KV heads ({npos} positions), "
                      f"plain-C fp64 oracle, {secs:.2f} s wall",
            "kept_positions_identical_frac": round(same / nlay, 6),
            "kept_positions_outside_tolerance": viol, "positions_inside_tolerance_band": band}


def time_steps(torch, step, steps, warmup):
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def run_layers(torch, snapkv, workloads, w, nlay, steps, warmup, dev, stages=True, separate=False):
    """All `nlay` layers resident, as stacked tensors or (separate) with q_win, k and v of every layer an
    allocation of its own; a step is one snapkv_compress_layers call over them."""
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[w.dtype]
    needles = []
    if separate:
        Q, K, V, gaps = [], [], [], []
        for l in range(nlay):
            c = workloads.generate(w, layer=l, device=dev)
            Q.append(c["q_win"]), K.append(c["k"]), V.append(c["v"])
            gaps.append(torch.empty(4096 + 512 * l, dtype=torch.uint8, device=dev))   # keeps the allocations apart
            needles.append(c["needle_pos"])
    else:
        K = torch.empty((nlay, w.Hkv, w.L, w.D), device=dev, dtype=tdt)
        V = torch.empty_like(K)
        Q = torch.empty((nlay, w.Hq, w.W, w.D), device=dev, dtype=tdt)
        for l in range(nlay):
            c = workloads.generate(w, layer=l, device=dev)
            K[l].copy_(c["k"])
            V[l].copy_(c["v"])
            Q[l].copy_(c["q_win"])
            needles.append(c["needle_pos"])
            del c
    ok = torch.empty((nlay, w.Hkv, w.C, w.D), dtype=tdt, device=dev)
    ov = torch.empty_like(ok)
    oi = torch.full((nlay, w.Hkv, w.C), -1, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    lists = [list(t) for t in (Q, K, V, ok, ov, oi)]

    def step(_):
        snapkv.snapkv_compress_layers(lists[0], lists[1], lists[2], w.pool_kind, w.p, w.C, lists[3], lists[4], lists[5],
                                      stream=stream)

    ms = time_steps(torch, step, steps, warmup)
    stage_ms = {}
    launches_per_step = 1.0
    if stages:
        # a step is one call of the entry, which may cut its layers into several runs of launches (its scratch is
        # capped): the stage times are per step, i.e. summed over the runs
        snapkv.snapkv_profile_start(min(4096, max(1, steps) * 64))
        for i in range(steps):
            step(i)
        stage_ms, ncalls = snapkv.snapkv_profile_stop()
        launches_per_step = ncalls / max(1, steps)
        stage_ms = {n: v * launches_per_step for n, v in stage_ms.items() if v > 0.0}
    torch.cuda.synchronize()
    return {"ms": ms, "stage_ms": stage_ms, "Q": Q, "K": K, "V": V, "oi": oi, "needles": needles, "step": step,
            "launches_per_step": launches_per_step}


def run_single(torch, snapkv, workloads, w, nres, steps, warmup, dev, stages=True):
    """`nres` distinct layers resident; a step is one snapkv_compress call, steps cycle over the layers."""
    layers = []
    for l in range(nres):
        c = workloads.generate(w, layer=l, device=dev)
        layers.append((c["q_win"], c["k"], c["v"]))
    out_k = torch.empty((w.Hkv, w.C, w.D), dtype=layers[0][1].dtype, device=dev)
    out_v = torch.empty_like(out_k)
    out_idx = torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()

    def step(i):
        q, k, v = layers[i % nres]
        snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, stream=stream)

    ms = time_steps(torch, step, steps, warmup)
    stage_ms = {}
    if stages:
        snapkv.snapkv_profile_start(max(1, steps))
        for i in range(steps):
            step(i)
        stage_ms, _ = snapkv.snapkv_profile_stop()
        stage_ms = {n: v for n, v in stage_ms.items() if v > 0.0}
    torch.cuda.synchronize()
    return {"ms": ms, "stage_ms": stage_ms, "layers": layers, "out_idx": out_idx, "step": step}


def config_lines(args, torch, np, snapkv, workloads, dev):
    """The other configurations, each with its GPU time per call (and per layer where the layers of a model
    run in one call), the whole path's share of the HBM peak, the oracle's rate on a bounded sample and the
    parity of the kept positions on that sample."""
    from oracle import c_oracle
    out = []

    def entry(w, step_name, ms, layers_per_step, cpu):
        scan_b, gather_b = algorithmic_bytes(w)
        per_layer_ms = ms / layers_per_step
        return {"workload": w.name, "step": step_name, "ms_per_step": round(ms, 4), "layers_per_step": layers_per_step,
                "ms_per_layer": round(per_layer_ms, 4),
                "value": round(w.Hkv * w.L / (per_layer_ms * 1e-3), 1), "unit": "KV-head-positions/s",
                "frac": round((scan_b + gather_b) / (per_layer_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "cpu_baseline": cpu}

    steps, warmup = 20, 3
    for name in ("tiny", "llama2_7b_16k"):
        w = workloads.CONFIGS[name]
        r = run_single(torch, snapkv, workloads, w, 4, steps, warmup, dev, stages=False)

        def gpu_idx(l, r=r):
            r["step"](l)
            torch.cuda.synchronize()
            return r["out_idx"].cpu().numpy()

        cpu = None if args.no_cpu_baseline else oracle_leg(np, workloads, c_oracle, w, r["layers"], gpu_idx, budget=3e10)
        out.append(entry(w, "one layer, one snapkv_compress call", r["ms"], 1, cpu))
        del r
    w = workloads.CONFIGS["mistral_7b_gqa_32k"]
    r1 = run_single(torch, snapkv, workloads, w, 4, steps, warmup, dev, stages=False)
    out.append(entry(w, "one layer, one snapkv_compress call", r1["ms"], 1, None))
    del r1
    r = run_layers(torch, snapkv, workloads, w, w.layers, 6, 2, dev, stages=False)
    cpu = None
    if not args.no_cpu_baseline:
        idx = r["oi"].cpu().numpy()
        cpu = oracle_leg(np, workloads, c_oracle, w, [(r["Q"][l], r["K"][l], r["V"][l]) for l in range(2)],
                         lambda l: idx[l], budget=3e10)
    out.append(entry(w, f"{w.layers} layers, one snapkv_compress_layers call", r["ms"], w.layers, cpu))
    del r
    w = workloads.CONFIGS["long_131k"]
    r1 = run_single(torch, snapkv, workloads, w, 4, steps, warmup, dev, stages=False)
    out.append(entry(w, "one layer, one snapkv_compress call", r1["ms"], 1, None))
    del r1
    # beyond the five configurations: the longest context the paper reports (Sec. 5.1.1: 380K tokens, C = 1024,
    # max pooling over 5, W = 16), at the long-context configuration's heads; longer than the single-read kernel holds
    w = workloads.CONFIGS["long_131k"].with_(name="long_380k", L=380000, W=16, p=5, C=1024, layers=1)
    r = run_single(torch, snapkv, workloads, w, 2, 10, 2, dev, stages=False)

    def gpu_idx_380(l, r=r):
        r["step"](l)
        torch.cuda.synchronize()
        return r["out_idx"].cpu().numpy()

    cpu = None if args.no_cpu_baseline else oracle_leg(np, workloads, c_oracle, w, r["layers"], gpu_idx_380, budget=3e10)
    out.append(entry(w, "one layer, one snapkv_compress call", r["ms"], 1, cpu))
    del r
    # the batch of eight prompts of different lengths
    ws = workloads.varlen_prompts()
    cases = [workloads.generate(x, device=dev) for x in ws]
    w0 = ws[0]
    qs, ks, vs = [c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases]
    oks = [torch.empty((w0.Hkv, w0.C, w0.D), dtype=ks[0].dtype, device=dev) for _ in ws]
    ovs = [torch.empty_like(t) for t in oks]
    ois = [torch.empty((w0.Hkv, w0.C), dtype=torch.int32, device=dev) for _ in ws]
    stream = torch.cuda.current_stream()
    ms = time_steps(torch, lambda _: snapkv.snapkv_compress_varlen(qs, ks, vs, w0.pool_kind, w0.p, w0.C, oks, ovs, ois,
                                                                   stream=stream), steps, warmup)
    e = 2
    pos = sum(x.Hkv * x.L for x in ws)
    alg = sum(x.Hkv * x.L * x.D * e + x.Hq * x.W * x.D * e + x.Hkv * (4 * x.C * x.D * e + 4 * x.C) for x in ws)
    cpu = None
    if not args.no_cpu_baseline:
        secs, npos, viol, band, same = 0.0, 0, 0, 0, 0.0
        for i in (1, 2):
            x, c = ws[i], cases[i]
            qh, kh, vh = (workloads.to_numpy_bits(t) for t in (c["q_win"], c["k"], c["v"]))
            c0 = time.perf_counter()
            _, _, oidx, _, score = c_oracle.compress(qh, kh, vh, x.W, x.pool_kind, x.p, x.C)
            secs += time.perf_counter() - c0
            a, b, cc = band_parity(np, x, score, oidx, ois[i].cpu().numpy())
            viol, band, same, npos = viol + a, band + b, same + cc, npos + x.Hkv * x.L
        cpu = {"value": round(npos / secs, 1), "unit": "KV-head-positions/s", "cores": c_oracle.threads(), "kind": "oracle",
               "sample": f"prompts 1 and 2 of the batch ({npos} positions), plain-C fp64 oracle, {secs:.2f} s wall",
               "kept_positions_identical_frac": round(same / 2, 6), "kept_positions_outside_tolerance": viol,
               "positions_inside_tolerance_band": band}
    out.append({"workload": "varlen", "step": "one batch of 8 prompts, one snapkv_compress_varlen call",
                "L": [x.L for x in ws], "ms_per_step": round(ms, 4), "value": round(pos / (ms * 1e-3), 1),
                "unit": "KV-head-positions/s", "frac": round(alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "cpu_baseline": cpu})
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="long_131k",
                    help="long_131k (default, the configuration the metric is quoted on), "
                         "llama2_7b_16k, mistral_7b_gqa_32k, tiny; decode_capped_b8 and decode_full_16k_b2 "
                         "time the decoding step over the cache instead; varlen times the batched-varlen configuration "
                         "through snapkv_compress_varlen (separate measurements)")
    ap.add_argument("--mode", default="auto", choices=["auto", "layers", "single"],
                    help="layers: all layers of the workload resident, a step is ONE snapkv_compress_layers call over them "
                         "(auto picks this for workloads of several layers with the default entry and layout); "
                         "single: a step is one snapkv_compress call on one layer, steps cycle over the resident layers")
    ap.add_argument("--resident-layers", type=int, default=0,
                    help="layers kept in HBM (default: all layers of the workload in layers mode, 4 in single mode)")
    ap.add_argument("--separate-layers", action="store_true",
                    help="layers mode: q_win, k and v of every layer are allocations of their own instead of slices of "
                         "stacked tensors (the call then reaches them through its table of layer addresses)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="leave out the other configurations' lines (`configs`)")
    ap.add_argument("--scheme", type=int, default=0,
                    help="kernel scheme bits for measurements (see snapkv_set_scoring_scheme); 0 = default")
    ap.add_argument("--entry", default="compress", choices=["compress", "lse", "per_query_head"],
                    help="compress (default): snapkv_compress, the headline path; lse: snapkv_compress_lse, "
                         "the variant that is handed the window rows' log-sum-exp; per_query_head: "
                         "snapkv_compress_per_query_head, one cache per query head (separate measurements)")
    ap.add_argument("--layout", default="head_major", choices=["head_major", "token_major", "paged"],
                    help="storage order of K/V: [Hkv, L, D] (default), [L, Hkv, D] through snapkv_compress_strided, or pages "
                         "[num_pages, 16, Hkv, D] behind a shuffled block table through snapkv_compress_paged")
    ap.add_argument("--window", type=int, default=0, metavar="W",
                    help="override the workload's observation window (e.g. 64 with --pool-width 13: the setting the "
                         "paper uses for Command-R; a separate measurement, named in config)")
    ap.add_argument("--pool-width", type=int, default=0, metavar="P", help="override the workload's pooling kernel size")
    ap.add_argument("--length", type=int, default=0, metavar="L",
                    help="override the workload's prompt length (e.g. the grouped-query configuration at 131072 tokens)")
    ap.add_argument("--capacity", type=int, default=0, metavar="C",
                    help="override the workload's cache capacity (e.g. --length 380000 --window 16 --pool-width 5 --capacity "
                         "1024: the 380K-token setting of Sec. 5.1.1)")
    ap.add_argument("--explicit-workspace", action="store_true",
                    help="time snapkv_compress_ws with a caller-provided workspace instead of snapkv_compress")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="run only a plain device copy of MIB mebibytes (8 launches) and exit: the "
                         "known-size kernel the HBM traffic counters are calibrated on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (heads, layers and prompts are independent; "
              "no multi-GPU path exists) - run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2404_14469_amd as snapkv
    from paper_2404_14469_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_probe > 0:
        src = torch.full((args.copy_probe << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel(), "copy_probe_bytes_written": dst.numel(),
                          "launches": 8}))
        return 0
    snapkv.load()
    if args.scheme:
        snapkv.snapkv_set_scoring_scheme(args.scheme)
    if args.workload == "varlen":
        return bench_varlen(args, snapkv, workloads, dev)
    if args.workload in workloads.DECODE_CONFIGS:
        return bench_decode(args, snapkv, workloads, workloads.DECODE_CONFIGS[args.workload], dev)
    w = workloads.CONFIGS[args.workload]
    if args.window or args.pool_width or args.length or args.capacity:
        w = w.with_(W=args.window or w.W, p=args.pool_width or w.p, L=args.length or w.L, C=args.capacity or w.C)
    plain = args.entry == "compress" and args.layout == "head_major" and not args.explicit_workspace
    mode = args.mode
    if mode == "auto":
        mode = "layers" if (w.layers > 1 and plain) else "single"
    if mode == "layers":
        if not plain:
            print("bench.py: --mode layers times snapkv_compress_layers on head-major K/V", file=sys.stderr)
            return 2
        return bench_layers(args, torch, np, snapkv, workloads, w, dev)

    nres = max(1, args.resident_layers or 4)
    if w.layers <= 1:
        nres = max(1, args.resident_layers or 4)
    layers = []
    for l in range(nres):
        c = workloads.generate(w, layer=l, device=dev)
        if args.layout == "token_major":
            c["k"] = c["k"].permute(1, 0, 2).contiguous().permute(1, 0, 2)
            c["v"] = c["v"].permute(1, 0, 2).contiguous().permute(1, 0, 2)
        if args.layout == "paged":      # scatter into 16-row pages in a shuffled order (input preparation)
            ps = 16
            npg = (w.L + ps - 1) // ps
            gen = torch.Generator().manual_seed(l)
            table = torch.randperm(npg, generator=gen).to(torch.int32).to(dev)
            pos = torch.arange(w.L, device=dev)
            pages = []
            for name in ("k", "v"):
                pg = torch.zeros((npg, ps, w.Hkv, w.D), dtype=c[name].dtype, device=dev)
                pg[table.long()[pos // ps], pos % ps] = c[name].permute(1, 0, 2)
                pages.append(pg)
            c["k"], c["v"], c["table"] = pages[0], pages[1], table
            layers.append((c["q_win"], c["k"], c["v"], c["table"]))
            continue
        layers.append((c["q_win"], c["k"], c["v"]))
    torch.cuda.synchronize()
    hout = w.Hq if args.entry == "per_query_head" else w.Hkv
    out_k = torch.empty((hout, w.C, w.D), dtype=layers[0][1].dtype, device=dev)
    out_v = torch.empty_like(out_k)
    out_idx = torch.empty((hout, w.C), dtype=torch.int32, device=dev)
    ws = None
    if args.explicit_workspace:
        ws = torch.empty(snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    lses = None
    if args.entry == "lse":
        # inputs of that entry point: the rows' log-sum-exp, here from plain torch ops on the GPU
        # (input preparation outside the timed region; the parity tests take it from the oracle)
        lses = []
        for q, k, v in layers:
            g = w.Hq // w.Hkv
            kk = k.float().repeat_interleave(g, dim=0)
            s_ = torch.einsum("hwd,hld->hwl", q.float(), kk) / (w.D ** 0.5)
            jj = torch.arange(w.L, device=dev)[None, None, :]
            ii = torch.arange(w.W, device=dev)[None, :, None]
            s_ = s_.masked_fill(jj > (w.L - w.W) + ii, float("-inf"))
            lses.append(torch.logsumexp(s_.double(), dim=2).float().contiguous())
            del kk, s_
        torch.cuda.synchronize()

    def step(i):
        if args.layout == "paged":
            q, kp, vp, table = layers[i % nres]
            snapkv.snapkv_compress_paged(q, kp, vp, table, w.L, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, stream=stream)
            return
        q, k, v = layers[i % nres]
        if args.layout == "token_major":
            snapkv.snapkv_compress_strided(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, stream=stream)
            return
        if args.entry == "per_query_head":
            snapkv.snapkv_compress_per_query_head(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, stream=stream)
            return
        if lses is not None:
            snapkv.snapkv_compress_lse(q, k, v, lses[i % nres], w.pool_kind, w.p, w.C, out_k, out_v, out_idx,
                                       stream=stream)
            return
        snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, stream=stream,
                               workspace=ws)

    ms_per_step = time_steps(torch, step, args.steps, args.warmup)
    positions = w.Hkv * w.L
    value = positions / (ms_per_step * 1e-3)

    # per-kernel durations from HIP events recorded by the library on the same stream
    snapkv.snapkv_profile_start(args.steps)
    for i in range(args.steps):
        step(i)
    stage_ms, ncalls = snapkv.snapkv_profile_stop()
    if snapkv.snapkv_sync_timeouts() != 0:
        print("bench.py: a bounded wait inside a kernel gave up during the timed calls", file=sys.stderr)
        return 1

    scan_b, gather_b = algorithmic_bytes(w)
    stage_ms = {n: v for n, v in stage_ms.items() if v > 0.0}      # stages this workload ran
    score_names = [n for n in stage_ms if n.startswith("score")]
    score_ms = sum(stage_ms[n] for n in score_names)
    kernel_achieved = scan_b / (score_ms * 1e-3) / 1e9 if score_ms > 0 else 0.0
    path_achieved = (scan_b + gather_b) / (ms_per_step * 1e-3) / 1e9
    roofline = {
        "bound": "hbm",
        # the whole path: algorithmic bytes of a call over the time of a call
        "achieved": round(path_achieved, 1),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(path_achieved / HBM_PEAK_GBS, 4),
        "traffic": None,
        "path_algorithmic_bytes": scan_b + gather_b,
        # the dominant kernel alone: its algorithmic bytes (K once, window queries) over its mean duration
        "kernel": "+".join(score_names).replace("score_fused", "score_lse" if args.entry == "lse" else "score_fused"),
        "kernel_ms": round(score_ms, 4),
        "algorithmic_bytes_per_launch": scan_b,
        "kernel_achieved": round(kernel_achieved, 1),
        "kernel_frac": round(kernel_achieved / HBM_PEAK_GBS, 4),
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        # evidence beside the bound: the scoring product's MFMA rate and the exponentials per second
        "mfma_tflops": round(2.0 * w.Hq * w.W * w.L * w.D / (score_ms * 1e-3) / 1e12, 1) if score_ms > 0 else None,
        "exp_per_s": round(float(w.Hq) * w.W * w.L / (score_ms * 1e-3), 1) if score_ms > 0 else None,
    }

    cpu = None
    if not args.no_cpu_baseline and args.entry != "per_query_head" and args.layout != "paged":
        from oracle import c_oracle

        def gpu_idx(l):
            step(l)
            torch.cuda.synchronize()
            return out_idx.cpu().numpy()

        cpu = oracle_leg(np, workloads, c_oracle, w, [x[:3] for x in layers], gpu_idx)
        if cpu["kept_positions_outside_tolerance"] != 0:
            print("bench.py: kept positions disagree with the oracle outside the tolerance band", file=sys.stderr)
            return 1

    line = {
        "metric": "prompt KV positions compressed/sec per GPU",
        "value": round(value, 1),
        "unit": "KV-head-positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "L": w.L, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "W": w.W,
                   "pool": ("max" if w.pool_kind == 0 else "avg"), "p": w.p, "C": w.C,
                   "step": "one layer, one call", "layers_per_step": 1, "entry": args.entry, "layout": args.layout,
                   "resident_layers": nres, "scheme": args.scheme,
                   "token_layers_per_s": round(w.L / (ms_per_step * 1e-3), 1)},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


def bench_layers(args, torch, np, snapkv, workloads, w, dev) -> int:
    """The headline measurement: every layer of the workload resident in HBM (68.7 GB of K and V at the
    long-context configuration), a step is ONE snapkv_compress_layers call that runs the whole hot path
    (score -> vote -> pool -> top-k -> gather) over all of them."""
    nlay = max(1, args.resident_layers or w.layers)
    r = run_layers(torch, snapkv, workloads, w, nlay, args.steps, args.warmup, dev, separate=args.separate_layers)
    if snapkv.snapkv_sync_timeouts() != 0:
        print("bench.py: a bounded wait inside a kernel gave up during the timed calls", file=sys.stderr)
        return 1
    ms_per_step = r["ms"]
    r_runs = round(r["launches_per_step"], 2)
    ms_per_layer = ms_per_step / nlay
    positions = nlay * w.Hkv * w.L
    value = positions / (ms_per_step * 1e-3)
    scan_b, gather_b = algorithmic_bytes(w)
    stage_ms = r["stage_ms"]
    score_names = [n for n in stage_ms if n.startswith("score")]
    score_ms = sum(stage_ms[n] for n in score_names)          # one launch per call: all layers' keys
    kernel_achieved = nlay * scan_b / (score_ms * 1e-3) / 1e9 if score_ms > 0 else 0.0
    path_achieved = nlay * (scan_b + gather_b) / (ms_per_step * 1e-3) / 1e9
    kernel = "+".join(score_names)
    traffic, traffic_note = (None, "not looked up")
    if nlay == w.layers and args.scheme == 0 and not args.separate_layers and r_runs == 1:
        traffic, traffic_note = measured_traffic(w.name, kernel)
    roofline = {
        "bound": "hbm",
        # the whole path: algorithmic bytes of a step over the time of a step
        "achieved": round(path_achieved, 1),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(path_achieved / HBM_PEAK_GBS, 4),
        # HBM bytes per launch of the dominant kernel from hardware counters, or null (see traffic_note)
        "traffic": traffic,
        "traffic_note": traffic_note,
        "path_algorithmic_bytes": nlay * (scan_b + gather_b),
        # the dominant kernel alone: its algorithmic bytes (every layer's K once, the window queries) over
        # its mean duration (HIP events the library records on the launch stream)
        "kernel": kernel,
        "kernel_ms": round(score_ms, 4),
        "algorithmic_bytes_per_launch": nlay * scan_b,
        "kernel_achieved": round(kernel_achieved, 1),
        "kernel_frac": round(kernel_achieved / HBM_PEAK_GBS, 4),
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "mfma_tflops": round(2.0 * nlay * w.Hq * w.W * w.L * w.D / (score_ms * 1e-3) / 1e12, 1) if score_ms > 0 else None,
        "exp_per_s": round(float(nlay) * w.Hq * w.W * w.L / (score_ms * 1e-3), 1) if score_ms > 0 else None,
    }
    idx = r["oi"].cpu().numpy()
    # the planted needle of the long-context workload and its neighbours within the pooling reach must be kept
    needle_kept = None
    if w.needle:
        needle_kept = True
        for l in range(nlay):
            for hk, pos in enumerate(r["needles"][l]):
                lo, hi = max(0, pos - w.p // 2), min(w.n - 1, pos + w.p // 2)
                have = set(idx[l, hk].tolist())
                needle_kept = needle_kept and all(j in have for j in range(lo, hi + 1))
        if not needle_kept:
            print("bench.py: a planted needle was not kept", file=sys.stderr)
            return 1
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import c_oracle
        cpu = oracle_leg(np, workloads, c_oracle, w, [(r["Q"][l], r["K"][l], r["V"][l]) for l in range(nlay)],
                         lambda l: idx[l])
        if cpu["kept_positions_outside_tolerance"] != 0:
            print("bench.py: kept positions disagree with the oracle outside the tolerance band", file=sys.stderr)
            return 1
    del r
    configs = None
    if not args.no_configs:
        torch.cuda.empty_cache()
        configs = config_lines(args, torch, np, snapkv, workloads, dev)
        if snapkv.snapkv_sync_timeouts() != 0:
            print("bench.py: a bounded wait inside a kernel gave up", file=sys.stderr)
            return 1
    line = {
        "metric": "prompt KV positions compressed/sec per GPU",
        "value": round(value, 1),
        "unit": "KV-head-positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "L": w.L, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "W": w.W,
                   "pool": ("max" if w.pool_kind == 0 else "avg"), "p": w.p, "C": w.C,
                   "step": f"{nlay} layers, one snapkv_compress_layers call", "layers_per_step": nlay,
                   "ms_per_layer": round(ms_per_layer, 4), "entry": "compress_layers", "layout": "head_major",
                   "layer_tensors": "separate allocations" if args.separate_layers else "stacked",
                   "resident_layers": nlay, "resident_kv_bytes": 2 * nlay * w.Hkv * w.L * w.D * 2, "scheme": args.scheme,
                   "runs_of_launches_per_step": r_runs,
                   "needle_kept": needle_kept, "token_layers_per_s": round(nlay * w.L / (ms_per_step * 1e-3), 1)},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "configs": configs,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
