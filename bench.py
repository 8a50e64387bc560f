#!/usr/bin/env python3
"""Benchmark of the A2SF hot path on one MI355X.

One "step" of this benchmark is one pass of the whole path over one batch of synthetic
input: the prompt phase (masked attention + forgotten scores + selection + gather into the
cache) followed by the workload's T generation steps (attention over the retained tokens,
score update, eviction).  Inputs are resident in HBM before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

Prints ONE JSON line.  `value` is generation steps per second (one generation step = one
a2sf_decode_step call covering all G heads), measured with HIP events on the launch stream
over every generation step of the K timed passes.  The roofline objects relate the two
heavy kernels to the machine: the fused decode kernel to the HBM peak, the prompt-phase
attention to the dense bf16 matrix-core peak.  `cpu_baseline` is the float64 oracle timed
on the host cores of this machine on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for _p in (ROOT, os.path.join(ROOT, "tests")):
    if _p not in sys.path:
        sys.path.insert(0, _p)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def decode_bytes_per_step(G, L, d, e):
    """Algorithmic bytes of one generation step: K and V rows read once, scores read and
    written, q read, o written, the new k/v rows written."""
    return G * (2 * L * d * e + 8 * L + 4 * d * e)


def prefill_model_flops(G, n, d, with_o=True):
    """One causal QK^T sweep (2 flop per MAC over the lower triangle incl. diagonal), plus one
    PV sweep when outputs are requested.  The score kernel's recomputation is not counted."""
    one = d * n * (n + 1)
    return G * one * (2 if with_o else 1)


TRAFFIC_FILE = os.path.join("profiles", "traffic.txt")


def read_traffic(name):
    """HBM bytes per launch as recorded in profiles/traffic.txt from two earlier `rocprofv3 --pmc`
    runs of this benchmark (FETCH_SIZE, then WRITE_SIZE, scaled by a 1 GiB copy).  Counters
    cannot be collected inside a timed run, so the figure is provenance, not a live measurement;
    the JSON line says so in `traffic_source`."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == name:
            return float(parts[1])
    return None


def similarity_kernel(spec):
    """`--similarity-kernel HEADSxROWS`: time of one a2sf_ideal_similarity call over rows of that
    length against its algorithmic bytes (the keys, read once)."""
    import torch

    import paper_2407_20485_amd as a2sf
    G, L = (int(x) for x in spec.lower().split("x"))
    d, cached, reps = 128, 200, 20
    k = torch.randn((G, L, d), device="cuda").to(torch.bfloat16)
    q = torch.randn((G, d), device="cuda").to(torch.bfloat16)
    cache = a2sf.Cache(G, cached + 1, d, torch.bfloat16)
    cache.len.fill_(min(cached, L - 1))
    cache.pos.copy_(torch.arange(cached + 1, dtype=torch.int32, device="cuda").expand(G, -1) % max(L - 1, 1))
    out = torch.empty(G, dtype=torch.float32, device="cuda")
    for _ in range(3):
        a2sf.a2sf_ideal_similarity(q, k, L, L - 1, cache, out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        a2sf.a2sf_ideal_similarity(q, k, L, L - 1, cache, out)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    nbytes = G * L * d * 2
    print(json.dumps({"kernel": "a2sf_ideal_similarity", "heads": G, "rows": L, "head_dim": d, "dtype": "bf16",
                      "us_per_call": us, "bytes_per_call": nbytes,
                      "roofline": {"bound": "hbm", "achieved": nbytes / us / 1e3, "peak": HBM_PEAK_GBS,
                                   "unit": "GB/s", "frac": nbytes / us / 1e3 / HBM_PEAK_GBS}}), flush=True)


def chunked_prompt(w, alpha, m, group=1):
    """`--chunked M`: the workload's prompt processed as n / M chunks with a2sf_prefill_chunk (the
    first into an empty cache), one eviction per chunk.  Model flops: a chunk row attends the
    tokens cached before the chunk and the chunk's tokens up to itself (QK^T + PV).  With
    `--group R` the workload's heads are R query heads per K/V head (G / R K/V heads, random
    K/V rows) and the call is a2sf_prefill_chunk_gqa."""
    import torch

    import paper_2407_20485_amd as a2sf
    from paper_2407_20485_amd import synth
    G, n, d = w.G, w.n, w.d
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    code = a2sf.A2SF_F32 if w.dtype == "f32" else a2sf.A2SF_BF16
    data = synth.generate(w)
    q, k, v = (torch.from_numpy(data[x]) for x in ("q", "k", "v"))
    if w.dtype == "bf16":
        q, k, v = (t.view(torch.int16).view(torch.bfloat16) for t in (q, k, v))
    q, k, v = q.cuda(), k.cuda(), v.cuda()
    del data
    GQ = G                       # query heads
    if group > 1:                # the first G / group heads' K/V rows serve a group each
        G = G // group
        GQ = G * group
        q = q[:GQ].view(G, group, n, d)
        k, v = k[:G].contiguous(), v[:G].contiguous()
    cap = w.budget + m + 1
    cache = a2sf.Cache(G, cap, d, tdt)
    ws = torch.empty(a2sf.a2sf_workspace_bytes(GQ, m, cap, d, code, w.select, w.recent), dtype=torch.uint8, device="cuda")
    chunks = [(a, min(m, n - a)) for a in range(0, n, m)]
    parts = [(q[..., a:a + mm, :].contiguous(), k[:, a:a + mm].contiguous(), v[:, a:a + mm].contiguous()) for a, mm in chunks]
    o = torch.empty((GQ, m, d), dtype=tdt, device="cuda")

    def run():
        cache.len.zero_()
        for (a, mm), (qc, kc, vc) in zip(chunks, parts):
            if group > 1:
                a2sf.a2sf_prefill_chunk_gqa(qc, kc, vc, mm, a, group, alpha, w.select, w.recent, cache, o=o, workspace=ws)
            else:
                a2sf.a2sf_prefill_chunk(qc, kc, vc, mm, a, alpha, w.select, w.recent, cache, o=o, workspace=ws)
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 3
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    # Model flops, and the bytes a chunk cannot avoid: its Q, K, V rows read and its outputs written,
    # the cached K/V rows read once, the rows the head keeps written once.  A chunk of a few hundred
    # tokens against a budget of the same order has far fewer flops per byte than the machine
    # (2500 TFLOP/s : 8 TB/s = 312): the bound that applies is reported first.
    e = 4 if w.dtype == "f32" else 2
    flops, nbytes, cached = 0, 0, 0
    for a, mm in chunks:
        flops += GQ * 2 * 2 * d * (mm * cached + mm * (mm + 1) // 2)
        kept = min(cached + mm, w.budget)
        nbytes += d * e * (GQ * 2 * mm + G * (2 * mm + 2 * cached + 2 * kept))   # Q in and O out per query head, the rest per K/V head
        cached = kept
    tf = flops / ms / 1e9
    gbs = nbytes / ms / 1e6
    mfma = {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": tf / MFMA_BF16_PEAK_TFLOPS}
    hbm = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
    hbm_bound = flops / nbytes < MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS
    print(json.dumps({"kernel": "a2sf_prefill_chunk_gqa" if group > 1 else "a2sf_prefill_chunk",
                      "workload": f"configs[{w.cfg_id}] {w.name}", "G": G, "group": group, "prompt": n,
                      "chunk": m, "budget": f"{w.select}+{w.recent}", "alpha": alpha, "dtype": w.dtype,
                      "ms_per_prompt": ms, "flops_model": flops, "bytes_compulsory": nbytes,
                      "flops_per_byte": flops / nbytes,
                      "roofline": hbm if hbm_bound else mfma, "roofline_other": mfma if hbm_bound else hbm}), flush=True)


def grouped_query_step(w, alpha, group, steps=60, kv_shape=None, graph=False):
    """`--group R`: generation steps of the workload's shape with R query heads per K/V head (G / R
    K/V heads; random rows).  Algorithmic bytes: K and V rows once per K/V head, scores read and
    written, R query and output rows, the new K/V rows.  `--kv-shape HEADSxSLOTS` replaces the
    workload's K/V heads and cache slots (the generation step only, with the workspace that lets
    few heads split their tokens over workgroups); `--graph` replays the steps from a HIP graph."""
    import torch

    import paper_2407_20485_amd as a2sf
    d, B = w.d, w.budget
    G = max(1, w.G // group)
    select, recent = w.select, w.recent
    if kv_shape:
        G, slots = (int(x) for x in kv_shape.lower().split("x"))
        B = slots - 1
        select, recent = B // 2, B - B // 2
    e = 4 if w.dtype == "f32" else 2
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    cap = B + 1
    c = a2sf.Cache(G, cap, d, tdt)
    c.k.copy_(torch.randn(G, cap, d, device="cuda"))
    c.v.copy_(torch.randn(G, cap, d, device="cuda"))
    c.scores.copy_(torch.rand(G, cap, device="cuda"))
    c.pos.copy_(torch.arange(cap, dtype=torch.int32, device="cuda").repeat(G, 1))
    c.len.fill_(B)
    q = torch.randn(G, group, d, device="cuda").to(tdt)
    kn, vn = (torch.randn(G, d, device="cuda").to(tdt) for _ in range(2))
    o = torch.empty((G, group, d), dtype=tdt, device="cuda")
    code = a2sf.A2SF_F32 if w.dtype == "f32" else a2sf.A2SF_BF16
    ws_step = None
    if kv_shape:   # room for the token-split form: the logits of every query head + 64 splits of (max, sum, output)
        ws_step = torch.empty(a2sf.a2sf_workspace_bytes(G * group, 0, cap, d, code, select, recent)
                              + 4 * G * group * (cap + 64 * (d + 2)), dtype=torch.uint8, device="cuda")

    def run(t0, cnt):
        for t in range(t0, t0 + cnt):
            a2sf.a2sf_decode_step_gqa(q, kn, vn, B + t, c, group, alpha, select, recent, o, workspace=ws_step)
    run(0, 5)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if graph:
        snap = c.snapshot()          # every replay starts from the same cache: positions must not repeat
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run(5, steps)
        c.restore(snap)
        g.replay()
        c.restore(snap)
        torch.cuda.synchronize()
        e0.record()
        g.replay()
        e1.record()
    else:
        e0.record()
        run(5, steps)
        e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / steps
    L = B + 1
    nbytes = G * (2 * L * d * e + 8 * L + (2 * group + 2) * d * e)
    if kv_shape:
        print(json.dumps({"kernel": "a2sf_decode_step_gqa", "kv_heads": G, "group": group, "slots": L, "head_dim": d,
                          "dtype": w.dtype, "launch": "hip graph" if graph else "one launch per kernel",
                          "us_per_step": us, "bytes_per_step": nbytes,
                          "roofline": {"bound": "hbm", "achieved": nbytes / us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": nbytes / us / 1e3 / HBM_PEAK_GBS}}), flush=True)
        return
    # the prompt phase of the same grouping (random rows; model flops as for the plain prompt phase:
    # every query head has its own QK^T and PV sweep)
    n = w.n
    del q, kn, vn, o
    qp = torch.randn(G, group, n, d, device="cuda").to(tdt)
    kp, vp = (torch.randn(G, n, d, device="cuda").to(tdt) for _ in range(2))
    op = torch.empty_like(qp)
    ws = torch.empty(a2sf.a2sf_workspace_bytes(G * group, n, cap, d, code, w.select, w.recent), dtype=torch.uint8,
                     device="cuda")

    def prompt():
        a2sf.a2sf_prefill_gqa(qp, kp, vp, n, group, alpha, w.select, w.recent, c, o=op, workspace=ws)
    prompt()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(3):
        prompt()
    e1.record()
    torch.cuda.synchronize()
    pre_ms = e0.elapsed_time(e1) / 3
    flops = prefill_model_flops(G * group, n, d, with_o=True)
    print(json.dumps({"kernel": "a2sf_decode_step_gqa", "kv_heads": G, "group": group, "slots": L, "head_dim": d,
                      "dtype": w.dtype, "us_per_step": us, "bytes_per_step": nbytes,
                      "roofline": {"bound": "hbm", "achieved": nbytes / us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                   "frac": nbytes / us / 1e3 / HBM_PEAK_GBS},
                      "prefill_gqa_ms": pre_ms, "prompt": n,
                      "roofline_prefill": {"kernel": "a2sf_prefill_gqa", "bound": "mfma", "achieved": flops / pre_ms / 1e9,
                                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                           "frac": flops / pre_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS}}), flush=True)


def cpu_baseline(w, alpha, budget_s=12.0):
    """The oracle, as it stands, on this machine's host cores: prompt phase of two heads, then
    generation steps head by head until about `budget_s` seconds have been spent."""
    import numpy as np

    from oracle import a2sf_oracle as orc
    from paper_2407_20485_amd import synth

    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:  # pragma: no cover
        blas_threads = 1
    heads = [0, w.G // 2]
    caches, data = [], []
    t0 = time.perf_counter()
    for g in heads:
        Q, K, V = (x.astype(np.float64) for x in synth.head_arrays(w, g))
        data.append((Q, K, V))
    t_gen = time.perf_counter() - t0
    t0 = time.perf_counter()
    for Q, K, V in data:
        if w.n <= 8192:
            _, _, c = orc.prefill(Q[:w.n], K[:w.n], V[:w.n], alpha, w.select, w.recent)
        else:
            S, _ = orc.forgotten_scores_streamed(Q[:w.n], K[:w.n], [alpha], V=V[:w.n])
            keep = orc.select_keep(S[float(alpha)], np.arange(w.n), w.select, w.recent)
            c = orc.HeadCache(K[keep], V[keep], S[float(alpha)][keep], keep)
        caches.append(c)
    t_prefill = (time.perf_counter() - t0) / len(heads)
    head_steps, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < budget_s:
        for (Q, K, V), c0 in zip(data, caches):
            c = c0.copy()
            for t in range(w.T):
                r = w.n + t
                orc.decode_step(c, Q[r], K[r], V[r], r, alpha, w.select, w.recent)
            head_steps += w.T
    t_dec = time.perf_counter() - t0
    per_head_step = t_dec / head_steps
    return {
        "value": 1.0 / (per_head_step * w.G), "unit": "steps/s", "cores": int(blas_threads),
        "kind": "oracle",
        "sample": (f"{len(heads)} of {w.G} heads: float64 prompt phase {t_prefill:.3f} s/head, then "
                   f"{head_steps} head-steps of the generation loop in {t_dec:.1f} s "
                   f"({per_head_step * 1e6:.1f} us per head-step); value = 1/(G * that), i.e. "
                   f"extrapolated linearly to all {w.G} heads; the per-head Python loop is serial, "
                   f"BLAS may use up to {blas_threads} threads"),
        "prefill_s_per_head": t_prefill,
        "prefill_s_all_heads_extrapolated": t_prefill * w.G,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-o", action="store_true", help="prompt phase without attention outputs")
    ap.add_argument("--mode", choices=["fast", "stable"], default="fast")
    ap.add_argument("--alpha", type=float, default=None,
                    help="forgetting factor (default: the workload's; config 4 sweeps 0.1, 0.5, 0.9, 1.0)")
    ap.add_argument("--score-tol", type=float, default=2.5e-5,
                    help="relative tolerance of the prompt scores (a2sf_prefill_windowed: rows that provably "
                         "cannot change a score by more are skipped); 0 = a2sf_prefill, every row of nonzero "
                         "fp32 weight.  The scores are held to 1e-4 against the full-sum oracle either way")
    ap.add_argument("--graph", action="store_true",
                    help="replay the T generation steps of a pass from one HIP graph instead of launching "
                         "them one by one (matters for the few-head configs, whose steps are shorter than "
                         "a host launch)")
    ap.add_argument("--similarity-kernel", metavar="HEADSxROWS", default=None,
                    help="instead of the pass: time the Ideal-mask similarity diagnostic alone (bf16, d = 128)")
    ap.add_argument("--chunked", type=int, metavar="M", default=None,
                    help="instead of the pass: the prompt phase as chunks of M tokens (a2sf_prefill_chunk)")
    ap.add_argument("--group", type=int, metavar="R", default=None,
                    help="instead of the pass: generation steps with R query heads per K/V head (a2sf_decode_step_gqa)")
    ap.add_argument("--kv-shape", metavar="HEADSxSLOTS", default=None,
                    help="with --group: time the generation step alone on this many K/V heads and cache slots")
    ap.add_argument("--ceilings", choices=["hbm", "mfma", "all"], default=None,
                    help="instead of the pass: run the stand-alone probe of the machine's ceilings "
                         "(streaming reads in the generation step's access pattern; sustained matrix-core rate)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU only (every head is an independent problem, so "
            "more GPUs would each take a share of the heads with no exchange). Run with --gpus 1.")
        sys.exit(2)

    if args.ceilings:
        import subprocess
        exe = os.path.join(ROOT, "paper_2407_20485_amd", "ceilings")
        if not os.path.exists(exe):
            log(f"bench.py: {exe} is missing: build it with `python -m paper_2407_20485_amd.build`")
            sys.exit(3)
        sys.exit(subprocess.run([exe] + ([] if args.ceilings == "all" else [args.ceilings])).returncode)

    import numpy as np
    import torch

    import paper_2407_20485_amd as a2sf
    from paper_2407_20485_amd import synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback.")
        sys.exit(3)
    if args.similarity_kernel:
        return similarity_kernel(args.similarity_kernel)
    w = synth.CONFIGS[args.config]
    alpha = w.alpha if args.alpha is None else args.alpha
    if args.chunked:
        return chunked_prompt(w, alpha, args.chunked, args.group or 1)
    if args.group:
        return grouped_query_step(w, alpha, args.group, kv_shape=args.kv_shape, graph=args.graph)
    G, n, d, T = w.G, w.n, w.d, w.T
    e = 4 if w.dtype == "f32" else 2
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    mode = a2sf.A2SF_EVICT_FAST if args.mode == "fast" else a2sf.A2SF_EVICT_STABLE

    log(f"[bench] generating config {w.cfg_id} ({w.name}): G={G} n={n} d={d} {w.dtype} T={T} "
        f"budget={w.select}+{w.recent} alpha={alpha}")
    t0 = time.perf_counter()
    data = synth.generate(w, progress=lambda c, H: log(f"[bench]   {c}/{H} heads"))
    dev = {}
    for k, v in data.items():
        t = torch.from_numpy(v)
        if w.dtype == "bf16":
            t = t.view(torch.int16).view(torch.bfloat16)
        dev[k] = t.cuda()
    del data
    log(f"[bench] inputs resident in HBM after {time.perf_counter() - t0:.1f} s")

    capacity = w.budget + 1
    cache = a2sf.Cache(G, capacity, d, tdt)
    code = a2sf.A2SF_F32 if w.dtype == "f32" else a2sf.A2SF_BF16
    ws = torch.empty(a2sf.a2sf_workspace_bytes(G, n, capacity, d, code, w.select, w.recent),
                     dtype=torch.uint8, device="cuda")
    o_pre = None if args.no_o else torch.empty((G, n, d), dtype=tdt, device="cuda")
    o_dec = torch.empty((G, d), dtype=tdt, device="cuda")

    graph = None

    def decode_steps():
        for t in range(T):
            a2sf.a2sf_decode_step(dev["qd"][t], dev["kd"][t], dev["vd"][t], n + t, cache, alpha,
                                  w.select, w.recent, o_dec, mode=mode, workspace=ws)

    def one_pass(ev=None):
        if ev:
            ev[0].record()
        if args.score_tol > 0:
            a2sf.a2sf_prefill_windowed(dev["q"], dev["k"], dev["v"], n, alpha, args.score_tol, w.select,
                                       w.recent, cache, o=o_pre, scores_full=None, workspace=ws)
        else:
            a2sf.a2sf_prefill(dev["q"], dev["k"], dev["v"], n, alpha, w.select, w.recent, cache,
                              o=o_pre, scores_full=None, workspace=ws)
        if ev:
            ev[1].record()
        if graph is not None:
            graph.replay()
        else:
            decode_steps()
        if ev:
            ev[2].record()

    if args.copy_calibration:   # a copy kernel of known size for the counter runs
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)     # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    if args.graph:   # the library only enqueues kernels: the T steps of a pass fit one HIP graph
        one_pass()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            decode_steps()
        torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_pass(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    prefill_ms = [ev[0].elapsed_time(ev[1]) for ev in events]
    decode_ms = [ev[1].elapsed_time(ev[2]) for ev in events]
    dec_s_per_step = sum(decode_ms) / 1e3 / (args.steps * T)
    pre_s = sum(prefill_ms) / 1e3 / args.steps
    lens = cache.len.cpu().numpy()
    assert np.all(lens == min(n + T, w.budget)), "cache lengths wrong after the timed passes"

    L = min(n, w.budget) + 1     # tokens a steady-state generation step reads
    dbytes = decode_bytes_per_step(G, L, d, e)
    if args.mode == "stable" and n + T > w.budget:
        # keeping the slots in ascending position costs row moves that the method itself does not
        # need: the victim is never one of the `recent` newest tokens, so at least those rows of K
        # and V move down one slot (read + write) in every step
        dbytes += G * 4 * w.recent * d * e
    flops = prefill_model_flops(G, n, d, with_o=not args.no_o)
    dec_gbs = dbytes / dec_s_per_step / 1e9
    pre_tflops = flops / pre_s / 1e12
    nsplit, rows_per_split, wave_slots, wave_heads = a2sf.a2sf_decode_plan(G, capacity, d)   # the library's launch plan
    if nsplit > 1:
        nsplit_note = f"tokens of a head split over {nsplit} workgroups + combine kernel"
    elif wave_slots and wave_heads > 1 and args.mode != "stable":
        nsplit_note = f"one fused kernel, persistent workgroups, {wave_heads} heads per wave, small writes held in LDS"
    else:
        nsplit_note = "one fused kernel, " + ("one wave per head" if wave_slots else "one workgroup per head")
    if args.mode == "stable":
        nsplit_note += ", then select + in-place compaction"

    out = {
        "metric": "decode steps/s (fused attn+A2SF+evict) & HBM GB/s; prefill score TFLOP/s",
        "value": 1.0 / dec_s_per_step,
        "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{w.cfg_id}] {w.name}", "G": G, "prompt": n, "head_dim": d,
                   "decode_steps": T, "budget": f"{w.select}+{w.recent}", "alpha": alpha,
                   "evict_mode": args.mode, "prefill_outputs": not args.no_o,
                   "prefill_call": (f"a2sf_prefill_windowed, score_rel_tol {args.score_tol:g}" if args.score_tol > 0
                                    else "a2sf_prefill"),
                   "decode_launch": "hip graph of the T steps" if args.graph else "one launch per kernel",
                   "pass": "prefill + T decode steps"},
        "decode_us_per_step": dec_s_per_step * 1e6,
        "decode_hbm_gbs_algorithmic": dec_gbs,
        "prefill_ms": pre_s * 1e3,
        "prefill_tflops_model": pre_tflops,
        "roofline": {"kernel": f"decode step ({nsplit_note})", "bound": "hbm", "achieved": dec_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dec_gbs / HBM_PEAK_GBS,
                     "bytes_per_launch": dbytes, "avg_launch_us": dec_s_per_step * 1e6,
                     "bytes_convention": ("K and V rows read once, scores read and written, q / o / new rows"
                                          + ("; plus the rows of the recent window moved down one slot "
                                             "(a lower bound of the stable mode's row moves)" if args.mode == "stable" else "")),
                     "traffic": read_traffic(f"decode_cfg{w.cfg_id}" + ("_stable" if args.mode == "stable" else "")),
                     "traffic_source": f"{TRAFFIC_FILE} (earlier rocprofv3 --pmc runs of this command; not measured in this run)"},
        "roofline_prefill": {"kernel": "a2sf_prefill (attention fwd + column scores + select + gather)",
                             "bound": "mfma", "achieved": pre_tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                             "unit": "TFLOP/s", "frac": pre_tflops / MFMA_BF16_PEAK_TFLOPS,
                             "flops_per_launch": flops, "avg_launch_ms": pre_s * 1e3,
                             "flop_convention": "model flops: one causal QK^T sweep + one PV sweep; "
                                                "the score kernel's recomputed QK^T is not counted",
                             "traffic": read_traffic(f"prefill_cfg{w.cfg_id}" + ("_no_o" if args.no_o else "")),
                             "traffic_source": f"{TRAFFIC_FILE} (earlier rocprofv3 --pmc runs of this command; not measured in this run)"},
    }
    if args.no_o:
        # Without outputs the call computes the log-sum-exp of the rows that can still contribute in
        # fp32 (Section 3.3: the forgetting factor takes older rows to 0) and nothing for the others,
        # so a full QK^T sweep is no measure of its work any more: the leg is priced by the bytes it
        # cannot avoid -- every key once, the query rows of that window, the kept rows gathered.
        rows = n if alpha >= 1.0 else (1 if alpha <= 0.0 else min(n, int(160.0 / -math.log2(alpha)) + 1))
        B = min(n, w.budget)
        pbytes = G * (n * d * e + rows * d * e + 2 * n * 4 + 2 * 2 * B * d * e)
        out["prefill_tflops_model_note"] = ("dense-equivalent: one full causal QK^T sweep over the time of a call "
                                            "that skips the rows whose weight is exactly 0 in fp32")
        out["roofline_prefill"] = {
            "kernel": "a2sf_prefill without outputs (log-sum-exp of the contributing rows + column scores + select + gather)",
            "bound": "hbm", "achieved": pbytes / pre_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": pbytes / pre_s / 1e9 / HBM_PEAK_GBS, "bytes_per_launch": pbytes, "avg_launch_ms": pre_s * 1e3,
            "bytes_convention": f"K read once, the {rows} query rows per head of nonzero fp32 weight, scores written and read, "
                                "kept K/V rows read and written",
            "dense_equivalent_tflops": pre_tflops,
            # flops of the rows that are processed: the log-sum-exp pass over the 128-row blocks from the
            # one holding row n - rows on, the score pass over the rows themselves (2 flop per MAC)
            "flops_of_rows_processed": G * 2 * d * (sum(i + 1 for i in range(((n - rows) // 128) * 128, n))
                                                    + sum(i + 1 for i in range(n - rows, n))),
            "traffic": read_traffic(f"prefill_cfg{w.cfg_id}_no_o"),
            "traffic_source": f"{TRAFFIC_FILE} (earlier rocprofv3 --pmc runs of this command; not measured in this run)"}
    if not args.no_cpu_baseline:
        log("[bench] timing the float64 oracle on the host cores ...")
        out["cpu_baseline"] = cpu_baseline(w, alpha)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
