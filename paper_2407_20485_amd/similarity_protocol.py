"""Similarity of pruning policies to the Ideal mask (Section 4.3, Table 2 of the paper) on the
GPU, token by token: every step first asks the library for the cosine between the policy's
attention row and the Ideal row, then runs the generation step that updates the cache.

    python -m paper_2407_20485_amd.similarity_protocol [--config 1] [--heads 32] [--ratio 0.2]

prints the average cosine of the paper's four policies on a seeded synthetic workload (the
paper's numbers need its models and datasets; this reproduces the protocol, not the table).
All arithmetic happens in liba2sf.so; this file only sequences the calls.
"""
from __future__ import annotations

import argparse
import dataclasses
import time

import torch

from . import binding as B
from . import synth


def mask_similarity(q, k, v, alpha, select, recent, workspace=None):
    """q, k, v: [G, n, d] device tensors (fp32 or bf16) of whole sequences.  Generates the
    sequence from an empty cache under the policy and returns cos [n, G] (fp32, device): row i
    is the similarity at the step that appends token i."""
    G, n, d = q.shape
    code = B.A2SF_F32 if q.dtype == torch.float32 else B.A2SF_BF16
    budget = select + recent
    cache = B.Cache(G, budget + 1, d, q.dtype)
    if workspace is None:
        workspace = torch.empty(B.a2sf_workspace_bytes(G, 1, budget + 1, d, code, select, recent),
                                dtype=torch.uint8, device=q.device)
    qt, kt, vt = (x.transpose(0, 1).contiguous() for x in (q, k, v))      # [n, G, d]: a step's rows together
    B.a2sf_prefill(qt[0].unsqueeze(1), kt[0].unsqueeze(1), vt[0].unsqueeze(1), 1, alpha, select, recent,
                   cache, workspace=workspace)
    cos = torch.ones((n, G), dtype=torch.float32, device=q.device)
    o = torch.empty((G, d), dtype=q.dtype, device=q.device)
    for i in range(1, n):
        B.a2sf_ideal_similarity(qt[i], k, n, i, cache, cos[i])
        B.a2sf_decode_step(qt[i], kt[i], vt[i], i, cache, alpha, select, recent, o, workspace=workspace)
    return cos


POLICIES = (   # name, alpha, share of the budget that is score-selected
    ("Local", 1.0, 0.0),
    ("H2O", 1.0, 0.5),
    ("A2SF 0.1", 0.1, 1.0),
    ("A2SF 0.5", 0.5, 1.0),
)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1, help="synthetic workload (shapes and salience recipe)")
    ap.add_argument("--heads", type=int, default=32)
    ap.add_argument("--length", type=int, default=None, help="sequence length (default: the config's prompt)")
    ap.add_argument("--ratio", type=float, default=0.2, help="cache ratio, as in the paper's Section 4.3")
    ap.add_argument("--salience-logit-shift", action="store_true",
                    help="plant the salient tokens so that their logits stand out by their full magnitude "
                         "(strongly peaked attention, as trained models show) instead of magnitude / sqrt(d)")
    a = ap.parse_args()
    w = synth.CONFIGS[a.config]
    if a.salience_logit_shift:
        w = dataclasses.replace(w, logit_shift=True)
    n = a.length or w.n
    heads = list(range(min(a.heads, w.G)))
    rows = [synth.head_arrays(w, g, length=n) for g in heads]
    dt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    q, k, v = (torch.stack([torch.from_numpy(r[j]) for r in rows]).to("cuda", dt) for j in range(3))
    budget = int(a.ratio * n)
    print(f"workload {w.name}{' (salient logits shifted)' if w.logit_shift else ''}: {len(heads)} heads, n = {n}, d = {w.d}, {w.dtype}; cache {budget} tokens "
          f"({a.ratio:.0%}); average cosine to the Ideal rows over the steps past the budget")
    for name, alpha, share in POLICIES:
        select = int(round(share * budget))
        t0 = time.time()
        cos = mask_similarity(q, k, v, alpha, select, budget - select)
        mean_dev = torch.empty(1, dtype=torch.float32, device=cos.device)
        B.a2sf_similarity_mean(cos, n, len(heads), budget + 1, mean_dev)
        mean = float(mean_dev.item())
        print(f"  {name:9s} alpha={alpha:<4} select={select:4d} recent={budget - select:4d}  "
              f"cosine {mean:.3f}   ({time.time() - t0:.1f} s)")


if __name__ == "__main__":
    main()
