"""Oracle side of the record-and-replay parity runs (numpy only; safe to import in a worker
process that never touches the GPU).

The GPU run of a workload records, for a sample of heads, what the HIP path produced: the
prompt phase's outputs and scores, and after every generation step the output row, the
retained positions and their scores (plus the cached K/V rows at a few steps).  A worker then
regenerates the head's inputs from its seed, runs the float64 oracle over the same prompt and
steps -- following the GPU's retained set only where the oracle itself accepts the difference
as an in-margin swap -- and compares everything element by element.

Tolerances (the target statement of this build): attention outputs max-abs 2e-2 for bf16,
1e-5 for fp32; scores relative 1e-4; retained sets identical, except that tokens whose scores
lie within 1e-6 of each other across the cut may be swapped.
"""
from __future__ import annotations

import os
import sys

import numpy as np

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if _ROOT not in sys.path:
    sys.path.insert(0, _ROOT)

from oracle import a2sf_oracle as orc  # noqa: E402

O_TOL = {"bf16": 2e-2, "f32": 1e-5}
SCORE_RTOL = 1e-4
MARGIN = 1e-6


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(np.asarray(got, dtype=np.float64) - want)
    return float((err / np.maximum(np.abs(want), 1e-300)).max()) if err.size else 0.0


class Mismatch(AssertionError):
    pass


def _compare_state(pos_g, s_g, rows_g, oc, what, ordered):
    """GPU slots (positions, scores, optional (K, V) rows) against the oracle's cache."""
    pos_g = np.asarray(pos_g, dtype=np.int64)
    if len(pos_g) != len(oc):
        raise Mismatch(f"{what}: len {len(pos_g)} vs oracle {len(oc)}")
    if len(set(pos_g.tolist())) != len(pos_g):
        raise Mismatch(f"{what}: duplicate positions")
    if ordered and not np.all(np.diff(pos_g) > 0):
        raise Mismatch(f"{what}: slots not in ascending position")
    order = np.argsort(pos_g)
    oo = oc.sorted_by_pos()
    if not np.array_equal(pos_g[order], oo.pos):
        raise Mismatch(f"{what}: retained sets differ")
    rel = rel_err(np.asarray(s_g)[order], oo.S)
    if rel > SCORE_RTOL:
        raise Mismatch(f"{what}: score rel error {rel:.3e}")
    if rows_g is not None:     # K/V rows are copies: bit-exact
        if not np.array_equal(np.asarray(rows_g[0], dtype=np.float64)[order], oo.K):
            raise Mismatch(f"{what}: K rows differ")
        if not np.array_equal(np.asarray(rows_g[1], dtype=np.float64)[order], oo.V):
            raise Mismatch(f"{what}: V rows differ")
    return rel


def replay_head(job):
    """One head, every forgetting factor that was run on it.

    job: dict(w=Workload, g=head id, select, recent, threads,
              runs={alpha: dict(o=[n,d] float32 | None, s_full=[n] float32, s_full_alt=[n] | None,
                                pre=(pos, scores, (K, V) | None), fast=bool,
                                steps=[(o[d], pos, scores, (K, V) | None), ...])})
    Returns dict(g, o_err, s_rel, swaps, failure | None).
    """
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=int(job.get("threads", 1)))
    except Exception:  # pragma: no cover
        limiter = None
    from paper_2407_20485_amd import synth

    w, g = job["w"], job["g"]
    select, recent = job["select"], job["recent"]
    res = {"g": g, "o_err": 0.0, "s_rel": 0.0, "swaps": 0, "failure": None}
    try:
        Q, K, V = (x.astype(np.float64) for x in synth.head_arrays(w, g))
        n = w.n
        alphas = [float(a) for a in job["runs"]]
        if n <= 8192:
            P = orc.causal_probabilities(Q[:n], K[:n])
            O = orc.attention_output(P, V[:n])
            S_by = {a: orc.forgotten_scores(P, a) for a in alphas}
            del P
        else:
            S_by, O = orc.forgotten_scores_streamed(Q[:n], K[:n], alphas, V=V[:n], rows_per_chunk=1024)
        for alpha_key, run in job["runs"].items():
            alpha = float(alpha_key)
            what = f"head {g} alpha {alpha}"
            S_full = S_by[alpha]
            if run.get("o") is not None:
                err = float(np.abs(np.asarray(run["o"], dtype=np.float64) - O).max())
                res["o_err"] = max(res["o_err"], err)
                if err > O_TOL[w.dtype]:
                    raise Mismatch(f"{what}: prompt output max-abs {err:.3e}")
            for key in ("s_full", "s_full_alt"):
                if run.get(key) is not None:
                    rel = rel_err(run[key], S_full)
                    res["s_rel"] = max(res["s_rel"], rel)
                    if rel > SCORE_RTOL:
                        raise Mismatch(f"{what}: prompt score ({key}) rel error {rel:.3e}")
            pos_g, s_g, rows_g = run["pre"]
            keep, sw = orc._resolve_keep(S_full, np.arange(n), select, recent,
                                         [int(p) for p in pos_g], MARGIN)
            res["swaps"] += sw
            oc = orc.HeadCache(K[keep], V[keep], S_full[keep], keep)
            res["s_rel"] = max(res["s_rel"], _compare_state(pos_g, s_g, rows_g, oc, f"{what} after the prompt", True))
            ascending = True
            for t, (o_g, pos_g, s_g, rows_g) in enumerate(run["steps"]):
                r = n + t
                evicts = len(oc) + 1 > select + recent
                if run.get("fast", True):
                    ascending = ascending and not evicts
                o_ref, _ = orc.attend_and_update(oc, Q[r], K[r], V[r], r, alpha)
                _, sw = orc.evict(oc, select, recent, forced_retained=[int(p) for p in pos_g], margin=MARGIN)
                res["swaps"] += sw
                err = float(np.abs(np.asarray(o_g, dtype=np.float64) - o_ref).max())
                res["o_err"] = max(res["o_err"], err)
                if err > O_TOL[w.dtype]:
                    raise Mismatch(f"{what} step {t}: output max-abs {err:.3e}")
                res["s_rel"] = max(res["s_rel"], _compare_state(pos_g, s_g, rows_g, oc, f"{what} step {t}", ascending))
    except (Mismatch, ValueError) as e:
        res["failure"] = f"{type(e).__name__}: {e}"
    finally:
        if limiter is not None:
            limiter.unregister() if hasattr(limiter, "unregister") else None
    return res


def _sorted_state(pos_g, s_g, oc, what):
    """Retained set and scores of a GPU head (any slot order) against the oracle's cache."""
    pos_g = np.asarray(pos_g, dtype=np.int64)
    if len(pos_g) != len(oc):
        raise Mismatch(f"{what}: len {len(pos_g)} vs oracle {len(oc)}")
    order = np.argsort(pos_g)
    oo = oc.sorted_by_pos()
    if not np.array_equal(pos_g[order], oo.pos):
        raise Mismatch(f"{what}: retained sets differ")
    rel = rel_err(np.asarray(s_g)[order], oo.S)
    if rel > SCORE_RTOL:
        raise Mismatch(f"{what}: score rel error {rel:.3e}")
    return rel, order, oo


def replay_head_chunks(job):
    """A prompt processed in chunks (one eviction per chunk) on one head.

    job: dict(w, g, select, recent, alpha, m, threads,
              chunks=[(o[m,d] float32, pos, scores), ...] one per chunk, rows=(K, V) after the last)
    Returns dict(g, o_err, s_rel, swaps, failure | None)."""
    from paper_2407_20485_amd import synth
    w, g = job["w"], job["g"]
    res = {"g": g, "o_err": 0.0, "s_rel": 0.0, "swaps": 0, "failure": None}
    try:
        Q, K, V = (x.astype(np.float64) for x in synth.head_arrays(w, g))
        m, d = job["m"], Q.shape[1]
        oc = orc.HeadCache(np.zeros((0, d)), np.zeros((0, d)), np.zeros(0), np.zeros(0, dtype=np.int64))
        for c, (o_g, pos_g, s_g) in enumerate(job["chunks"]):
            r0 = c * m
            O, _, sw = orc.prefill_chunk(oc, Q[r0:r0 + m], K[r0:r0 + m], V[r0:r0 + m], r0, job["alpha"],
                                         job["select"], job["recent"],
                                         forced_retained=[int(p) for p in pos_g], margin=MARGIN)
            res["swaps"] += sw
            err = float(np.abs(np.asarray(o_g, dtype=np.float64) - O).max())
            res["o_err"] = max(res["o_err"], err)
            if err > O_TOL[w.dtype]:
                raise Mismatch(f"head {g} chunk {c}: output max-abs {err:.3e}")
            rel, order, oo = _sorted_state(pos_g, s_g, oc, f"head {g} chunk {c}")
            res["s_rel"] = max(res["s_rel"], rel)
            if not np.all(np.diff(np.asarray(pos_g)) > 0):
                raise Mismatch(f"head {g} chunk {c}: slots not in ascending position")
        Kg, Vg = job["rows"]
        if not (np.array_equal(np.asarray(Kg, dtype=np.float64)[order], oo.K)
                and np.array_equal(np.asarray(Vg, dtype=np.float64)[order], oo.V)):
            raise Mismatch(f"head {g}: cached rows differ after the last chunk")
    except (Mismatch, ValueError) as e:
        res["failure"] = f"{type(e).__name__}: {e}"
    return res


def replay_kv_head_group(job):
    """Grouped-query heads: `group` consecutive heads of the workload act as the query heads of
    one K/V head (keys and values of the first of them).

    job: dict(w, g (K/V head), group, select, recent, alpha,
              o=[group, rows, d] float32 (the last `rows` prompt rows), s_full=[n],
              pre=(pos, scores), steps=[(o[group, d], pos, scores), ...])"""
    from paper_2407_20485_amd import synth
    w, g, R = job["w"], job["g"], job["group"]
    res = {"g": g, "o_err": 0.0, "s_rel": 0.0, "swaps": 0, "failure": None}
    try:
        heads = [synth.head_arrays(w, g * R + r) for r in range(R)]
        Qs = np.stack([h[0].astype(np.float64) for h in heads])            # [R, n + T, d]
        K, V = heads[0][1].astype(np.float64), heads[0][2].astype(np.float64)
        n = w.n
        pos_g, s_g = job["pre"]
        O, S_full, oc = orc.gqa_prefill(Qs[:, :n], K[:n], V[:n], job["alpha"], job["select"], job["recent"],
                                        forced_retained=[int(p) for p in pos_g], margin=MARGIN)
        rows = job["o"].shape[1]
        err = float(np.abs(np.asarray(job["o"], dtype=np.float64) - O[:, n - rows:]).max())
        res["o_err"] = err
        if err > O_TOL[w.dtype]:
            raise Mismatch(f"K/V head {g}: prompt output max-abs {err:.3e}")
        rel = rel_err(job["s_full"], S_full)
        res["s_rel"] = rel
        if rel > SCORE_RTOL:
            raise Mismatch(f"K/V head {g}: prompt score rel error {rel:.3e}")
        res["s_rel"] = max(res["s_rel"], _sorted_state(pos_g, s_g, oc, f"K/V head {g} after the prompt")[0])
        for t, (o_g, pos_g, s_g) in enumerate(job["steps"]):
            r = n + t
            o_ref, _, _, sw = orc.gqa_decode_step(oc, Qs[:, r], K[r], V[r], r, job["alpha"], job["select"],
                                                  job["recent"], forced_retained=[int(p) for p in pos_g],
                                                  margin=MARGIN)
            res["swaps"] += sw
            err = float(np.abs(np.asarray(o_g, dtype=np.float64) - o_ref).max())
            res["o_err"] = max(res["o_err"], err)
            if err > O_TOL[w.dtype]:
                raise Mismatch(f"K/V head {g} step {t}: output max-abs {err:.3e}")
            res["s_rel"] = max(res["s_rel"], _sorted_state(pos_g, s_g, oc, f"K/V head {g} step {t}")[0])
    except (Mismatch, ValueError) as e:
        res["failure"] = f"{type(e).__name__}: {e}"
    return res
