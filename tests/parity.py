"""Lock-step comparison of the HIP path (through the C ABI) with the float64 oracle.

Tolerances (the target statement of this build): attention outputs max-abs 2e-2 for bf16,
1e-5 for fp32; scores relative 1e-4; retained sets identical, except that tokens whose
scores lie within 1e-6 of each other across the cut may be swapped - then the oracle is
told to follow the GPU's choice (it refuses if the swap is outside the margin).
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2407_20485_amd as a2sf
from oracle import a2sf_oracle as orc
from paper_2407_20485_amd import synth

from oracle_replay import MARGIN, O_TOL, SCORE_RTOL   # the tolerances, stated once


def to_device(arr: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(arr)
    if dtype == "bf16":
        t = t.view(torch.int16).view(torch.bfloat16)
    return t.cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def torch_dtype(dtype: str):
    return torch.float32 if dtype == "f32" else torch.bfloat16


class Problem:
    """A workload on the GPU plus what the oracle needs for a chosen sample of heads."""

    def __init__(self, w: synth.Workload, heads=None, sample=None, capacity=None, threads=None,
                 progress=None, host_copies=True):
        self.w = w
        self.heads = list(range(w.G)) if heads is None else list(heads)   # heads on the GPU
        self.G = len(self.heads)
        self.sample = list(range(self.G)) if sample is None else list(sample)  # indices into heads
        data = synth.generate(w, self.heads, threads=threads, progress=progress)
        self.host = {}
        for i in (self.sample if host_copies else []):   # float64 copies for the oracle
            self.host[i] = tuple(
                np.concatenate([self._f32(data[k][i]), self._f32(data[k + "d"][:, i])]).astype(np.float64)
                for k in ("q", "k", "v"))
        self.dev = {k: to_device(v, w.dtype) for k, v in data.items()}
        del data
        self.capacity = capacity if capacity is not None else w.budget + 1
        self.cache = a2sf.Cache(self.G, self.capacity, w.d, torch_dtype(w.dtype))
        code = a2sf.A2SF_F32 if w.dtype == "f32" else a2sf.A2SF_BF16
        nbytes = a2sf.a2sf_workspace_bytes(self.G, w.n, self.capacity, w.d, code, w.select, w.recent)
        assert nbytes > 0
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.o_dec = torch.empty((self.G, w.d), dtype=torch_dtype(w.dtype), device="cuda")

    def _f32(self, a):
        return a if self.w.dtype == "f32" else synth.bf16_bits_to_f32(a)

    # ---- GPU calls
    def gpu_prefill(self, alpha, want_o=True, want_scores=True, select=None, recent=None, tol=None):
        """alpha: one factor, or a sequence of G per-head factors.  tol: relative tolerance of the
        scores (a2sf_prefill_windowed); None = a2sf_prefill."""
        w = self.w
        select = w.select if select is None else select
        recent = w.recent if recent is None else recent
        o = torch.empty_like(self.dev["q"]) if want_o else None
        s = torch.empty((self.G, w.n), dtype=torch.float32, device="cuda") if want_scores else None
        if tol is not None:
            a2sf.a2sf_prefill_windowed(self.dev["q"], self.dev["k"], self.dev["v"], w.n, float(alpha), tol,
                                       select, recent, self.cache, o=o, scores_full=s, workspace=self.ws)
        elif np.ndim(alpha) == 0:
            a2sf.a2sf_prefill(self.dev["q"], self.dev["k"], self.dev["v"], w.n, float(alpha), select,
                              recent, self.cache, o=o, scores_full=s, workspace=self.ws)
        else:
            ah = torch.tensor(np.asarray(alpha, dtype=np.float32), device="cuda")
            a2sf.a2sf_prefill_alpha_per_head(self.dev["q"], self.dev["k"], self.dev["v"], w.n, ah,
                                             float(np.max(alpha)), select, recent, self.cache, o=o,
                                             scores_full=s, workspace=self.ws)
        return o, s

    def gpu_decode(self, t, alpha, mode=a2sf.A2SF_EVICT_FAST, select=None, recent=None):
        w = self.w
        select = w.select if select is None else select
        recent = w.recent if recent is None else recent
        if np.ndim(alpha) == 0:
            a2sf.a2sf_decode_step(self.dev["qd"][t], self.dev["kd"][t], self.dev["vd"][t], w.n + t,
                                  self.cache, float(alpha), select, recent, self.o_dec, mode=mode,
                                  workspace=self.ws)
        else:
            ah = torch.tensor(np.asarray(alpha, dtype=np.float32), device="cuda")
            a2sf.a2sf_decode_step_alpha_per_head(self.dev["qd"][t], self.dev["kd"][t], self.dev["vd"][t],
                                                 w.n + t, self.cache, ah, select, recent, self.o_dec,
                                                 mode=mode, workspace=self.ws)
        return self.o_dec

    def fetch(self, rows=True):
        """Download the cache state of the sampled heads in a few copies; afterwards
        gpu_cache_of(i) serves from that snapshot."""
        idx = torch.as_tensor(self.sample, device="cuda")
        c = self.cache
        snap = {"len": c.len[idx].cpu().numpy(), "pos": c.pos[idx].cpu().numpy().astype(np.int64),
                "scores": c.scores[idx].cpu().numpy().astype(np.float64)}
        if rows:
            snap["k"] = to_f64(c.k[idx])
            snap["v"] = to_f64(c.v[idx])
        self._snap = snap
        self._where = {h: j for j, h in enumerate(self.sample)}

    def gpu_cache_of(self, i):
        """(len, pos[len], scores[len], K[len,d] | None, V[len,d] | None) of sampled head i."""
        s, j = self._snap, self._where[i]
        L = int(s["len"][j])
        return (L, s["pos"][j, :L], s["scores"][j, :L],
                s["k"][j, :L] if "k" in s else None, s["v"][j, :L] if "v" in s else None)


def compare_scores(got, want, what):
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(np.asarray(got, dtype=np.float64) - want)
    bad = err > SCORE_RTOL * np.abs(want) + 1e-30
    assert not bad.any(), (f"{what}: {int(bad.sum())} scores off, worst rel "
                           f"{(err / np.maximum(np.abs(want), 1e-300)).max():.3e}")
    return float((err / np.maximum(np.abs(want), 1e-300)).max())


def compare_cache(p: Problem, i: int, oc: orc.HeadCache, what: str, check_rows=True, ordered=False):
    """GPU head i against the oracle cache (which already follows the GPU's retained set)."""
    L, pos, S, K, V = p.gpu_cache_of(i)
    assert L == len(oc), f"{what}: len {L} vs oracle {len(oc)}"
    assert len(set(pos.tolist())) == L, f"{what}: duplicate positions"
    if ordered:
        assert np.all(np.diff(pos) > 0), f"{what}: slots not in ascending position"
    order = np.argsort(pos)
    assert np.array_equal(pos[order], np.sort(oc.pos)), f"{what}: retained sets differ"
    oo = oc.sorted_by_pos()
    rel = compare_scores(S[order], oo.S, what)
    if check_rows and K is not None:   # K/V rows are copies: bit-exact
        assert np.array_equal(K[order], oo.K), f"{what}: K rows differ"
        assert np.array_equal(V[order], oo.V), f"{what}: V rows differ"
    return rel


class LockStep:
    """Runs prefill + decode on the GPU for all heads and on the oracle for the sample."""

    def __init__(self, p: Problem, alpha: float, select=None, recent=None):
        self.p, self.alpha = p, alpha
        self.select = p.w.select if select is None else select
        self.recent = p.w.recent if recent is None else recent
        self.oc = {}
        self.swaps = 0
        self.max_o_err = 0.0
        self.max_s_rel = 0.0
        self.check_rows = True
        self.ascending = True    # slots in ascending position so far (lost by a fast-mode eviction)

    def alpha_of(self, i):
        """Factor of GPU head i as the kernels see it (fp32)."""
        a = self.alpha if np.ndim(self.alpha) == 0 else self.alpha[i]
        return float(np.float32(a))

    def prefill(self, check_o_rows=None):
        p, w = self.p, self.p.w
        o, s = p.gpu_prefill(self.alpha, select=self.select, recent=self.recent)
        torch.cuda.synchronize()
        p.fetch()
        for i in p.sample:
            Q, K, V = (x[:w.n] for x in p.host[i])
            _, gpos, _, _, _ = p.gpu_cache_of(i)
            O, S_full, oc = orc.prefill(Q, K, V, self.alpha_of(i), self.select, self.recent)
            if set(gpos.tolist()) != set(oc.pos.tolist()):
                before = set(oc.pos.tolist())
                O, S_full, oc = orc.prefill(Q, K, V, self.alpha_of(i), self.select, self.recent,
                                            forced_retained=gpos.tolist(), margin=MARGIN)
                self.swaps += len(before - set(gpos.tolist()))
            self.oc[i] = oc
            og = to_f64(o[i])
            err = np.abs(og - O).max()
            self.max_o_err = max(self.max_o_err, err)
            assert err <= O_TOL[w.dtype], f"head {i}: prefill output max-abs {err:.3e}"
            self.max_s_rel = max(self.max_s_rel,
                                 compare_scores(s[i].cpu().numpy(), S_full, f"head {i} prompt scores"))
            self.max_s_rel = max(self.max_s_rel,
                                 compare_cache(p, i, oc, f"head {i} after prefill", ordered=True))
        return o, s

    def step(self, t, mode=a2sf.A2SF_EVICT_FAST):
        p, w = self.p, self.p.w
        if mode != a2sf.A2SF_EVICT_STABLE:
            # a fast-mode eviction refills the hole; stable mode keeps whatever order it finds
            evicts = len(self.oc[p.sample[0]]) + 1 > self.select + self.recent
            self.ascending = self.ascending and not evicts
        o = p.gpu_decode(t, self.alpha, mode=mode, select=self.select, recent=self.recent)
        torch.cuda.synchronize()
        p.fetch(rows=self.check_rows)
        og = to_f64(o)
        for i in p.sample:
            Q, K, V = p.host[i]
            oc = self.oc[i]
            r = w.n + t
            _, gpos, _, _, _ = p.gpu_cache_of(i)
            o_ref, a = orc.attend_and_update(oc, Q[r], K[r], V[r], r, self.alpha_of(i))
            _, sw = orc.evict(oc, self.select, self.recent, forced_retained=gpos.tolist(), margin=MARGIN)
            self.swaps += sw
            err = np.abs(og[i] - o_ref).max()
            self.max_o_err = max(self.max_o_err, err)
            assert err <= O_TOL[w.dtype], f"head {i} step {t}: output max-abs {err:.3e}"
            self.max_s_rel = max(self.max_s_rel, compare_cache(
                p, i, oc, f"head {i} step {t}", ordered=self.ascending))


class Replay:
    """Record-and-replay comparison for the full-size configurations.

    The GPU runs the prompt phase and every generation step for all heads without waiting for
    the host; for a sample of heads everything the steps produce is recorded.  Afterwards one
    worker process per head regenerates the head's inputs from its seed and runs the oracle over
    the same prompt and steps (tests/oracle_replay.py), so hundreds of heads are checked element
    by element -- outputs of every step, scores and retained set after every step, the cached
    K/V rows at a few steps -- in the time a handful took in lock-step."""

    def __init__(self, p: Problem, select=None, recent=None):
        self.p = p
        self.select = p.w.select if select is None else select
        self.recent = p.w.recent if recent is None else recent
        self.runs = {i: {} for i in p.sample}
        self.idx = torch.as_tensor(p.sample, device="cuda")
        self.o_err = self.s_rel = 0.0
        self.swaps = 0

    def _state(self, rows):
        c, idx = self.p.cache, self.idx
        lens = c.len[idx].cpu().numpy()
        pos = c.pos[idx].cpu().numpy()
        sc = c.scores[idx].cpu().numpy()
        kv = (c.k[idx].float().cpu().numpy(), c.v[idx].float().cpu().numpy()) if rows else None
        return lens, pos, sc, kv

    def run_gpu(self, alpha, steps=None, mode=a2sf.A2SF_EVICT_FAST, row_steps=None, keep_o=True, tol=None,
                also_exact_scores=False):
        """One prompt phase + `steps` generation steps at forgetting factor `alpha`, recorded.
        tol: the prompt phase runs as a2sf_prefill_windowed with that tolerance; with
        also_exact_scores the scores of a plain a2sf_prefill are recorded beside it."""
        p, w = self.p, self.p.w
        T = w.T if steps is None else steps
        row_steps = {0, T // 2, T - 1} if row_steps is None else set(row_steps)
        s_alt = None
        if also_exact_scores:
            _, s_exact = p.gpu_prefill(alpha, want_o=False, select=self.select, recent=self.recent)
            s_alt = s_exact[self.idx].cpu().numpy()
            del s_exact
        o, s = p.gpu_prefill(alpha, select=self.select, recent=self.recent, tol=tol)
        torch.cuda.synchronize()
        lens, pos, sc, kv = self._state(True)
        o_s = o[self.idx].float().cpu().numpy() if keep_o else None
        s_s = s[self.idx].cpu().numpy()
        for j, i in enumerate(p.sample):
            L = int(lens[j])
            self.runs[i][float(np.float32(alpha))] = {
                "o": None if o_s is None else o_s[j], "s_full": s_s[j],
                "s_full_alt": None if s_alt is None else s_alt[j],
                "pre": (pos[j, :L].copy(), sc[j, :L].copy(), (kv[0][j, :L].copy(), kv[1][j, :L].copy())),
                "fast": mode != a2sf.A2SF_EVICT_STABLE, "steps": []}
        self.s_full = s
        del o
        for t in range(T):
            od = p.gpu_decode(t, alpha, mode=mode, select=self.select, recent=self.recent)
            o_t = od[self.idx].float().cpu().numpy()
            lens, pos, sc, kv = self._state(t in row_steps)
            for j, i in enumerate(p.sample):
                L = int(lens[j])
                self.runs[i][float(np.float32(alpha))]["steps"].append(
                    (o_t[j], pos[j, :L].copy(), sc[j, :L].copy(),
                     None if kv is None else (kv[0][j, :L].copy(), kv[1][j, :L].copy())))
        return s

    def check(self, say=None, workers=None, threads=1):
        """Runs the oracle over every recorded head in worker processes; raises on any mismatch."""
        import multiprocessing as mp
        import os

        import oracle_replay

        p = self.p
        jobs = [{"w": p.w, "g": p.heads[i], "select": self.select, "recent": self.recent,
                 "threads": threads, "runs": self.runs[i]} for i in p.sample]
        if workers is None:
            workers = max(1, min(16, len(os.sched_getaffinity(0)), len(jobs)))
        failures = []
        with mp.get_context("spawn").Pool(workers) as pool:
            for k, r in enumerate(pool.imap_unordered(oracle_replay.replay_head, jobs)):
                self.o_err = max(self.o_err, r["o_err"])
                self.s_rel = max(self.s_rel, r["s_rel"])
                self.swaps += r["swaps"]
                if r["failure"]:
                    failures.append(r["failure"])
                if say and (k + 1) % 64 == 0:
                    say(f"    oracle replay: {k + 1}/{len(jobs)} heads")
        assert not failures, f"{len(failures)} of {len(jobs)} heads differ: " + "; ".join(failures[:5])
        return self
