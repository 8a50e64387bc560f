"""Seeded synthetic workloads shaped like the paper's OPT / LLaMA attention layers.

This module only draws inputs.  It contains none of the method's arithmetic (no softmax,
no score, no selection) and is the one piece of code that both the CPU oracle's tests and
the GPU path's tests/benchmark consume, so that both sides see identical numbers.

Every (layer, batch, head) triple is an independent problem ("head").  A head's arrays come
from its own counter-based Philox stream keyed by (seed, config id, head index), so any
subset of heads can be regenerated without materialising the whole configuration.

Recipe per head (lengths n + T: rows < n are the prompt, row n+t feeds decode step t):
  Q, K, V ~ N(0, 1) in float32;  u = a unit vector drawn from the same stream;
  salient set = {token 0} plus each other position independently with probability p;
  Q_i += u for every i;  K_j += m_j * u for salient j, where m_j = 3 ("fixed") or
  m_j = min(1 + Pareto(1.5), 8) ("pareto"; token 0 gets 8 when the config asks for a sink);
  for bf16 configs the three arrays are then rounded to bf16 (round to nearest even) and
  both sides consume the rounded values.  `logit_shift` (off in the five configurations)
  multiplies the planted component by d^(1/4) on Q and K, which makes the salient logits
  stand out by m instead of m / sqrt(d).
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    cfg_id: int
    name: str
    layers: int
    batch: int
    heads: int
    d: int
    dtype: str            # "f32" or "bf16"
    n: int                # prompt length
    T: int                # decode steps
    select: int
    recent: int
    alphas: tuple
    p_salient: float
    magnitude: str        # "fixed" or "pareto"
    sink: bool = False
    seed: int = 0
    logit_shift: bool = False   # planted component times d^(1/4) on Q and K: shifts in logit units

    @property
    def G(self) -> int:
        return self.layers * self.batch * self.heads

    @property
    def budget(self) -> int:
        return self.select + self.recent

    @property
    def alpha(self) -> float:
        return self.alphas[0]


def _split(ratio: float, n: int):
    """Budget B = floor(ratio*n), select = floor(B/2), recent = B - select."""
    B = int(np.floor(ratio * n + 1e-9))
    return B // 2, B - B // 2


CONFIGS = {
    0: Workload(0, "tiny", 1, 1, 4, 64, "f32", 256, 32, 32, 32, (0.3,), 0.02, "fixed"),
    1: Workload(1, "llama2-7b-layer", 1, 1, 32, 128, "bf16", 1024, 256, *_split(0.2, 1024),
                (0.3,), 0.02, "fixed"),
    2: Workload(2, "batched-decode", 32, 16, 32, 128, "bf16", 2048, 128, 100, 100,
                (0.5,), 0.01, "pareto"),
    3: Workload(3, "opt-13b-shape", 1, 8, 40, 128, "bf16", 4096, 64, *_split(0.1, 4096),
                (0.1,), 0.02, "fixed"),
    4: Workload(4, "long-context", 1, 1, 32, 128, "bf16", 32768, 64, *_split(0.1, 32768),
                (0.1, 0.5, 0.9, 1.0), 0.005, "pareto", sink=True),
}


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def head_arrays(w: Workload, g: int, length: int | None = None):
    """Q, K, V of head ``g`` as float32 [n+T, d] (already bf16-representable for bf16 configs)."""
    total = w.n + w.T if length is None else length
    rng = np.random.Generator(np.random.Philox(key=[(w.seed << 32) | w.cfg_id, g]))
    x = rng.standard_normal((3, total, w.d), dtype=np.float32)
    u = rng.standard_normal(w.d, dtype=np.float32)
    u /= np.sqrt(np.sum(u.astype(np.float64) ** 2)).astype(np.float32)
    salient = rng.random(total) < w.p_salient
    salient[0] = True
    if w.magnitude == "fixed":
        m = np.full(total, 3.0, dtype=np.float32)
    else:
        m = np.minimum(1.0 + rng.pareto(1.5, size=total), 8.0).astype(np.float32)
        if w.sink:
            m[0] = 8.0
    Q, K, V = x[0], x[1], x[2]
    # The literal recipe moves a salient logit by only m / sqrt(d) after the 1/sqrt(d) scale
    # (0.27 at d = 128 for m = 3).  With logit_shift the planted component is scaled by d^(1/4)
    # on both sides, so the shift is m in logit units: strongly peaked attention.
    boost = np.float32(w.d ** 0.25) if w.logit_shift else np.float32(1.0)
    Q += boost * u[None, :]
    K[salient] += boost * m[salient, None] * u[None, :]
    if w.dtype == "bf16":
        Q = bf16_bits_to_f32(round_to_bf16_bits(Q))
        K = bf16_bits_to_f32(round_to_bf16_bits(K))
        V = bf16_bits_to_f32(round_to_bf16_bits(V))
    return Q, K, V


def generate(w: Workload, heads=None, threads: int | None = None, progress=None):
    """Materialise a set of heads in the layouts the library takes.

    Returns a dict of numpy arrays: prompt ``q, k, v`` [H, n, d] and decode inputs
    ``qd, kd, vd`` [T, H, d]; float32 for f32 configs, uint16 bf16 bit patterns for bf16
    ones.  ``heads`` defaults to all G heads of the config.
    """
    heads = list(range(w.G)) if heads is None else list(heads)
    H = len(heads)
    dt = np.float32 if w.dtype == "f32" else np.uint16
    out = {k: np.empty((H, w.n, w.d), dtype=dt) for k in ("q", "k", "v")}
    out.update({k: np.empty((w.T, H, w.d), dtype=dt) for k in ("qd", "kd", "vd")})
    if threads is None:
        threads = max(1, min(16, len(os.sched_getaffinity(0))))

    def one(i):
        Q, K, V = head_arrays(w, heads[i])
        for name, a in (("q", Q), ("k", K), ("v", V)):
            if w.dtype == "bf16":
                a = (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
            out[name][i] = a[:w.n]
            out[name + "d"][:, i, :] = a[w.n:]
        return i

    if threads == 1 or H < 4:
        for i in range(H):
            one(i)
    else:
        with ThreadPoolExecutor(threads) as ex:
            for c, _ in enumerate(ex.map(one, range(H))):
                if progress is not None and (c + 1) % 2048 == 0:
                    progress(c + 1, H)
    return out
