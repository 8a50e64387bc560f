"""Float64 CPU oracle for A2SF (Accumulative Attention Score with Forgetting Factor).

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow, obviously-correct statement of
what the GPU library computes.  Only the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product path never does.  It shares no code with
the HIP path and imports nothing from it.

Everything is numpy float64, one head at a time (the paper keeps a separate score per
layer and per head: Section 2.2 "head-wise Token Pruning", Section 3.1 Eq.2).  Indices
are 0-based: row ``i`` here is query ``q = i+1`` of the paper and the paper's ``n`` is the
number of rows seen so far.

Definitions followed
--------------------
* Masked self-attention (Section 1; Section 3.1 Eq.3): ``P = rowsoftmax(Q K^T / sqrt(d))``
  with every entry above the diagonal forced to probability 0.  The diagonal is kept
  (Eq.4 starts its sum at q = k).
* A2SF score (Section 3.3 Eq.5/Eq.6):  ``A_{n,k} = sum_q alpha^(n-q) * S_{q,k}``; in 0-based
  form ``S_j = sum_{i>=j} alpha^(n-1-i) * P[i, j]``.  ``alpha = 1`` is the plain accumulative
  score of Eq.4; ``alpha = 0`` keeps the newest row only (Section 4.4.2), i.e. 0**0 = 1.
* Generation-step form (abstract; Section 3.3 "repeatedly multiplied"): ``S <- alpha*S + a_t``
  where ``a_t`` is the softmax over the tokens still in the cache (Section 2.2, the remark
  on the softmax denominator after pruning).
* Eviction (Section 2.2, Section 3.1, Section 4.1): tokens with the smallest accumulated
  score leave the cache so that a fixed budget stays; the budget is split into a
  score-selected part and a most-recent part (either may be 0).

* Prompt processed in chunks (beyond the paper, which evicts once per generation step): a chunk
  of m tokens is m generation steps without eviction in between -- each row attends the cached
  tokens and the chunk's tokens up to itself, S <- alpha*S + a row by row -- followed by ONE
  eviction down to the budget.  Written here in matrix form; the tests tie it to the
  step-by-step form, to ``prefill`` (one chunk, empty cache) and to ``decode_step`` (m = 1).
* Grouped-query heads (beyond the paper, whose models are all multi-head): r query heads share
  one K/V head, so a token is kept or evicted for the whole group.  Reading: the group's score
  of a token is the SUM of its query heads' accumulated scores, as Eq.1 of the paper sums over
  heads where one pruning decision serves all of them.

* Similarity to the Ideal mask (Section 4.3, Table 2): at every generation step the Ideal
  computes the attention of the query over ALL earlier tokens (nothing is ever removed) and
  keeps the entries of the tokens with the largest attention score, as many as the cache
  allows; a pruning method's row has entries only on the tokens still in its cache.  The
  figure of merit is the cosine between the two rows, averaged over steps.

Readings where the paper is silent:
ties go to the lower original position; exactly ``len - budget`` tokens leave per step;
selection after the prompt happens once, on the scores of the whole prompt.

Parity status: every function here is pinned by tests that do not re-use its own formula
(closed-form geometric sum, harmonic-number special case, brute-force triple loops,
alpha=0 / alpha=1 reductions, decode-vs-prefill consistency, exhaustive subset search).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "causal_probabilities", "attention_output", "forgotten_scores",
    "forgotten_scores_recurrence", "forgotten_scores_streamed", "select_keep",
    "HeadCache", "prefill", "attend_and_update", "evict", "decode_step",
    "pruned_row", "ideal_row", "cosine_similarity", "similarity_to_ideal",
    "chunk_attend_and_update", "prefill_chunk", "gqa_prefill", "gqa_attend_and_update",
    "gqa_decode_step", "gqa_chunk_attend_and_update", "gqa_prefill_chunk",
]


# --------------------------------------------------------------------------- attention
def causal_probabilities(Q: np.ndarray, K: np.ndarray) -> np.ndarray:
    """Masked softmax matrix P[i, j] of one head (Section 1; Section 3.1 Eq.3).

    Q, K: [n, d].  Returns [n, n] float64, zero above the diagonal, rows summing to 1.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n, d = Q.shape
    s = (Q @ K.T) / np.sqrt(float(d))
    future = np.triu(np.ones((n, n), dtype=bool), k=1)
    s[future] = -np.inf
    s -= s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def attention_output(P: np.ndarray, V: np.ndarray) -> np.ndarray:
    """O = P V (the attention layer's output rows)."""
    return np.asarray(P, dtype=np.float64) @ np.asarray(V, dtype=np.float64)


# --------------------------------------------------------------------------- scores
def _weights(n: int, alpha: float) -> np.ndarray:
    """w_i = alpha^(n-1-i) with w_{n-1} = 1 for every alpha (0**0 = 1)."""
    e = np.arange(n - 1, -1, -1, dtype=np.float64)
    w = np.power(float(alpha), e)
    w[n - 1] = 1.0
    return w


def forgotten_scores(P: np.ndarray, alpha: float) -> np.ndarray:
    """Closed form of Eq.5: S_j = sum_i alpha^(n-1-i) P[i, j]."""
    P = np.asarray(P, dtype=np.float64)
    return _weights(P.shape[0], alpha) @ P


def forgotten_scores_recurrence(P: np.ndarray, alpha: float) -> np.ndarray:
    """Generation-step form: start from 0, for each row S <- alpha*S + P[i, :]."""
    P = np.asarray(P, dtype=np.float64)
    S = np.zeros(P.shape[1], dtype=np.float64)
    for i in range(P.shape[0]):
        S = float(alpha) * S + P[i]
    return S


def forgotten_scores_streamed(Q, K, alphas, V=None, rows_per_chunk: int = 512):
    """Eq.5 for long prompts without holding the n x n matrix: softmax rows are formed a
    chunk of rows at a time (each row is complete, so nothing about the definition
    changes) and added with their closed-form weight.  P does not depend on alpha, so
    several alphas are served by one sweep.  Returns {alpha: S[n]}, and with ``V`` given
    (S_by_alpha, O[n, d]).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n, d = Q.shape
    out = {float(a): np.zeros(n, dtype=np.float64) for a in alphas}
    w = {a: _weights(n, a) for a in out}
    O = None
    if V is not None:
        V = np.asarray(V, dtype=np.float64)
        O = np.zeros((n, V.shape[1]), dtype=np.float64)
    for r0 in range(0, n, rows_per_chunk):
        r1 = min(n, r0 + rows_per_chunk)
        s = (Q[r0:r1] @ K[:r1].T) / np.sqrt(float(d))
        rows = np.arange(r0, r1)[:, None]
        cols = np.arange(r1)[None, :]
        s[cols > rows] = -np.inf
        s -= s.max(axis=1, keepdims=True)
        e = np.exp(s)
        p = e / e.sum(axis=1, keepdims=True)
        for a in out:
            out[a][:r1] += w[a][r0:r1] @ p
        if O is not None:
            O[r0:r1] = p @ V[:r1]
    return out if O is None else (out, O)


# --------------------------------------------------------------------------- selection
def select_keep(scores, pos, select: int, recent: int) -> np.ndarray:
    """Which cached tokens survive (Section 2.2 / 3.1 eviction, Section 4.1 budget split).

    scores, pos: [L].  The ``recent`` tokens with the largest original position are
    always kept; of the others the ``select`` with the largest score are kept, a tie
    going to the lower original position.  If L <= select+recent everything is kept.
    Returns slot indices, ordered by ascending original position.
    """
    scores = np.asarray(scores, dtype=np.float64)
    pos = np.asarray(pos)
    L = scores.shape[0]
    if L <= select + recent:
        keep = list(range(L))
    else:
        by_age = sorted(range(L), key=lambda s: int(pos[s]))
        newest = by_age[L - recent:] if recent > 0 else []
        older = by_age[:L - recent] if recent > 0 else by_age
        ranked = sorted(older, key=lambda s: (-scores[s], int(pos[s])))
        keep = ranked[:select] + newest
    keep.sort(key=lambda s: int(pos[s]))
    return np.asarray(keep, dtype=np.int64)


def _resolve_keep(S, pos, select, recent, forced_retained, margin):
    """select_keep, or the caller's forced survivor set if it is a legitimate in-margin
    variant of it (see ``evict``).  Returns (slot indices by ascending position, n_swapped)."""
    keep = select_keep(S, pos, select, recent)
    if forced_retained is None:
        return keep, 0
    want = set(int(p) for p in forced_retained)
    own = set(int(p) for p in np.asarray(pos)[keep])
    if want == own:
        return keep, 0
    by_pos = {int(p): s for s, p in enumerate(pos)}
    if len(want) != len(own) or not want <= set(by_pos):
        raise ValueError("forced retained set has the wrong size or unknown tokens")
    L = len(by_pos)
    newest = set(sorted(by_pos)[L - recent:]) if recent > 0 else set()
    if not newest <= want:
        raise ValueError("forced retained set drops a token of the recent window")
    moved = (own - want) | (want - own)
    vals = [float(S[by_pos[p]]) for p in moved]
    if max(vals) - min(vals) > margin:
        raise ValueError("forced retained set differs outside the margin: spread "
                         f"{max(vals) - min(vals):.3e}")
    keep = np.asarray(sorted((by_pos[p] for p in want), key=lambda s: int(pos[s])),
                      dtype=np.int64)
    return keep, len(own - want)


# --------------------------------------------------------------------------- cache
class HeadCache:
    """Retained tokens of one head: K rows, V rows, accumulated score, original position."""

    def __init__(self, K, V, S, pos):
        self.K = np.array(K, dtype=np.float64)
        self.V = np.array(V, dtype=np.float64)
        self.S = np.array(S, dtype=np.float64)
        self.pos = np.array(pos, dtype=np.int64)

    def __len__(self):
        return int(self.pos.shape[0])

    def copy(self):
        return HeadCache(self.K, self.V, self.S, self.pos)

    def sorted_by_pos(self):
        o = np.argsort(self.pos, kind="stable")
        return HeadCache(self.K[o], self.V[o], self.S[o], self.pos[o])


def prefill(Q, K, V, alpha: float, select: int, recent: int, forced_retained=None,
            margin: float = 1e-6):
    """Prompt phase of one head.

    Full causal attention over the n prompt tokens, Eq.5 scores of all of them, then one
    selection down to the budget (``forced_retained`` as in ``evict``).
    Returns (O[n, d], S_full[n], HeadCache).
    """
    P = causal_probabilities(Q, K)
    O = attention_output(P, V)
    S_full = forgotten_scores(P, alpha)
    n = P.shape[0]
    keep, _ = _resolve_keep(S_full, np.arange(n), select, recent, forced_retained, margin)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    return O, S_full, HeadCache(K[keep], V[keep], S_full[keep], keep)


def attend_and_update(cache: HeadCache, q, k_new, v_new, t_pos: int, alpha: float):
    """First half of a generation step, in place on ``cache`` (no eviction yet).

    Append the new token with score 0; a = softmax(K_c q / sqrt(d)) over the cached tokens
    only (Section 2.2: pruning changes the softmax denominator); o = a^T V_c; then the
    forgetting update S <- alpha*S + a on every cached token (abstract; Section 3.3).
    Returns (o[d], a[L]) with a in slot order of the grown cache.
    """
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[0]
    cache.K = np.vstack([cache.K, np.asarray(k_new, dtype=np.float64)[None, :]])
    cache.V = np.vstack([cache.V, np.asarray(v_new, dtype=np.float64)[None, :]])
    cache.S = np.append(cache.S, 0.0)
    cache.pos = np.append(cache.pos, int(t_pos))
    z = (cache.K @ q) / np.sqrt(float(d))
    z -= z.max()
    e = np.exp(z)
    a = e / e.sum()
    o = a @ cache.V
    cache.S = float(alpha) * cache.S + a
    return o, a


def evict(cache: HeadCache, select: int, recent: int, forced_retained=None,
          margin: float = 1e-6):
    """Second half of a generation step: drop tokens until the budget holds, in place.

    ``forced_retained`` (an iterable of original positions) replaces the oracle's own
    choice of survivors.  It exists because two scores closer than ``margin`` may be
    ordered differently by an fp32 implementation; after such a legitimate swap every
    later step differs, so a lock-step comparison must be able to follow the other side.
    It is accepted only when it keeps the whole recent window, has the right size, and
    every token it swaps in or out has a score within ``margin`` of all the others
    swapped; otherwise ValueError.

    Returns (evicted_positions, n_swapped).
    """
    keep, swaps = _resolve_keep(cache.S, cache.pos, select, recent, forced_retained, margin)
    gone = sorted(set(int(p) for p in cache.pos) - set(int(p) for p in cache.pos[keep]))
    cache.K, cache.V = cache.K[keep], cache.V[keep]
    cache.S, cache.pos = cache.S[keep], cache.pos[keep]
    return gone, swaps


def decode_step(cache: HeadCache, q, k_new, v_new, t_pos: int, alpha: float,
                select: int, recent: int, forced_retained=None, margin: float = 1e-6):
    """One whole generation step of one head: attend_and_update, then evict.

    Eviction at the end of the step that overfilled the cache is the same computation as
    eviction "in the next Generation Step" before its append (Section 3.1): nothing reads
    the cache in between.  Returns (o[d], a[L], evicted_positions, n_swapped).
    """
    o, a = attend_and_update(cache, q, k_new, v_new, t_pos, alpha)
    gone, swaps = evict(cache, select, recent, forced_retained, margin)
    return o, a, gone, swaps


# --------------------------------------------------------------------------- chunks of a prompt
def chunk_attend_and_update(cache: HeadCache, Qc, Kc, Vc, pos0: int, alpha: float):
    """A chunk of m new tokens against a cache of L earlier ones, in place, no eviction yet.

    Row i of the chunk attends every cached token and the chunk's tokens 0..i (softmax over
    exactly those: Section 2.2, Section 3.1 Eq.3 for the masked part); O = P [V_c; Vc].
    Scores: the recurrence S <- alpha*S + a (abstract; Section 3.3) applied once per row, i.e.
    a cached token ends with alpha^m S_j + sum_i alpha^(m-1-i) P[i, j] and chunk token c with
    sum_{i>=c} alpha^(m-1-i) P[i, L+c] (Eq.5 restricted to the rows that exist).  The chunk's
    tokens get positions pos0 .. pos0+m-1.  Returns (O[m, d], P[m, L+m])."""
    Qc, Kc, Vc = (np.asarray(x, dtype=np.float64) for x in (Qc, Kc, Vc))
    m, d = Qc.shape
    L = len(cache)
    K_all = np.vstack([cache.K.reshape(L, d), Kc])
    V_all = np.vstack([cache.V.reshape(L, d), Vc])
    s = (Qc @ K_all.T) / np.sqrt(float(d))
    rows = np.arange(m)[:, None]
    cols = np.arange(L + m)[None, :]
    s[cols > L + rows] = -np.inf            # chunk token c is visible to chunk rows i >= c only
    s -= s.max(axis=1, keepdims=True)
    e = np.exp(s)
    P = e / e.sum(axis=1, keepdims=True)
    O = P @ V_all
    S_old = np.concatenate([cache.S, np.zeros(m, dtype=np.float64)])
    decay = float(alpha) ** m               # 0**m = 0 for m >= 1: alpha = 0 forgets everything older
    cache.S = decay * S_old + _weights(m, alpha) @ P
    cache.K, cache.V = K_all, V_all
    cache.pos = np.concatenate([cache.pos, np.arange(pos0, pos0 + m, dtype=np.int64)])
    return O, P


def prefill_chunk(cache: HeadCache, Qc, Kc, Vc, pos0: int, alpha: float, select: int, recent: int,
                  forced_retained=None, margin: float = 1e-6):
    """chunk_attend_and_update, then one eviction down to the budget (``evict``).
    Returns (O[m, d], evicted_positions, n_swapped)."""
    O, _ = chunk_attend_and_update(cache, Qc, Kc, Vc, pos0, alpha)
    gone, swaps = evict(cache, select, recent, forced_retained, margin)
    return O, gone, swaps


# --------------------------------------------------------------------------- grouped-query heads
def gqa_prefill(Qs, K, V, alpha: float, select: int, recent: int, forced_retained=None,
                margin: float = 1e-6):
    """Prompt phase of one K/V head shared by r query heads.  Qs: [r, n, d]; K, V: [n, d].

    Every query head has its own masked softmax and output; the score of a token is the sum of
    the r heads' Eq.5 scores, and one selection on that sum serves the whole group.
    Returns (O[r, n, d], S_full[n], HeadCache)."""
    Qs = np.asarray(Qs, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    r, n, _ = Qs.shape
    O = np.zeros((r, n, V.shape[1]), dtype=np.float64)
    S_full = np.zeros(n, dtype=np.float64)
    for h in range(r):
        P = causal_probabilities(Qs[h], K)
        O[h] = attention_output(P, V)
        S_full += forgotten_scores(P, alpha)
    keep, _ = _resolve_keep(S_full, np.arange(n), select, recent, forced_retained, margin)
    return O, S_full, HeadCache(K[keep], V[keep], S_full[keep], keep)


def gqa_attend_and_update(cache: HeadCache, qs, k_new, v_new, t_pos: int, alpha: float):
    """First half of a generation step of one K/V head with r query heads (qs: [r, d]), in
    place: every query head takes its own softmax over the cached tokens and its own output;
    the forgetting update adds the SUM of the r probability rows.  Returns (o[r, d], a[r, L])."""
    qs = np.asarray(qs, dtype=np.float64)
    r, d = qs.shape
    cache.K = np.vstack([cache.K.reshape(-1, d), np.asarray(k_new, dtype=np.float64)[None, :]])
    cache.V = np.vstack([cache.V.reshape(-1, d), np.asarray(v_new, dtype=np.float64)[None, :]])
    cache.S = np.append(cache.S, 0.0)
    cache.pos = np.append(cache.pos, int(t_pos))
    z = (qs @ cache.K.T) / np.sqrt(float(d))
    z -= z.max(axis=1, keepdims=True)
    e = np.exp(z)
    a = e / e.sum(axis=1, keepdims=True)
    o = a @ cache.V
    cache.S = float(alpha) * cache.S + a.sum(axis=0)
    return o, a


def gqa_decode_step(cache: HeadCache, qs, k_new, v_new, t_pos: int, alpha: float, select: int,
                    recent: int, forced_retained=None, margin: float = 1e-6):
    """gqa_attend_and_update, then ``evict``.  Returns (o[r, d], a[r, L], evicted, n_swapped)."""
    o, a = gqa_attend_and_update(cache, qs, k_new, v_new, t_pos, alpha)
    gone, swaps = evict(cache, select, recent, forced_retained, margin)
    return o, a, gone, swaps


def gqa_chunk_attend_and_update(cache: HeadCache, Qcs, Kc, Vc, pos0: int, alpha: float):
    """A chunk of m new tokens of one K/V head with r query heads (Qcs: [r, m, d]; Kc, Vc: [m, d])
    against a cache of L earlier tokens, in place, no eviction yet.  Every query head attends as
    a single head's chunk does (``chunk_attend_and_update``: the cached tokens and the chunk's
    tokens up to its own), with its own softmax and output; the scores take the recurrence
    S <- alpha*S + (sum of the r heads' probability rows) once per chunk row, i.e. a cached
    token ends with alpha^m S_j + sum_h sum_i alpha^(m-1-i) P_h[i, j].
    Returns (O[r, m, d], P[r, m, L+m])."""
    Qcs = np.asarray(Qcs, dtype=np.float64)
    Kc, Vc = (np.asarray(x, dtype=np.float64) for x in (Kc, Vc))
    r, m, d = Qcs.shape
    L = len(cache)
    K_all = np.vstack([cache.K.reshape(L, d), Kc])
    V_all = np.vstack([cache.V.reshape(L, d), Vc])
    rows = np.arange(m)[:, None]
    cols = np.arange(L + m)[None, :]
    O = np.zeros((r, m, d), dtype=np.float64)
    P = np.zeros((r, m, L + m), dtype=np.float64)
    S_new = (float(alpha) ** m) * np.concatenate([cache.S, np.zeros(m, dtype=np.float64)])
    for h in range(r):
        s = (Qcs[h] @ K_all.T) / np.sqrt(float(d))
        s[np.broadcast_to(cols > L + rows, s.shape)] = -np.inf
        s -= s.max(axis=1, keepdims=True)
        e = np.exp(s)
        P[h] = e / e.sum(axis=1, keepdims=True)
        O[h] = P[h] @ V_all
        S_new += _weights(m, alpha) @ P[h]
    cache.S = S_new
    cache.K, cache.V = K_all, V_all
    cache.pos = np.concatenate([cache.pos, np.arange(pos0, pos0 + m, dtype=np.int64)])
    return O, P


def gqa_prefill_chunk(cache: HeadCache, Qcs, Kc, Vc, pos0: int, alpha: float, select: int, recent: int,
                      forced_retained=None, margin: float = 1e-6):
    """gqa_chunk_attend_and_update, then one eviction down to the budget (``evict``).
    Returns (O[r, m, d], evicted_positions, n_swapped)."""
    O, _ = gqa_chunk_attend_and_update(cache, Qcs, Kc, Vc, pos0, alpha)
    gone, swaps = evict(cache, select, recent, forced_retained, margin)
    return O, gone, swaps


# --------------------------------------------------------------------------- similarity to Ideal
def _logits(q, K) -> np.ndarray:
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    return (K @ q) / np.sqrt(float(K.shape[1]))


def pruned_row(q, K, retained) -> np.ndarray:
    """Attention row of one query when only the tokens `retained` (positions, rows of K) can
    be attended: softmax over those tokens (Section 2.2: after pruning the denominator runs
    over what is left), zero everywhere else.  K: [L, d], all tokens so far; returns [L]."""
    s = _logits(q, K)
    idx = np.asarray(sorted(int(p) for p in retained), dtype=np.int64)
    if len(idx) == 0 or idx[0] < 0 or idx[-1] >= len(s) or len(set(idx.tolist())) != len(idx):
        raise ValueError("retained positions must be distinct rows of K")
    e = np.exp(s[idx] - s[idx].max())
    row = np.zeros(len(s), dtype=np.float64)
    row[idx] = e / e.sum()
    return row


def ideal_row(q, K, keep: int) -> np.ndarray:
    """Row of the Ideal mask (Section 4.3): the query attends all L tokens so far, the `keep`
    tokens with the largest attention score are selected (tie -> lower position, as
    everywhere here), and the row is the attention restricted to them.  Which tokens were
    selected at earlier steps plays no role: nothing is removed for good."""
    if keep < 1:
        raise ValueError("keep must be at least 1")
    s = _logits(q, K)
    order = sorted(range(len(s)), key=lambda j: (-s[j], j))
    return pruned_row(q, K, order[:min(int(keep), len(s))])


def cosine_similarity(u, v) -> float:
    u = np.asarray(u, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    return float(np.dot(u, v) / np.sqrt(np.dot(u, u) * np.dot(v, v)))


def similarity_to_ideal(Q, K, V, alpha: float, select: int, recent: int, forced_retained=None,
                        margin: float = 1e-6):
    """Table 2 protocol on one head: the sequence is generated token by token from an empty
    cache under the policy (alpha, select, recent); at step i the policy's row has entries on
    its cached tokens and on token i itself, the Ideal row on equally many tokens.

    forced_retained: optional list, per step i >= 1, of the positions the caller's cache holds
    after that step (see ``evict``).  Returns (cos[n], cache after the last step)."""
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    n = Q.shape[0]
    _, _, cache = prefill(Q[:1], K[:1], V[:1], alpha, select, recent)
    cos = np.ones(n, dtype=np.float64)     # step 0: one token, both rows are [1]
    for i in range(1, n):
        retained = [int(p) for p in cache.pos] + [i]
        cos[i] = cosine_similarity(pruned_row(Q[i], K[:i + 1], retained),
                                   ideal_row(Q[i], K[:i + 1], len(retained)))
        decode_step(cache, Q[i], K[i], V[i], i, alpha, select, recent,
                    None if forced_retained is None else forced_retained[i], margin)
    return cos, cache
