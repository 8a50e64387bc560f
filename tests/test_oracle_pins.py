"""Pins for the float64 oracle: every check here rests on something other than the oracle's
own formulas - closed forms, exact rationals, brute-force loops over explicit attention
matrices, the alpha = 0 / alpha = 1 reductions, exhaustive subset search, and consistency
between the prompt form (Section 3.3 Eq.5) and the generation-step form of the score.
The last class plants plausible mistakes in the oracle (on the CPU) and checks that the
pins notice each of them.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import a2sf_oracle as orc

RNG = np.random.default_rng(20240720)


def rand_head(n, d, scale=1.0, rng=RNG):
    return (rng.standard_normal((n, d)) * scale, rng.standard_normal((n, d)) * scale,
            rng.standard_normal((n, d)))


# ---------------------------------------------------------------- brute force (pure loops)
def brute_probabilities(Q, K):
    """Section 3.1 Eq.3 and the masked softmax of Section 1 with explicit loops."""
    n, d = len(Q), len(Q[0])
    P = [[0.0] * n for _ in range(n)]
    for i in range(n):
        logit = []
        for j in range(i + 1):
            acc = 0.0
            for c in range(d):
                acc += Q[i][c] * K[j][c]
            logit.append(acc / math.sqrt(d))
        top = max(logit)
        ex = [math.exp(x - top) for x in logit]
        tot = math.fsum(ex)
        for j in range(i + 1):
            P[i][j] = ex[j] / tot
    return P


def brute_scores(P, alpha):
    """Section 3.3 Eq.6 term by term: S_{n,k} + alpha S_{n-1,k} + alpha^2 S_{n-2,k} + ..."""
    n = len(P)
    out = []
    for k in range(n):
        terms = []
        for back in range(0, n - k):          # back = n-1-i
            i = n - 1 - back
            wt = 1.0
            for _ in range(back):
                wt *= alpha
            terms.append(wt * P[i][k])
        out.append(math.fsum(terms))
    return out


class TestAttentionMatrix:
    def test_brute_force_matrix(self):
        Q, K, V = rand_head(24, 8)
        P = orc.causal_probabilities(Q, K)
        Pb = np.array(brute_probabilities(Q.tolist(), K.tolist()))
        assert np.abs(P - Pb).max() < 1e-14

    def test_mask_rows_and_diagonal(self):
        Q, K, _ = rand_head(40, 16)
        P = orc.causal_probabilities(Q, K)
        assert np.all(np.triu(P, k=1) == 0.0)           # Eq.3: exactly zero above the diagonal
        assert np.all(np.diag(P) > 0.0)                  # Eq.4: q = k term is present
        assert P[0, 0] == 1.0
        assert np.abs(P.sum(axis=1) - 1.0).max() < 1e-14

    def test_scale_is_one_over_sqrt_d(self):
        # two keys, one query: P ratio must be exp((q.k0 - q.k1)/sqrt(d))
        d = 16
        q = np.ones((2, d))
        K = np.stack([np.full(d, 0.5), np.full(d, -0.25)])
        P = orc.causal_probabilities(q, K)
        assert math.isclose(P[1, 0] / P[1, 1], math.exp((8.0 + 4.0) / 4.0), rel_tol=1e-13)

    def test_not_transposed(self):
        # Make key 0 attractive only: column 0 large for all rows, row 0 is [1, 0, ...].
        n, d = 6, 4
        Q = np.ones((n, d))
        K = np.zeros((n, d))
        K[0] = 5.0
        P = orc.causal_probabilities(Q, K)
        assert np.all(P[1:, 0] > 0.99)

    def test_output_uniform_attention(self):
        n, d = 10, 4
        V = RNG.standard_normal((n, d))
        P = orc.causal_probabilities(np.zeros((n, d)), RNG.standard_normal((n, d)))
        O = orc.attention_output(P, V)
        running = np.cumsum(V, axis=0) / np.arange(1, n + 1)[:, None]
        assert np.abs(O - running).max() < 1e-14


class TestForgottenScore:
    @pytest.mark.parametrize("alpha", [0.0, 0.1, 0.3, 0.5, 0.9, 1.0])
    def test_brute_force_eq6(self, alpha):
        Q, K, _ = rand_head(20, 8)
        Pb = brute_probabilities(Q.tolist(), K.tolist())
        S = orc.forgotten_scores(np.array(Pb), alpha)
        assert np.abs(S - np.array(brute_scores(Pb, alpha))).max() < 1e-14

    @pytest.mark.parametrize("alpha,n", [(0.3, 256), (0.5, 64), (0.9, 100), (0.1, 7)])
    def test_geometric_total(self, alpha, n):
        Q, K, _ = rand_head(n, 8)
        S = orc.forgotten_scores(orc.causal_probabilities(Q, K), alpha)
        assert math.isclose(S.sum(), (1 - alpha ** n) / (1 - alpha), rel_tol=1e-12)

    def test_totals_at_the_ends(self):
        Q, K, _ = rand_head(33, 8)
        P = orc.causal_probabilities(Q, K)
        assert math.isclose(orc.forgotten_scores(P, 1.0).sum(), 33.0, rel_tol=1e-13)
        assert math.isclose(orc.forgotten_scores(P, 0.0).sum(), 1.0, rel_tol=1e-13)

    def test_alpha_one_is_plain_accumulation(self):     # Section 3.1 Eq.4
        Q, K, _ = rand_head(50, 8)
        P = orc.causal_probabilities(Q, K)
        assert np.abs(orc.forgotten_scores(P, 1.0) - P.sum(axis=0)).max() < 1e-13

    def test_alpha_zero_is_last_row(self):              # Section 4.4.2
        Q, K, _ = rand_head(50, 8)
        P = orc.causal_probabilities(Q, K)
        assert np.array_equal(orc.forgotten_scores(P, 0.0), P[-1])

    @pytest.mark.parametrize("alpha", [0.0, 0.3, 1.0])
    def test_recurrence_equals_closed_form(self, alpha):
        Q, K, _ = rand_head(64, 8)
        P = orc.causal_probabilities(Q, K)
        assert np.abs(orc.forgotten_scores(P, alpha)
                      - orc.forgotten_scores_recurrence(P, alpha)).max() < 1e-13

    def test_harmonic_fixture(self):
        """Uniform attention (Q = 0): exact rationals from tests/golden (H_n - H_j at alpha=1)."""
        path = os.path.join(os.path.dirname(__file__), "golden", "harmonic_uniform_attention.txt")
        rows = [l.split() for l in open(path) if not l.startswith("#")]
        n = int(rows[0][0])
        P = orc.causal_probabilities(np.zeros((n, 4)), RNG.standard_normal((n, 4)))
        seen = 0
        for _, an, ad, j, sn, sd in rows:
            alpha = int(an) / int(ad)
            S = orc.forgotten_scores(P, alpha)
            assert math.isclose(S[int(j)], int(sn) / int(sd), rel_tol=1e-14)
            seen += 1
        assert seen == 2 * n
        # textbook: H_12 = 86021/27720
        assert math.isclose(orc.forgotten_scores(P, 1.0)[0], 86021 / 27720, rel_tol=1e-14)

    def test_early_token_bias_of_plain_accumulation(self):   # Section 3.1, after Eq.4
        n = 30
        P = orc.causal_probabilities(np.zeros((n, 4)), np.zeros((n, 4)))
        S1 = orc.forgotten_scores(P, 1.0)
        assert np.all(np.diff(S1) < 0)
        exact = [float(sum(Fraction(1, i + 1) for i in range(j, n))) for j in range(n)]
        assert np.abs(S1 - np.array(exact)).max() < 1e-14

    def test_truncation_bound(self):
        n, W, alpha = 200, 12, 0.3
        Q, K, _ = rand_head(n, 8)
        P = orc.causal_probabilities(Q, K)
        full = orc.forgotten_scores(P, alpha)
        Pt = P.copy()
        Pt[: n - W] = 0.0
        cut = orc.forgotten_scores(Pt, alpha)
        bound = alpha ** W / (1 - alpha) * P[: n - W].max(axis=0)
        assert np.all(full - cut >= 0) and np.all(full - cut <= bound + 1e-18)

    @pytest.mark.parametrize("alpha", [0.1, 0.5, 0.9])
    @pytest.mark.parametrize("spread", [1.0, 4.0])
    def test_window_from_the_newest_row_keeps_the_relative_error(self, alpha, spread):
        """The a-priori row window of a2sf_prefill_windowed, stated on the oracle: all rows before
        n - W add at most alpha^W / (1 - alpha) to any score while S_j >= P[n-1, j], so with
        alpha^W <= tol (1 - alpha) min_j P[n-1, j] (the minimum over a group of keys) every score
        of the group keeps a relative error <= tol when those rows are dropped."""
        n, d, tol, group = 600, 16, 2.5e-5, 64
        rng = np.random.default_rng(int(alpha * 100 + spread))
        Q = spread * rng.standard_normal((n, d))
        K = rng.standard_normal((n, d))
        P = orc.causal_probabilities(Q, K)
        full = orc.forgotten_scores(P, alpha)
        for j0 in range(0, n, group):
            p_min = P[n - 1, j0:j0 + group].min()
            W = int(np.ceil(np.log(tol * (1 - alpha) * p_min) / np.log(alpha)))
            assert W >= 1
            Pt = P.copy()
            Pt[: max(0, n - W)] = 0.0
            cut = orc.forgotten_scores(Pt, alpha)[j0:j0 + group]
            rel = (full[j0:j0 + group] - cut) / full[j0:j0 + group]
            assert np.all(rel >= 0) and rel.max() <= tol, (j0, W, rel.max())

    def test_streamed_equals_matrix_form(self):
        Q, K, V = rand_head(300, 16)
        P = orc.causal_probabilities(Q, K)
        got, O = orc.forgotten_scores_streamed(Q, K, [0.0, 0.4, 1.0], V=V, rows_per_chunk=37)
        for a in (0.0, 0.4, 1.0):
            assert np.abs(got[a] - orc.forgotten_scores(P, a)).max() < 1e-13
        assert np.abs(O - orc.attention_output(P, V)).max() < 1e-13

    def test_heads_are_independent(self):
        heads = [rand_head(32, 8) for _ in range(3)]
        a = [orc.prefill(*h, 0.3, 4, 4)[1] for h in heads]
        b = [orc.prefill(*h, 0.3, 4, 4)[1] for h in reversed(heads)]
        for x, y in zip(a, reversed(b)):
            assert np.array_equal(x, y)


# ---------------------------------------------------------------- selection
def exhaustive_keep(scores, pos, select, recent):
    """Among all subsets that hold the `recent` newest tokens plus `select` others, the one
    with the largest score total; ties between equal-score tokens resolved by preferring the
    lexicographically smallest position list.  Built without sorting by score."""
    L = len(scores)
    if L <= select + recent:
        return sorted(range(L), key=lambda s: pos[s])
    order = sorted(range(L), key=lambda s: pos[s])
    newest = order[L - recent:] if recent else []
    older = order[:L - recent] if recent else order
    best, best_key = None, None
    for sub in itertools.combinations(older, select):
        key = (-math.fsum(scores[s] for s in sub), sorted(pos[s] for s in sub))
        if best_key is None or key < best_key:
            best, best_key = sub, key
    return sorted(list(best) + newest, key=lambda s: pos[s])


class TestSelection:
    @pytest.mark.parametrize("seed", range(6))
    def test_exhaustive(self, seed):
        r = np.random.default_rng(seed)
        L = int(r.integers(5, 11))
        select, recent = int(r.integers(0, 4)), int(r.integers(0, 4))
        if select + recent == 0:
            select = 1
        # dyadic scores: sums are exact, so the brute-force comparison is exact
        scores = r.integers(0, 6, size=L) / 8.0
        pos = r.permutation(50)[:L]
        got = orc.select_keep(scores, pos, select, recent)
        assert list(got) == exhaustive_keep(scores.tolist(), pos.tolist(), select, recent)

    def test_all_equal_keeps_lowest_positions(self):
        got = orc.select_keep(np.ones(10), np.arange(10), 3, 2)
        assert list(got) == [0, 1, 2, 8, 9]

    def test_tie_at_the_cut_goes_to_lower_position(self):
        scores = np.array([0.5, 0.2, 0.2, 0.9, 0.2, 0.1])
        got = orc.select_keep(scores, np.arange(6), 3, 1)
        assert list(got) == [0, 1, 3, 5]

    def test_recent_is_by_position_not_slot(self):
        scores = np.array([9.0, 0.0, 9.0, 0.0])
        pos = np.array([7, 100, 3, 50])
        got = orc.select_keep(scores, pos, 1, 1)
        assert sorted(pos[got]) == [3, 100]          # newest pos kept; tie 9.0 -> lower pos 3
        assert list(pos[got]) == sorted(pos[got])    # ascending position

    def test_keeps_everything_under_budget(self):
        assert list(orc.select_keep(np.zeros(5), np.arange(5), 4, 4)) == [0, 1, 2, 3, 4]

    def test_pure_policies(self):
        s = np.array([0.1, 0.9, 0.3, 0.8, 0.2])
        assert list(orc.select_keep(s, np.arange(5), 0, 2)) == [3, 4]       # local window
        assert list(orc.select_keep(s, np.arange(5), 2, 0)) == [1, 3]       # the paper's A2SF split


# ---------------------------------------------------------------- generation steps
class TestDecode:
    def test_no_eviction_matches_prompt_form(self):
        """With a budget that never binds, prefill(n) + T steps must equal full causal attention
        over n+T tokens: outputs are its rows, scores its Eq.5 scores."""
        n, T, d, alpha = 40, 17, 8, 0.35
        Q, K, V = rand_head(n + T, d)
        P = orc.causal_probabilities(Q, K)
        O_full = orc.attention_output(P, V)
        _, _, cache = orc.prefill(Q[:n], K[:n], V[:n], alpha, n + T, 0)
        for t in range(T):
            o, a, gone, _ = orc.decode_step(cache, Q[n + t], K[n + t], V[n + t], n + t, alpha, n + T, 0)
            assert gone == []
            assert np.abs(o - O_full[n + t]).max() < 1e-13
            assert np.abs(a - P[n + t, : n + t + 1]).max() < 1e-14
        assert np.abs(cache.S - orc.forgotten_scores(P, alpha)).max() < 1e-13
        assert list(cache.pos) == list(range(n + T))

    def test_step_invariants_with_eviction(self):
        n, T, d, alpha, sel, rec = 64, 30, 8, 0.3, 6, 5
        Q, K, V = rand_head(n + T, d)
        _, _, cache = orc.prefill(Q[:n], K[:n], V[:n], alpha, sel, rec)
        assert len(cache) == sel + rec
        for t in range(T):
            before = cache.S.sum()
            grown = cache.copy()
            o, a = orc.attend_and_update(grown, Q[n + t], K[n + t], V[n + t], n + t, alpha)
            assert np.all(a >= 0) and math.isclose(a.sum(), 1.0, rel_tol=1e-13)
            assert math.isclose(grown.S.sum(), alpha * before + 1.0, rel_tol=1e-13)
            assert grown.S[-1] == a[-1]                      # the new token started from 0
            o2, a2, gone, _ = orc.decode_step(cache, Q[n + t], K[n + t], V[n + t], n + t, alpha, sel, rec)
            assert np.array_equal(o, o2)
            assert len(gone) == 1 and len(cache) == sel + rec
            assert np.all(np.diff(cache.pos) > 0)
            assert list(cache.pos[-rec:]) == list(range(n + t - rec + 1, n + t + 1))
            # the evicted token was the worst non-recent one
            worst = min((grown.S[s], -grown.pos[s]) for s in range(len(grown))
                        if grown.pos[s] <= n + t - rec)
            assert -worst[1] == gone[0]

    def test_softmax_is_over_retained_tokens_only(self):
        n, d = 30, 8
        Q, K, V = rand_head(n + 1, d)
        _, _, cache = orc.prefill(Q[:n], K[:n], V[:n], 0.5, 3, 2)
        kept = list(cache.pos) + [n]
        z = np.array([Q[n] @ K[p] for p in kept]) / math.sqrt(d)
        ref = np.exp(z - z.max())
        ref /= ref.sum()
        o, a, _, _ = orc.decode_step(cache, Q[n], K[n], V[n], n, 0.5, 3, 2)
        assert np.abs(a - ref).max() < 1e-14
        assert np.abs(o - ref @ V[kept]).max() < 1e-13

    def test_budget_fills_before_evicting(self):
        n, d = 4, 8
        Q, K, V = rand_head(12, d)
        _, _, cache = orc.prefill(Q[:n], K[:n], V[:n], 0.3, 3, 3)
        sizes = []
        for t in range(8):
            orc.decode_step(cache, Q[n + t], K[n + t], V[n + t], n + t, 0.3, 3, 3)
            sizes.append(len(cache))
        assert sizes == [5, 6, 6, 6, 6, 6, 6, 6]

    def test_strong_sink_survives(self):        # Section 4.3: the sink keeps a large score
        n, T, d = 128, 64, 16
        r = np.random.default_rng(5)
        Q, K, V = rand_head(n + T, d, rng=r)
        u = np.zeros(d)
        u[0] = 1.0
        Q += 4.0 * u
        K[0] += 6.0 * u
        _, _, cache = orc.prefill(Q[:n], K[:n], V[:n], 0.3, 8, 0)
        assert 0 in cache.pos
        for t in range(T):
            orc.decode_step(cache, Q[n + t], K[n + t], V[n + t], n + t, 0.3, 8, 0)
            assert 0 in cache.pos

    def test_forced_choice_rules(self):
        K = np.eye(4)
        c = orc.HeadCache(K, K, [0.5, 0.2, 0.2 + 4e-7, 0.9], [0, 1, 2, 3])
        c1 = c.copy()
        gone, swaps = orc.evict(c1, 2, 1)
        assert gone == [1] and swaps == 0
        c2 = c.copy()
        gone, swaps = orc.evict(c2, 2, 1, forced_retained=[0, 1, 3])
        assert gone == [2] and swaps == 1                   # inside the 1e-6 margin: accepted
        with pytest.raises(ValueError):
            orc.evict(c.copy(), 2, 1, forced_retained=[1, 2, 3])     # 0.5 vs 0.2: outside
        with pytest.raises(ValueError):
            orc.evict(c.copy(), 2, 1, forced_retained=[0, 1, 2])     # drops the recent token
        with pytest.raises(ValueError):
            orc.evict(c.copy(), 2, 1, forced_retained=[0, 3])        # wrong size



# ---------------------------------------------------------------- chunks of a prompt
def brute_chunk(cacheK, cacheV, cacheS, Qc, Kc, Vc, alpha):
    """A chunk against a cache with explicit loops: row i attends the L cached tokens and the
    chunk's tokens 0..i; the scores follow S <- alpha*S + a once per row (abstract, Section 3.3)."""
    L, m, d = len(cacheK), len(Qc), len(Qc[0])
    keys = [list(r) for r in cacheK] + [list(r) for r in Kc]
    vals = [list(r) for r in cacheV] + [list(r) for r in Vc]
    S = [float(x) for x in cacheS] + [0.0] * m
    O = []
    for i in range(m):
        vis = L + i + 1
        logit = [sum(Qc[i][c] * keys[j][c] for c in range(d)) / math.sqrt(d) for j in range(vis)]
        top = max(logit)
        ex = [math.exp(x - top) for x in logit]
        tot = math.fsum(ex)
        a = [x / tot for x in ex]
        O.append([math.fsum(a[j] * vals[j][c] for j in range(vis)) for c in range(len(vals[0]))])
        S = [alpha * S[j] + (a[j] if j < vis else 0.0) for j in range(L + m)]
    return O, S


class TestChunks:
    def _cache(self, L, d, rng):
        K, V = rng.standard_normal((L, d)), rng.standard_normal((L, d))
        S = rng.random(L)
        pos = np.sort(rng.choice(5 * L + 3, size=L, replace=False))
        return orc.HeadCache(K, V, S, pos)

    @pytest.mark.parametrize("alpha", [0.0, 0.3, 1.0])
    def test_brute_force_chunk(self, alpha):
        rng = np.random.default_rng(11)
        L, m, d = 7, 5, 4
        c = self._cache(L, d, rng)
        Qc, Kc, Vc = (rng.standard_normal((m, d)) for _ in range(3))
        O_ref, S_ref = brute_chunk(c.K.tolist(), c.V.tolist(), c.S.tolist(), Qc.tolist(), Kc.tolist(),
                                   Vc.tolist(), alpha)
        first = int(c.pos.max()) + 1
        O, P = orc.chunk_attend_and_update(c, Qc, Kc, Vc, first, alpha)
        assert np.abs(O - np.array(O_ref)).max() < 1e-13
        assert np.abs(c.S - np.array(S_ref)).max() < 1e-13
        assert np.all(P[np.arange(m)[:, None] + L < np.arange(L + m)[None, :]] == 0.0)   # masked part
        assert np.allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-14)
        assert list(c.pos[L:]) == list(range(first, first + m))

    @pytest.mark.parametrize("alpha", [0.0, 0.4, 1.0])
    def test_chunk_is_steps_without_eviction_then_one_eviction(self, alpha):
        """The matrix form against the generation-step form: m calls of attend_and_update with
        no eviction in between, then evict -- same outputs, scores and survivors."""
        rng = np.random.default_rng(5)
        L, m, d, sel, rec = 20, 9, 8, 8, 6
        c1 = self._cache(L, d, rng)
        c2 = c1.copy()
        Qc, Kc, Vc = (rng.standard_normal((m, d)) for _ in range(3))
        first = int(c1.pos.max()) + 1
        O, gone, _ = orc.prefill_chunk(c1, Qc, Kc, Vc, first, alpha, sel, rec)
        for i in range(m):
            o, _ = orc.attend_and_update(c2, Qc[i], Kc[i], Vc[i], first + i, alpha)
            assert np.abs(o - O[i]).max() < 1e-13
        gone2, _ = orc.evict(c2, sel, rec)
        assert gone == gone2 and len(gone) == L + m - (sel + rec)
        assert list(c1.pos) == list(c2.pos)
        assert np.abs(c1.S - c2.S).max() < 1e-13
        assert np.array_equal(c1.K, c2.K) and np.array_equal(c1.V, c2.V)

    def test_chunk_of_one_is_a_generation_step(self):
        rng = np.random.default_rng(6)
        c1 = self._cache(15, 8, rng)
        c2 = c1.copy()
        q, k, v = (rng.standard_normal(8) for _ in range(3))
        t = int(c1.pos.max()) + 4
        O, gone, _ = orc.prefill_chunk(c1, q[None], k[None], v[None], t, 0.6, 5, 5)
        o, _, gone2, _ = orc.decode_step(c2, q, k, v, t, 0.6, 5, 5)
        assert np.abs(O[0] - o).max() < 1e-14 and gone == gone2
        assert list(c1.pos) == list(c2.pos) and np.abs(c1.S - c2.S).max() < 1e-14

    @pytest.mark.parametrize("alpha", [0.0, 0.25, 1.0])
    def test_one_chunk_on_an_empty_cache_is_the_prompt_phase(self, alpha):
        n, d, sel, rec = 48, 8, 7, 5
        Q, K, V = rand_head(n, d)
        O_ref, S_full, c_ref = orc.prefill(Q, K, V, alpha, sel, rec)
        c = orc.HeadCache(np.zeros((0, d)), np.zeros((0, d)), np.zeros(0), np.zeros(0, dtype=np.int64))
        O, P = orc.chunk_attend_and_update(c, Q, K, V, 0, alpha)
        assert np.abs(O - O_ref).max() < 1e-13
        assert np.abs(c.S - S_full).max() < 1e-13
        assert np.abs(P - orc.causal_probabilities(Q, K)).max() < 1e-14
        orc.evict(c, sel, rec)
        assert list(c.pos) == list(c_ref.pos) and np.abs(c.S - c_ref.S).max() < 1e-13

    @pytest.mark.parametrize("sizes", [(30, 18), (1, 47), (24, 1, 23), (16, 16, 16)])
    def test_chunks_without_eviction_equal_the_whole_prompt(self, sizes):
        """With a budget that never binds, any split of the prompt into chunks gives the rows
        and the Eq.5 scores of the whole prompt."""
        n, d, alpha = sum(sizes), 8, 0.45
        Q, K, V = rand_head(n, d)
        P = orc.causal_probabilities(Q, K)
        c = orc.HeadCache(np.zeros((0, d)), np.zeros((0, d)), np.zeros(0), np.zeros(0, dtype=np.int64))
        at = 0
        for m in sizes:
            O, gone, _ = orc.prefill_chunk(c, Q[at:at + m], K[at:at + m], V[at:at + m], at, alpha, n, 0)
            assert gone == []
            assert np.abs(O - orc.attention_output(P, V)[at:at + m]).max() < 1e-13
            at += m
        assert np.abs(c.S - orc.forgotten_scores(P, alpha)).max() < 1e-13

    @pytest.mark.parametrize("alpha", [0.3, 1.0])
    def test_chunk_score_total(self, alpha):
        """Rows sum to 1, so the chunk adds sum_i alpha^(m-1-i) to the decayed total."""
        rng = np.random.default_rng(8)
        c = self._cache(12, 4, rng)
        before = c.S.sum()
        m = 6
        Qc, Kc, Vc = (rng.standard_normal((m, 4)) for _ in range(3))
        orc.chunk_attend_and_update(c, Qc, Kc, Vc, int(c.pos.max()) + 1, alpha)
        add = float(m) if alpha == 1.0 else (1 - alpha ** m) / (1 - alpha)
        assert math.isclose(c.S.sum(), alpha ** m * before + add, rel_tol=1e-13)


# ---------------------------------------------------------------- grouped-query heads
class TestGroupedQueryHeads:
    def test_group_of_one_is_the_plain_path(self):
        n, T, d, alpha, sel, rec = 40, 9, 8, 0.3, 6, 4
        Q, K, V = rand_head(n + T, d)
        O1, S1, c1 = orc.prefill(Q[:n], K[:n], V[:n], alpha, sel, rec)
        O2, S2, c2 = orc.gqa_prefill(Q[None, :n], K[:n], V[:n], alpha, sel, rec)
        assert np.array_equal(O1, O2[0]) and np.array_equal(S1, S2) and list(c1.pos) == list(c2.pos)
        for t in range(T):
            o1, _, g1, _ = orc.decode_step(c1, Q[n + t], K[n + t], V[n + t], n + t, alpha, sel, rec)
            o2, _, g2, _ = orc.gqa_decode_step(c2, Q[None, n + t], K[n + t], V[n + t], n + t, alpha, sel, rec)
            assert np.abs(o1 - o2[0]).max() < 1e-15 and g1 == g2
        assert np.abs(c1.S - c2.S).max() < 1e-15

    def test_group_score_is_the_sum_over_its_query_heads(self):
        """Each query head's output is what that head computes alone on the shared K/V; the
        group's score is the sum of the single-head scores (prompt and generation steps, no
        eviction so that the single-head caches stay comparable)."""
        r, n, T, d, alpha = 3, 30, 6, 8, 0.5
        rng = np.random.default_rng(13)
        Qs = rng.standard_normal((r, n + T, d))
        K, V = rng.standard_normal((n + T, d)), rng.standard_normal((n + T, d))
        big = n + T
        O, S, c = orc.gqa_prefill(Qs[:, :n], K[:n], V[:n], alpha, big, 0)
        singles = [orc.prefill(Qs[h, :n], K[:n], V[:n], alpha, big, 0) for h in range(r)]
        assert np.abs(S - sum(x[1] for x in singles)).max() < 1e-13
        for h in range(r):
            assert np.abs(O[h] - singles[h][0]).max() < 1e-14
        caches = [x[2] for x in singles]
        for t in range(T):
            o, a, _, _ = orc.gqa_decode_step(c, Qs[:, n + t], K[n + t], V[n + t], n + t, alpha, big, 0)
            for h in range(r):
                oh, ah, _, _ = orc.decode_step(caches[h], Qs[h, n + t], K[n + t], V[n + t], n + t, alpha, big, 0)
                assert np.abs(o[h] - oh).max() < 1e-14 and np.abs(a[h] - ah).max() < 1e-15
            assert np.abs(c.S - sum(x.S for x in caches)).max() < 1e-13

    def test_group_totals(self):
        """r rows of probabilities are added per step: total_after = alpha * total_before + r."""
        r, n, d, alpha = 4, 25, 8, 0.3
        rng = np.random.default_rng(14)
        Qs = rng.standard_normal((r, n + 1, d))
        K, V = rng.standard_normal((n + 1, d)), rng.standard_normal((n + 1, d))
        _, S, c = orc.gqa_prefill(Qs[:, :n], K[:n], V[:n], alpha, 6, 6)
        assert math.isclose(S.sum(), r * (1 - alpha ** n) / (1 - alpha), rel_tol=1e-12)
        before = c.S.sum()
        orc.gqa_attend_and_update(c, Qs[:, n], K[n], V[n], n, alpha)
        assert math.isclose(c.S.sum(), alpha * before + r, rel_tol=1e-13)

    @pytest.mark.parametrize("alpha", [0.0, 0.4, 1.0])
    def test_grouped_chunk_is_grouped_steps_then_one_eviction(self, alpha):
        """A chunk of a grouped head against m calls of gqa_attend_and_update with no eviction in
        between, then evict: same outputs, scores and survivors."""
        rng = np.random.default_rng(21)
        r, L, m, d, sel, rec = 3, 18, 7, 8, 7, 5
        c1 = orc.HeadCache(rng.standard_normal((L, d)), rng.standard_normal((L, d)), rng.random(L),
                           np.sort(rng.choice(60, L, replace=False)))
        c2 = c1.copy()
        Qcs = rng.standard_normal((r, m, d))
        Kc, Vc = rng.standard_normal((m, d)), rng.standard_normal((m, d))
        first = int(c1.pos.max()) + 1
        O, gone, _ = orc.gqa_prefill_chunk(c1, Qcs, Kc, Vc, first, alpha, sel, rec)
        for i in range(m):
            o, _ = orc.gqa_attend_and_update(c2, Qcs[:, i], Kc[i], Vc[i], first + i, alpha)
            assert np.abs(o - O[:, i]).max() < 1e-13
        gone2, _ = orc.evict(c2, sel, rec)
        assert gone == gone2 and len(gone) == L + m - (sel + rec)
        assert list(c1.pos) == list(c2.pos) and np.abs(c1.S - c2.S).max() < 1e-13
        assert np.array_equal(c1.K, c2.K) and np.array_equal(c1.V, c2.V)

    def test_grouped_chunk_of_one_group_member_is_the_plain_chunk(self):
        rng = np.random.default_rng(22)
        L, m, d = 12, 9, 8
        c1 = orc.HeadCache(rng.standard_normal((L, d)), rng.standard_normal((L, d)), rng.random(L), np.arange(L))
        c2 = c1.copy()
        Qc, Kc, Vc = (rng.standard_normal((m, d)) for _ in range(3))
        O1, g1, _ = orc.prefill_chunk(c1, Qc, Kc, Vc, L, 0.35, 6, 5)
        O2, g2, _ = orc.gqa_prefill_chunk(c2, Qc[None], Kc, Vc, L, 0.35, 6, 5)
        assert np.abs(O1 - O2[0]).max() < 1e-15 and g1 == g2
        assert list(c1.pos) == list(c2.pos) and np.abs(c1.S - c2.S).max() < 1e-15

    def test_grouped_chunk_by_brute_force(self):
        """Python loops over heads, rows and keys against the matrix form: softmax over the cached
        tokens and the chunk's tokens up to the row's own, weights alpha^(m-1-i), old scores
        times alpha^m, all r heads added."""
        rng = np.random.default_rng(23)
        r, L, m, d, alpha = 2, 5, 4, 3, 0.6
        c = orc.HeadCache(rng.standard_normal((L, d)), rng.standard_normal((L, d)), rng.random(L), np.arange(L))
        S0, K0, V0 = c.S.copy(), c.K.copy(), c.V.copy()
        Qcs = rng.standard_normal((r, m, d))
        Kc, Vc = rng.standard_normal((m, d)), rng.standard_normal((m, d))
        O, P = orc.gqa_chunk_attend_and_update(c, Qcs, Kc, Vc, L, alpha)
        keys = [list(K0[j]) for j in range(L)] + [list(Kc[j]) for j in range(m)]
        vals = [list(V0[j]) for j in range(L)] + [list(Vc[j]) for j in range(m)]
        S_ref = [alpha ** m * S0[j] for j in range(L)] + [0.0] * m
        for h in range(r):
            for i in range(m):
                vis = L + i + 1
                z = [sum(Qcs[h, i, e] * keys[j][e] for e in range(d)) / math.sqrt(d) for j in range(vis)]
                mx = max(z)
                ex = [math.exp(x - mx) for x in z]
                tot = sum(ex)
                for j in range(vis):
                    pj = ex[j] / tot
                    assert abs(P[h, i, j] - pj) < 1e-14
                    S_ref[j] += alpha ** (m - 1 - i) * pj
                for e in range(d):
                    assert abs(O[h, i, e] - sum(ex[j] / tot * vals[j][e] for j in range(vis))) < 1e-13
                assert np.all(P[h, i, vis:] == 0.0)
        assert np.abs(c.S - np.array(S_ref)).max() < 1e-13

    def test_grouped_chunk_score_total(self):
        """r probability rows per chunk row: total_after = alpha^m total_before + r (1 - alpha^m)/(1 - alpha)."""
        rng = np.random.default_rng(24)
        r, L, m, d, alpha = 5, 14, 11, 8, 0.3
        c = orc.HeadCache(rng.standard_normal((L, d)), rng.standard_normal((L, d)), rng.random(L), np.arange(L))
        before = c.S.sum()
        orc.gqa_chunk_attend_and_update(c, rng.standard_normal((r, m, d)), rng.standard_normal((m, d)),
                                        rng.standard_normal((m, d)), L, alpha)
        assert math.isclose(c.S.sum(), alpha ** m * before + r * (1 - alpha ** m) / (1 - alpha), rel_tol=1e-13)

    def test_one_grouped_chunk_on_an_empty_cache_is_the_grouped_prompt_phase(self):
        rng = np.random.default_rng(25)
        r, n, d, alpha, sel, rec = 3, 40, 8, 0.45, 6, 5
        Qs = rng.standard_normal((r, n, d))
        K, V = rng.standard_normal((n, d)), rng.standard_normal((n, d))
        O_ref, S_full, c_ref = orc.gqa_prefill(Qs, K, V, alpha, sel, rec)
        c = orc.HeadCache(np.zeros((0, d)), np.zeros((0, d)), np.zeros(0), np.zeros(0, dtype=np.int64))
        O, _, _ = orc.gqa_prefill_chunk(c, Qs, K, V, 0, alpha, sel, rec)
        assert np.abs(O - O_ref).max() < 1e-13
        assert list(c.pos) == list(c_ref.pos) and np.abs(c.S - c_ref.S).max() < 1e-13

    def test_one_eviction_serves_the_group(self):
        """The token with the smallest SUMMED score leaves, even where a single query head
        would have evicted another one."""
        d = 4
        K = np.eye(4)[:3].astype(float) * 6.0          # three tokens along different axes
        V = np.zeros((3, d))
        cache = orc.HeadCache(K, V, np.zeros(3), np.arange(3))
        qs = np.array([[6.0, 0, 0, 0], [0, 0, 6.0, 0]])            # head 0 likes token 0, head 1 token 2
        _, a, gone, _ = orc.gqa_decode_step(cache, qs, np.zeros(d), np.zeros(d), 3, 1.0, 3, 0)
        assert gone == [1] or gone == [3]              # token 1 (no head likes it) or the new token
        assert a[0].argmax() == 0 and a[1].argmax() == 2
        assert 0 in cache.pos and 2 in cache.pos


# ---------------------------------------------------------------- planted mistakes
def brute_row(q, K, allowed):
    """Softmax of q.k/sqrt(d) over the positions in `allowed`, explicit loops."""
    d = len(q)
    logit = {}
    for j in allowed:
        acc = 0.0
        for c in range(d):
            acc += q[c] * K[j][c]
        logit[j] = acc / math.sqrt(d)
    top = max(logit.values())
    tot = math.fsum(math.exp(x - top) for x in logit.values())
    row = [0.0] * len(K)
    for j, x in logit.items():
        row[j] = math.exp(x - top) / tot
    return row


class TestSimilarityToIdeal:
    """Section 4.3 / Table 2: rows of a pruning method against rows of the Ideal mask."""

    def test_no_pruning_is_the_full_attention_row_and_similarity_one(self):
        Q, K, V = rand_head(40, 8)
        P = orc.causal_probabilities(Q, K)        # pinned above
        for i in (0, 5, 39):
            np.testing.assert_allclose(orc.ideal_row(Q[i], K[:i + 1], keep=i + 1), P[i, :i + 1], rtol=1e-12)
            np.testing.assert_allclose(orc.pruned_row(Q[i], K[:i + 1], range(i + 1)), P[i, :i + 1], rtol=1e-12)
        cos, cache = orc.similarity_to_ideal(Q, K, V, 0.4, select=30, recent=30)
        np.testing.assert_allclose(cos, 1.0, rtol=0, atol=1e-12)
        assert len(cache) == 40

    def test_rows_by_brute_force(self):
        Q, K, _ = rand_head(14, 5, scale=1.5)
        i, keep = 13, 4
        full = brute_row(Q[i].tolist(), K.tolist(), range(i + 1))
        best = sorted(range(i + 1), key=lambda j: (-full[j], j))[:keep]
        np.testing.assert_allclose(orc.ideal_row(Q[i], K, keep), brute_row(Q[i].tolist(), K.tolist(), best),
                                   rtol=1e-12, atol=1e-300)
        some = [0, 3, 7, 13]
        np.testing.assert_allclose(orc.pruned_row(Q[i], K, some), brute_row(Q[i].tolist(), K.tolist(), some),
                                   rtol=1e-12, atol=1e-300)

    def test_ideal_subset_holds_the_most_attention(self):
        """"The Mask with the largest Attention Score given the Cache Size": no other subset of
        that size collects more of the full row's probability (exhaustive search)."""
        Q, K, _ = rand_head(9, 4, scale=2.0)
        i, keep = 8, 3
        full = np.asarray(brute_row(Q[i].tolist(), K.tolist(), range(i + 1)))
        ideal = orc.ideal_row(Q[i], K, keep)
        chosen = tuple(np.nonzero(ideal)[0])
        assert len(chosen) == keep
        best = max(itertools.combinations(range(i + 1), keep), key=lambda c: full[list(c)].sum())
        assert chosen == best
        # inside the subset the row is the full row renormalised
        np.testing.assert_allclose(ideal[list(chosen)], full[list(chosen)] / full[list(chosen)].sum(), rtol=1e-12)

    def test_uniform_attention_local_window_closed_form(self):
        """All keys equal: every attention entry is 1/len.  The Ideal keeps the lowest positions
        (tie rule), a pure recent window keeps the newest: with B cached tokens plus the current
        one on either side, cos = max(0, 2B + 1 - i) / (B + 1) from step i = B on."""
        n, d, B = 40, 4, 6
        Q = RNG.standard_normal((n, d))
        K = np.tile(RNG.standard_normal(d), (n, 1))
        V = RNG.standard_normal((n, d))
        cos, cache = orc.similarity_to_ideal(Q, K, V, 0.5, select=0, recent=B)
        want = [1.0 if i <= B else max(0, 2 * B + 1 - i) / (B + 1) for i in range(n)]
        np.testing.assert_allclose(cos, want, rtol=0, atol=1e-12)
        assert sorted(cache.pos.tolist()) == list(range(n - B, n))

    def test_tie_goes_to_lower_position(self):
        q = np.array([1.0, 0.0])
        K = np.array([[0.0, 1.0], [2.0, 0.0], [2.0, 5.0], [1.0, 0.0]])   # logits 0, 2, 2, 1 (times 1/sqrt 2)
        row = orc.ideal_row(q, K, keep=1)
        assert np.nonzero(row)[0].tolist() == [1] and row[1] == 1.0
        assert np.nonzero(orc.ideal_row(q, K, keep=3))[0].tolist() == [1, 2, 3]

    def test_cosine(self):
        assert orc.cosine_similarity([1, 0, 0], [0, 3, 0]) == 0.0
        assert abs(orc.cosine_similarity([0.2, 0.3, 0.5], [0.4, 0.6, 1.0]) - 1.0) < 1e-15
        assert abs(orc.cosine_similarity([1, 1, 0, 0], [1, 0, 1, 0]) - 0.5) < 1e-15

    def test_heavy_tokens_far_back_separate_score_policies_from_a_recent_window(self):
        """Qualitative content of Table 2 on planted data: with a few heavy tokens far back, a
        cache that selects by accumulated score stays much closer to the Ideal rows than a pure
        recent window, which loses them."""
        rng = np.random.default_rng(5)
        n, d, B = 160, 16, 16
        u = rng.standard_normal(d)
        u /= np.linalg.norm(u)
        Q = rng.standard_normal((n, d)) + 1.0 * u
        K = rng.standard_normal((n, d))
        K[[0, 7, 23, 40, 41, 77]] += 20.0 * u
        V = rng.standard_normal((n, d))
        local, _ = orc.similarity_to_ideal(Q, K, V, 0.3, select=0, recent=B)
        scored, _ = orc.similarity_to_ideal(Q, K, V, 0.3, select=B // 2, recent=B // 2)
        plain, _ = orc.similarity_to_ideal(Q, K, V, 1.0, select=B // 2, recent=B // 2)
        assert local[100:].mean() < 0.2
        assert scored[B + 1:].mean() > local[B + 1:].mean() + 0.2
        assert plain[B + 1:].mean() > local[B + 1:].mean() + 0.2


class TestPinsCatchMistakes:
    """Each case swaps one oracle function for a plausibly wrong one and requires that at
    least one of the pins above fails."""

    PINS = [
        (TestAttentionMatrix, "test_brute_force_matrix", ()),
        (TestAttentionMatrix, "test_mask_rows_and_diagonal", ()),
        (TestAttentionMatrix, "test_scale_is_one_over_sqrt_d", ()),
        (TestForgottenScore, "test_geometric_total", (0.3, 256)),
        (TestForgottenScore, "test_brute_force_eq6", (0.3,)),
        (TestForgottenScore, "test_alpha_zero_is_last_row", ()),
        (TestForgottenScore, "test_harmonic_fixture", ()),
        (TestSelection, "test_tie_at_the_cut_goes_to_lower_position", ()),
        (TestSelection, "test_recent_is_by_position_not_slot", ()),
        (TestDecode, "test_no_eviction_matches_prompt_form", ()),
        (TestDecode, "test_step_invariants_with_eviction", ()),
        (TestDecode, "test_softmax_is_over_retained_tokens_only", ()),
        (TestSimilarityToIdeal, "test_no_pruning_is_the_full_attention_row_and_similarity_one", ()),
        (TestSimilarityToIdeal, "test_rows_by_brute_force", ()),
        (TestSimilarityToIdeal, "test_ideal_subset_holds_the_most_attention", ()),
        (TestSimilarityToIdeal, "test_uniform_attention_local_window_closed_form", ()),
        (TestSimilarityToIdeal, "test_tie_goes_to_lower_position", ()),
        (TestSimilarityToIdeal, "test_cosine", ()),
        (TestChunks, "test_brute_force_chunk", (0.3,)),
        (TestChunks, "test_chunk_is_steps_without_eviction_then_one_eviction", (0.4,)),
        (TestChunks, "test_one_chunk_on_an_empty_cache_is_the_prompt_phase", (0.25,)),
        (TestChunks, "test_chunk_score_total", (0.3,)),
        (TestGroupedQueryHeads, "test_group_score_is_the_sum_over_its_query_heads", ()),
        (TestGroupedQueryHeads, "test_group_totals", ()),
        (TestGroupedQueryHeads, "test_one_eviction_serves_the_group", ()),
        (TestGroupedQueryHeads, "test_grouped_chunk_is_grouped_steps_then_one_eviction", (0.4,)),
        (TestGroupedQueryHeads, "test_grouped_chunk_by_brute_force", ()),
        (TestGroupedQueryHeads, "test_grouped_chunk_score_total", ()),
    ]

    def _some_pin_fails(self):
        for cls, name, args in self.PINS:
            try:
                getattr(cls(), name)(*args)
            except (AssertionError, ValueError, IndexError, ZeroDivisionError):
                return True
        return False

    def test_pins_pass_unmodified(self):
        assert not self._some_pin_fails()

    def test_off_by_one_exponent(self, monkeypatch):
        def bad(n, alpha):
            return np.power(float(alpha), np.arange(n, 0, -1, dtype=np.float64))
        monkeypatch.setattr(orc, "_weights", bad)
        assert self._some_pin_fails()

    def test_reversed_weights(self, monkeypatch):
        def bad(n, alpha):
            return np.power(float(alpha), np.arange(n, dtype=np.float64))
        monkeypatch.setattr(orc, "_weights", bad)
        assert self._some_pin_fails()

    def test_strict_mask_drops_diagonal(self, monkeypatch):
        def bad(Q, K):
            Q, K = np.asarray(Q, float), np.asarray(K, float)
            n, d = Q.shape
            s = Q @ K.T / np.sqrt(d)
            s[np.triu(np.ones((n, n), bool), k=0)] = -np.inf
            s[0, 0] = 0.0
            e = np.exp(s - s.max(axis=1, keepdims=True))
            return e / e.sum(axis=1, keepdims=True)
        monkeypatch.setattr(orc, "causal_probabilities", bad)
        assert self._some_pin_fails()

    def test_missing_scale(self, monkeypatch):
        def bad(Q, K):
            Q, K = np.asarray(Q, float), np.asarray(K, float)
            n = Q.shape[0]
            s = Q @ K.T
            s[np.triu(np.ones((n, n), bool), k=1)] = -np.inf
            e = np.exp(s - s.max(axis=1, keepdims=True))
            return e / e.sum(axis=1, keepdims=True)
        monkeypatch.setattr(orc, "causal_probabilities", bad)
        assert self._some_pin_fails()

    def test_transposed_logits(self, monkeypatch):
        def bad(Q, K):
            Q, K = np.asarray(Q, float), np.asarray(K, float)
            n, d = Q.shape
            s = (K @ Q.T) / np.sqrt(d)
            s[np.triu(np.ones((n, n), bool), k=1)] = -np.inf
            e = np.exp(s - s.max(axis=1, keepdims=True))
            return e / e.sum(axis=1, keepdims=True)
        monkeypatch.setattr(orc, "causal_probabilities", bad)
        assert self._some_pin_fails()

    def test_tie_to_higher_position(self, monkeypatch):
        real = orc.select_keep

        def bad(scores, pos, select, recent):
            return real(scores, -np.asarray(pos), select, recent)[::-1]
        monkeypatch.setattr(orc, "select_keep", bad)
        assert self._some_pin_fails()

    def test_forgetting_skipped_in_decode(self, monkeypatch):
        real = orc.attend_and_update

        def bad(cache, q, k, v, t, alpha):
            return real(cache, q, k, v, t, 1.0)
        monkeypatch.setattr(orc, "attend_and_update", bad)
        assert self._some_pin_fails()

    def test_ideal_keeps_the_smallest(self, monkeypatch):
        def bad(q, K, keep):
            s = orc._logits(q, K)
            order = sorted(range(len(s)), key=lambda j: (s[j], j))
            return orc.pruned_row(q, K, order[:min(keep, len(s))])
        monkeypatch.setattr(orc, "ideal_row", bad)
        assert self._some_pin_fails()

    def test_ideal_row_not_renormalised(self, monkeypatch):
        def bad(q, K, keep):
            s = orc._logits(q, K)
            e = np.exp(s - s.max())
            p = e / e.sum()
            order = sorted(range(len(s)), key=lambda j: (-s[j], j))[:min(keep, len(s))]
            row = np.zeros(len(s))
            row[order] = p[order]
            return row
        monkeypatch.setattr(orc, "ideal_row", bad)
        assert self._some_pin_fails()

    def test_ideal_tie_to_higher_position(self, monkeypatch):
        def bad(q, K, keep):
            s = orc._logits(q, K)
            order = sorted(range(len(s)), key=lambda j: (-s[j], -j))
            return orc.pruned_row(q, K, order[:min(keep, len(s))])
        monkeypatch.setattr(orc, "ideal_row", bad)
        assert self._some_pin_fails()

    def test_method_row_forgets_the_current_token(self, monkeypatch):
        real = orc.pruned_row

        def bad(q, K, retained):
            r = sorted(int(p) for p in retained)
            return real(q, K, r[:-1] if len(r) > 1 and r[-1] == len(K) - 1 else r)
        monkeypatch.setattr(orc, "pruned_row", bad)
        assert self._some_pin_fails()

    def test_cosine_without_normalisation(self, monkeypatch):
        monkeypatch.setattr(orc, "cosine_similarity", lambda u, v: float(np.dot(u, v)))
        assert self._some_pin_fails()

    def test_chunk_decay_forgotten(self, monkeypatch):
        """A chunk that does not decay the cached scores by alpha^m."""
        real = orc.chunk_attend_and_update

        def bad(cache, Qc, Kc, Vc, pos0, alpha):
            old = cache.S.copy()
            out = real(cache, Qc, Kc, Vc, pos0, alpha)
            m = len(np.asarray(Qc))
            cache.S[:len(old)] += (1.0 - float(alpha) ** m) * old
            return out
        monkeypatch.setattr(orc, "chunk_attend_and_update", bad)
        assert self._some_pin_fails()

    def test_chunk_rows_see_the_whole_chunk(self, monkeypatch):
        """A chunk whose rows also attend the chunk's LATER tokens (mask forgotten)."""
        def bad(cache, Qc, Kc, Vc, pos0, alpha):
            Qc, Kc, Vc = (np.asarray(x, float) for x in (Qc, Kc, Vc))
            m, d = Qc.shape
            L = len(cache)
            K_all, V_all = np.vstack([cache.K.reshape(L, d), Kc]), np.vstack([cache.V.reshape(L, d), Vc])
            s = Qc @ K_all.T / np.sqrt(d)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            P = e / e.sum(axis=1, keepdims=True)
            cache.S = float(alpha) ** m * np.concatenate([cache.S, np.zeros(m)]) + orc._weights(m, alpha) @ P
            cache.K, cache.V = K_all, V_all
            cache.pos = np.concatenate([cache.pos, np.arange(pos0, pos0 + m)])
            return P @ V_all, P
        monkeypatch.setattr(orc, "chunk_attend_and_update", bad)
        assert self._some_pin_fails()

    def test_grouped_chunk_decay_forgotten(self, monkeypatch):
        real = orc.gqa_chunk_attend_and_update

        def bad(cache, Qcs, Kc, Vc, pos0, alpha):
            old = np.concatenate([cache.S, np.zeros(len(Kc))])
            m = len(Kc)
            O, P = real(cache, Qcs, Kc, Vc, pos0, alpha)
            cache.S = cache.S - float(alpha) ** m * old + old      # older scores not decayed
            return O, P
        monkeypatch.setattr(orc, "gqa_chunk_attend_and_update", bad)
        assert self._some_pin_fails()

    def test_grouped_chunk_counts_one_head_only(self, monkeypatch):
        real = orc.gqa_chunk_attend_and_update

        def bad(cache, Qcs, Kc, Vc, pos0, alpha):
            c0 = cache.copy()
            O, P = real(cache, Qcs, Kc, Vc, pos0, alpha)
            real(c0, np.asarray(Qcs)[:1], Kc, Vc, pos0, alpha)
            cache.S = c0.S                                          # the other heads' rows dropped
            return O, P
        monkeypatch.setattr(orc, "gqa_chunk_attend_and_update", bad)
        assert self._some_pin_fails()

    def test_group_score_averaged_instead_of_summed(self, monkeypatch):
        real = orc.gqa_attend_and_update

        def bad(cache, qs, k_new, v_new, t_pos, alpha):
            old = np.append(cache.S, 0.0)
            o, a = real(cache, qs, k_new, v_new, t_pos, alpha)
            cache.S = float(alpha) * old + a.mean(axis=0)
            return o, a
        monkeypatch.setattr(orc, "gqa_attend_and_update", bad)
        assert self._some_pin_fails()
