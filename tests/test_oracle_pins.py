"""Pins for the CPU oracle: hand-worked fixtures, closed forms, invariants,
library routines and brute force.  CPU only; nothing here touches the HIP path.

Each test names the equation / algorithm of the paper it pins.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import tca_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(v) for v in line.split()])
    return rows


# ----------------------------------------------------------------- Eq. 3 --
def test_eq3_hand_worked_candidates():
    gold = np.array(read_rows("eq3_b4_sigma1.txt"))
    got = orc.candidates(4, 3, 1.0)
    assert got.shape == (3, 3)
    np.testing.assert_allclose(got, gold, atol=2e-10, rtol=0)


def test_eq3_properties():
    b, M, sigma = 128, 14, 1.0
    mus = orc.candidate_mus(b, M)
    assert mus[0] == 0.0 and abs(mus[-1] - 7.0) < 1e-12
    assert np.all(np.diff(mus) > 0)
    C = orc.candidates(b, M, sigma)
    assert C.shape == (14, 8)
    np.testing.assert_allclose(C.sum(axis=1), 1.0, atol=1e-14)
    # mean budget strictly increasing along the sweep (exponential family in mu)
    means = [orc.mean_budget(b, p) for p in C]
    assert np.all(np.diff(means) > 0)
    # integer mu: weights symmetric about it, mode at 2^mu
    p = orc.config_from_mu(b, 3.0, sigma)
    assert np.argmax(p) == 3
    assert abs(p[2] / p[3] - p[4] / p[3]) < 1e-14
    assert abs(p[2] / p[3] - math.exp(-0.5)) < 1e-14
    # sigma -> 0: one-hot at the nearest allowed count
    p = orc.config_from_mu(b, 4.2, 1e-3)
    assert p[4] > 1 - 1e-12


def test_config_from_budget_hits_target_and_saturates():
    b, sigma = 128, 1.0
    for f in (0.05, 0.1, 0.25, 0.5, 0.7):
        p = orc.config_from_budget(b, sigma, f)
        assert abs(orc.mean_budget(b, p) - f * b) < 1e-9
        assert abs(p.sum() - 1) < 1e-14
    assert list(orc.config_from_budget(b, sigma, 1.0)) == [0] * 7 + [1]
    assert list(orc.config_from_budget(b, sigma, 0.001)) == [1] + [0] * 7
    hi = orc.config_from_budget(b, sigma, 0.99)
    np.testing.assert_allclose(hi, orc.config_from_mu(b, 7.0, sigma))
    # one-hot at b keeps every row of every block
    assert orc.selected_rows(b, 10, orc.config_from_budget(b, sigma, 1.0)) == 10 * b


# ----------------------------------------------------------------- Eq. 5 --
def test_eq5_matches_library_softmax_and_sums_to_one():
    rng = np.random.default_rng(0)
    K = rng.standard_normal((50, 8))
    q = rng.standard_normal(8)
    s = orc.token_scores(q, K)
    assert abs(s.sum() - 1) < 1e-14
    np.testing.assert_allclose(s, scipy_softmax(K @ q / math.sqrt(8)), rtol=1e-13)
    # operand order: a transposed / swapped operand would break this non-square case
    x = orc.last_query_logits(q, K)
    assert x.shape == (50,)
    assert abs(x[7] - float(np.dot(K[7], q)) / math.sqrt(8)) < 1e-14
    # explicit scale overrides 1/sqrt(d)
    np.testing.assert_allclose(orc.last_query_logits(q, K, scale=2.0), 2.0 * (K @ q), rtol=1e-13)


# ----------------------------------------------------------------- Eq. 6 --
def test_eq6_hand_worked():
    gold = read_rows("eq6_b2_L4.txt")[0]
    x = np.array([0.0, math.log(3.0), 0.0, 0.0])
    np.testing.assert_allclose(orc.block_metric(x, 2, 0.25), gold, atol=1e-15)


def test_eq6_entropy_variant_hand_worked_and_closed_forms():
    gold = read_rows("eq6_entropy_b2_L4.txt")[0]
    x = np.array([0.0, math.log(3.0), 0.0, 0.0])
    np.testing.assert_allclose(orc.block_metric(x, 2, 0.5, "entropy"), gold, atol=1e-15)
    b, alpha = 8, 0.3
    # uniform logits: the renormalised block distribution is uniform, entropy / ln b = 1
    x = np.full(3 * b + 5, -0.4)
    np.testing.assert_allclose(orc.block_metric(x, b, alpha, "entropy"),
                               (1 - alpha) * b / len(x) + alpha * 1.0, atol=1e-15)
    # two equal tokens carry a block, the rest are negligible: entropy = ln 2
    x = np.full(2 * b, -800.0)
    x[b + 1] = x[b + 5] = 0.0
    h = orc.block_metric(x, b, alpha, "entropy")
    np.testing.assert_allclose(h[1], (1 - alpha) * 1.0 + alpha * math.log(2) / math.log(b), atol=1e-15)
    # alpha = 0 removes the concentration term: both metrics give the block mass
    x = np.random.default_rng(3).normal(size=4 * b)
    np.testing.assert_allclose(orc.block_metric(x, b, 0.0, "entropy"), orc.block_metric(x, b, 0.0), atol=0)
    # entropy in nats against scipy, block by block
    from scipy.stats import entropy as sp_entropy
    s = orc.softmax(x)
    ref = np.array([0.5 * s[j * b:(j + 1) * b].sum() + 0.5 * sp_entropy(s[j * b:(j + 1) * b]) / math.log(b)
                    for j in range(4)])
    np.testing.assert_allclose(orc.block_metric(x, b, 0.5, "entropy"), ref, atol=1e-14)
    with pytest.raises(ValueError):
        orc.block_metric(x, b, 0.5, "gini")


def test_eq6_closed_forms_and_invariances():
    b, alpha = 8, 0.5
    # uniform logits: every block has mass b/L and concentration 1/b
    x = np.full(4 * b + 3, 1.7)
    h = orc.block_metric(x, b, alpha)
    L = len(x)
    np.testing.assert_allclose(h, (1 - alpha) * b / L + alpha * (1 - 1 / b), atol=1e-15)
    assert len(h) == 4                                    # tail of 3 tokens forms no block
    # one token dominates a block: concentration term -> 0, mass -> ~1
    x = np.zeros(2 * b)
    x[3] = 80.0
    h = orc.block_metric(x, b, alpha)
    assert abs(h[0] - (1 - alpha) * 1.0) < 1e-12
    # block 1 has underflowing mass but a well-defined uniform concentration term
    assert abs(h[1] - alpha * (1 - 1 / b)) < 1e-12
    # range
    rng = np.random.default_rng(1)
    x = 5 * rng.standard_normal(20 * b + 5)
    h = orc.block_metric(x, b, alpha)
    assert np.all(h >= 0) and np.all(h <= (1 - alpha) + alpha * (1 - 1 / b))
    # adding a constant to all logits changes nothing (softmax shift invariance)
    np.testing.assert_allclose(orc.block_metric(x + 11.0, b, alpha), h, rtol=1e-12)
    # alpha = 0: pure mass, and masses over blocks + tail sum to 1
    s = scipy_softmax(x)
    mass = orc.block_metric(x, b, 0.0)
    np.testing.assert_allclose(mass, s[: 20 * b].reshape(20, b).sum(1), rtol=1e-12)
    assert abs(mass.sum() + s[20 * b:].sum() - 1) < 1e-13
    # alpha = 1: pure (1 - HHI) from the plain definition on s
    conc = orc.block_metric(x, b, 1.0)
    sb = s[: 20 * b].reshape(20, b)
    np.testing.assert_allclose(conc, 1 - (sb ** 2).sum(1) / sb.sum(1) ** 2, rtol=1e-10)


# ------------------------------------------------------------ Eq. 7 and 8 --
def test_eq7_eq8_hand_worked():
    rows = read_rows("eq7_eq8_b4_m4.txt")
    t_gold = np.array(rows[0], int)
    S_gold = np.array(rows[1], int)
    p = np.array([0.5, 0.25, 0.25])
    h = np.array([0.1, 0.9, 0.5, 0.3])
    assert list(orc.psi_list(4, 4, p)) == [1, 1, 2, 4]
    t = orc.block_budgets(4, h, p)
    assert list(t) == list(t_gold)
    scores = np.array([[0.2, 0.9, 0.1, 0.5], [0.3, 0.1, 0.2, 0.6], [0.7, 0.1, 0.7, 0.3], [0.4, 0.4, 0.4, 0.4]])
    S = np.concatenate([4 * j + orc.top_t(scores[j], t[j]) for j in range(4)])
    assert list(S) == list(S_gold)


def test_eq7_counts_and_deficit():
    b = 128
    for m in (1, 7, 256, 1024, 1000):
        for p in orc.candidates(b, 14, 1.0):
            c = orc.psi_counts(m, p)
            assert c.sum() == m and np.all(c >= 0)
            fl = np.floor(m * p + 1e-9).astype(int)
            assert np.all(c[1:] == fl[1:]) and c[0] == fl[0] + (m - fl.sum())
            psi = orc.psi_list(b, m, p)
            assert len(psi) == m and np.all(np.diff(psi) >= 0)
            assert orc.selected_rows(b, m, p) == psi.sum()
    # exact products must not lose a block to rounding: p = (1/4, 3/4), m = 8
    assert list(orc.psi_counts(8, np.array([0.25, 0.75]))) == [2, 6]
    # one-hot
    assert list(orc.psi_counts(5, np.array([0.0, 0.0, 1.0]))) == [0, 0, 5]


def test_rank_direction_and_ties():
    h = np.array([0.3, 0.1, 0.3, 0.2])
    assert list(orc.block_ranks(h)) == [2, 0, 3, 1]          # ties: lower block index first
    assert list(orc.block_ranks(np.zeros(4))) == [0, 1, 2, 3]
    # densest block (largest h) receives the largest budget
    p = np.array([0.5, 0.25, 0.25])
    t = orc.block_budgets(4, np.array([0.9, 0.1, 0.2, 0.3]), p)
    assert t[0] == 4 and t[1] == 1


def test_eq8_brute_force():
    """Top(t; B) maximises the total score over all C(b,t) subsets, and among
    maximisers is the lexicographically smallest (ties to the lower position)."""
    rng = np.random.default_rng(2)
    for b in (2, 4, 8):
        for trial in range(20):
            x = rng.integers(0, 4, size=b).astype(float) if trial % 2 else rng.standard_normal(b)
            for t in [k for k in (1, 2, 4, 8) if k <= b]:
                got = tuple(orc.top_t(x, t))
                best = max(itertools.combinations(range(b), t),
                           key=lambda c: (sum(x[i] for i in c), tuple(-i for i in c)))
                assert got == best, (x, t)


def test_select_invariants_and_brute_force_small():
    rng = np.random.default_rng(3)
    for (L, b, d) in [(32, 4, 8), (29, 8, 4), (16, 2, 4), (7, 8, 4)]:
        K = rng.standard_normal((L, d))
        q = rng.standard_normal(d)
        nk = int(math.log2(b)) + 1
        p = rng.dirichlet(np.ones(nk))
        sel = orc.select(q, K, b, p, 0.5)
        m = L // b
        assert len(sel.t) == m and len(sel.h) == m
        assert len(sel.S) == orc.selected_rows(b, m, p) == sel.t.sum()
        assert np.all(np.diff(sel.S) > 0)
        if m:
            assert sel.S.min() >= 0 and sel.S.max() < m * b          # tail never selected
        # independent re-derivation with python sorting on the definition
        x = (K @ q) / math.sqrt(d)
        s = scipy_softmax(x)
        hs = []
        for j in range(m):
            sb = s[j * b:(j + 1) * b]
            hs.append(0.5 * sb.sum() + 0.5 * (1 - (sb ** 2).sum() / sb.sum() ** 2))
        order = sorted(range(m), key=lambda j: (hs[j], j))
        counts = [int(math.floor(m * pk + 1e-9)) for pk in p]
        counts[0] += m - sum(counts)
        psi = [2 ** e for e, c in enumerate(counts) for _ in range(c)]
        S = []
        for r, j in enumerate(order):
            best = sorted(range(b), key=lambda i: (-x[j * b + i], i))[: psi[r]]
            S += [j * b + i for i in best]
        assert sorted(S) == list(sel.S)


def test_select_zero_query_is_decided_by_tie_breaks():
    """Q = 0: s uniform, every h_j equal, so ranks follow the block index and
    each block keeps its first t_j positions."""
    b, m, d = 4, 6, 8
    rng = np.random.default_rng(4)
    K = rng.standard_normal((m * b + 2, d))
    p = np.array([0.5, 0.34, 0.16])
    sel = orc.select(np.zeros(d), K, b, p, 0.5)
    psi = orc.psi_list(b, m, p)
    assert list(sel.t) == list(psi)
    expect = [j * b + i for j in range(m) for i in range(psi[j])]
    assert list(sel.S) == expect


# ------------------------------------------------------------ Eq. 1 and 2 --
def _dense_causal_library(Q, K, V):
    L, d = Q.shape
    logits = Q @ K.T / math.sqrt(d)
    logits[np.triu_indices(L, 1)] = -np.inf
    return scipy_softmax(logits, axis=1) @ V


def test_eq1_dense_against_library():
    rng = np.random.default_rng(5)
    Q, K, V = (rng.standard_normal((17, 8)) for _ in range(3))
    np.testing.assert_allclose(orc.dense_causal_attention(Q, K, V), _dense_causal_library(Q, K, V), rtol=1e-12)


def test_eq2_full_budget_or_wide_window_is_dense():
    rng = np.random.default_rng(6)
    L, b, d = 40, 4, 8
    Q, K, V = (rng.standard_normal((1, L, d)) for _ in range(3))
    dense = _dense_causal_library(Q[0], K[0], V[0])
    p_full = np.array([[0.0, 0.0, 1.0]])
    O, sels = orc.tca_prefill(Q, K, V, b, 8, p_full, 0.5)
    assert list(sels[0].S) == list(range(L))
    np.testing.assert_allclose(O[0], dense, rtol=1e-12)
    # window covering the sequence: selection is irrelevant
    p_min = np.array([[1.0, 0.0, 0.0]])
    O, _ = orc.tca_prefill(Q, K, V, b, L, p_min, 0.5)
    np.testing.assert_allclose(O[0], dense, rtol=1e-12)
    # L < b: no block, everything local
    O, sels = orc.tca_prefill(Q[:, :3], K[:, :3], V[:, :3], b, 4, p_min, 0.5)
    assert len(sels[0].S) == 0
    np.testing.assert_allclose(O[0], dense[:3], rtol=1e-12)


def test_eq2_visible_set_no_overlap_and_masking():
    S = np.array([0, 3, 4, 9, 10, 15])
    w = 4
    # query 12: window (8,12]; global rows that left it: <= 8
    T = orc.visible_keys(12, S, w)
    assert list(T) == [0, 3, 4, 9, 10, 11, 12]
    assert len(set(T)) == len(T)
    # early query: window clipped at 0, no global row visible
    assert list(orc.visible_keys(2, S, w)) == [0, 1, 2]
    # manual softmax over exactly that set
    rng = np.random.default_rng(7)
    K, V = rng.standard_normal((16, 4)), rng.standard_normal((16, 4))
    q = rng.standard_normal(4)
    out = orc.attention_row(q, 12, K, V, S, w)
    ref = scipy_softmax(K[T] @ q / 2.0) @ V[T]
    np.testing.assert_allclose(out, ref, rtol=1e-13)
    # convex combination: inside the per-column range of the attended rows
    assert np.all(out <= V[T].max(0) + 1e-12) and np.all(out >= V[T].min(0) - 1e-12)
    # order of stored global rows is irrelevant
    out2 = orc.attention_row(q, 12, K, V, S[::-1].copy(), w)
    np.testing.assert_allclose(out, out2, rtol=1e-13)


def test_gqa_equals_mha_with_repeated_kv():
    rng = np.random.default_rng(8)
    Hq, Hkv, L, d, b, w = 4, 2, 24, 8, 4, 8
    Q = rng.standard_normal((Hq, L, d))
    K = rng.standard_normal((Hkv, L, d))
    V = rng.standard_normal((Hkv, L, d))
    p = rng.dirichlet(np.ones(3), size=Hq)
    O1, s1 = orc.tca_prefill(Q, K, V, b, w, p, 0.5)
    O2, s2 = orc.tca_prefill(Q, np.repeat(K, 2, 0), np.repeat(V, 2, 0), b, w, p, 0.5)
    np.testing.assert_allclose(O1, O2, rtol=1e-13)
    for a, c in zip(s1, s2):
        assert list(a.S) == list(c.S)
    # heads are independent: permuting heads permutes outputs
    perm = [2, 3, 0, 1]
    O3, _ = orc.tca_prefill(Q[perm], K[[1, 0]], V[[1, 0]], b, w, p[perm], 0.5)
    np.testing.assert_allclose(O3, O1[perm], rtol=1e-13)


# ------------------------------------------------------------------ decode --
def test_decode_step_equals_last_prefill_row():
    rng = np.random.default_rng(9)
    Hq, Hkv, L, d, b, w = 2, 1, 43, 8, 4, 8
    Q = rng.standard_normal((Hq, L, d))
    K = rng.standard_normal((Hkv, L, d))
    V = rng.standard_normal((Hkv, L, d))
    p = rng.dirichlet(np.ones(3), size=Hq)
    O, sels = orc.tca_prefill(Q, K, V, b, w, p, 0.5)
    cache = orc.HeadCache(S=[s.S.copy() for s in sels], K=K[:, : L - 1].copy(), V=V[:, : L - 1].copy())
    out = orc.decode_step(cache, Q[:, L - 1], K[:, L - 1], V[:, L - 1], b, w, p)
    np.testing.assert_allclose(out, O[:, L - 1], rtol=1e-12)
    assert cache.length == L


def test_decode_selection_replay():
    """Decoding from an empty cache: after n steps the global subset is the
    union, over completed blocks, of the top-t rows scored by the query of the
    completing step; outputs follow Eq. 2 with the set as it stood."""
    rng = np.random.default_rng(10)
    Hq, Hkv, d, b, w, n = 2, 1, 4, 4, 4, 19
    p = np.array([[0.2, 0.5, 0.3], [0.7, 0.2, 0.1]])
    q = rng.standard_normal((n, Hq, d))
    k = rng.standard_normal((n, Hkv, d))
    v = rng.standard_normal((n, Hkv, d))
    cache = orc.HeadCache(S=[np.zeros(0, np.int64) for _ in range(Hq)])
    outs = [orc.decode_step(cache, q[s], k[s], v[s], b, w, p) for s in range(n)]
    for h in range(Hq):
        t = int(math.floor(sum(kk * pk for kk, pk in zip((1, 2, 4), p[h])) + 1e-9))
        expect = []
        for j in range(n // b):
            T = (j + 1) * b - 1
            x = k[j * b:(j + 1) * b, 0] @ q[T, h]
            expect += sorted(j * b + i for i in sorted(range(b), key=lambda i: (-x[i], i))[:t])
        assert list(cache.S[h]) == expect
        # output of the last step: keys = expect rows <= T-w, plus window
        T = n - 1
        keys = [e for e in expect if e <= T - w] + list(range(T - w + 1, T + 1))
        ref = scipy_softmax(k[keys, 0] @ q[T, h] / 2.0) @ v[keys, 0]
        np.testing.assert_allclose(outs[-1][h], ref, rtol=1e-12)
    assert orc.decode_budget(4, p[0]) == 2 and orc.decode_budget(4, p[1]) == 1
    assert orc.decode_budget(128, np.eye(8)[7]) == 128


# ------------------------------------------------------- Eq. 4 and Alg. 1 --
def test_eq4_uniform_hand_worked_and_harmonic_closed_form():
    gold = [Fraction(int(a), int(b_)) for a, b_ in read_rows("eq4_uniform_L5.txt")]
    A = orc.dense_causal_probs(np.zeros((5, 3)), np.ones((5, 3)))
    abar = orc.column_means(A)
    np.testing.assert_allclose(abar, [float(g) for g in gold], rtol=1e-14)
    L = 300
    abar = orc.column_means(orc.dense_causal_probs(np.zeros((L, 2)), np.zeros((L, 2))))
    H = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, L + 1))])
    np.testing.assert_allclose(abar, (H[L] - H[:L]) / (L - np.arange(L)), rtol=1e-12)


def test_eq4_probs_match_library_and_sum():
    rng = np.random.default_rng(11)
    L, d = 30, 4
    Q, K = rng.standard_normal((L, d)), rng.standard_normal((L, d))
    A = orc.dense_causal_probs(Q, K)
    logits = Q @ K.T / 2.0
    logits[np.triu_indices(L, 1)] = -np.inf
    np.testing.assert_allclose(A, scipy_softmax(logits, axis=1), rtol=1e-12, atol=1e-300)
    abar = orc.column_means(A)
    assert abar.sum() >= 1 - 1e-12            # sum of column means >= 1 always
    # a_i with S = everything is that sum; with S = {3, 7} it is two entries
    assert abs(orc.cumulative_score(abar, np.arange(L)) - abar.sum()) < 1e-14
    assert abs(orc.cumulative_score(abar, np.array([3, 7])) - (A[3:, 3].mean() + A[7:, 7].mean())) < 1e-14


def test_alg1_threshold_behaviour():
    rng = np.random.default_rng(12)
    L, d, b, M = 64, 8, 8, 6
    Q, K = 2 * rng.standard_normal((L, d)), rng.standard_normal((L, d))
    cands = orc.candidates(b, M, 1.0)
    c0 = orc.calibrate_head(Q, K, b, cands, 0.0, 0.5)
    assert c0.index == int(np.argmin(c0.n)) and not c0.fallback          # tau=0: everything valid
    assert np.all(np.diff(c0.n) >= 0)                                     # |S_i| grows along the sweep
    chigh = orc.calibrate_head(Q, K, b, cands, 1e9, 0.5)
    assert chigh.index == M - 1 and chigh.fallback                        # nothing valid
    # a threshold between two candidates' scores picks the sparsest that clears it
    a = c0.a
    tau = 0.5 * (a[2] + a[3]) if a[3] > a[2] else a[3]
    c = orc.calibrate_head(Q, K, b, cands, tau, 0.5)
    valid = [i for i in range(M) if a[i] >= tau]
    assert c.index == min(valid, key=lambda i: (c0.n[i], i))
    # a_i recomputed from the definition for one candidate
    S = orc.select(Q[L - 1], K, b, cands[2], 0.5).S
    A = orc.dense_causal_probs(Q, K)
    assert abs(a[2] - sum(A[k:, k].sum() / (L - k) for k in S)) < 1e-12


# --------------------------------------------------------------- Theorem 1 --
def test_theorem1_identity_and_bounds():
    rng = np.random.default_rng(13)
    L, d, b, w = 96, 8, 8, 16
    Q, K, V = 1.5 * rng.standard_normal((L, d)), rng.standard_normal((L, d)), rng.standard_normal((L, d))
    p = orc.config_from_budget(b, 1.0, 0.3)
    S = orc.select(Q[L - 1], K, b, p, 0.5).S
    dense = orc.dense_causal_attention(Q, K, V)
    for i in (0, 5, 17, 40, 95):
        gamma, l1, att, att_sparse = orc.theorem_quantities(Q[i], i, K, V, S, w)
        assert 0 <= gamma <= 1
        assert abs(l1 - 2 * gamma) < 1e-12                 # identity in the proof of Theorem 1
        np.testing.assert_allclose(att, dense[i], rtol=1e-12)
        np.testing.assert_allclose(att_sparse, orc.attention_row(Q[i], i, K, V, S, w), rtol=1e-12)
        err = att - att_sparse
        assert np.abs(err).max() <= 2 * gamma * np.abs(V).max() + 1e-12
        assert np.abs(err).sum() <= 2 * gamma * np.abs(V).sum(1).max() + 1e-12
    # early queries see everything through the window: gamma = 0
    assert orc.theorem_quantities(Q[10], 10, K, V, S, w)[0] == 0.0


# ----------------------------------------------- planted-mistake sanity check --
def test_pins_would_catch_a_swapped_rank_direction(monkeypatch):
    """Plant a mistake in the oracle (descending instead of ascending rank) and
    check the hand-worked Eq. 7 fixture fails: the pins are not vacuous."""
    real = orc.block_ranks
    monkeypatch.setattr(orc, "block_ranks", lambda h: len(h) - 1 - real(h))
    t = orc.block_budgets(4, np.array([0.1, 0.9, 0.5, 0.3]), np.array([0.5, 0.25, 0.25]))
    assert list(t) != [1, 4, 2, 1]


# ------------------------------------------------------- chunked prefill --
def test_chunked_prefill_reduces_to_alg2_and_follows_its_definition():
    rng = np.random.default_rng(14)
    Hq, Hkv, L, d, b, w = 2, 1, 70, 8, 4, 8
    Q = rng.standard_normal((Hq, L, d))
    K = rng.standard_normal((Hkv, L, d))
    V = rng.standard_normal((Hkv, L, d))
    p = rng.dirichlet(np.ones(3), size=Hq)
    O1, sels = orc.tca_prefill(Q, K, V, b, w, p, 0.5)
    # one chunk covering the sequence is Alg. 2
    O2, S2 = orc.tca_prefill_chunked(Q, K, V, b, w, p, 0.5, chunk=72)
    np.testing.assert_allclose(O2, O1, rtol=1e-13)
    for h in range(Hq):
        assert list(S2[h]) == list(sels[h].S)
    # three chunks: index sets are the per-chunk selections put end to end; a row
    # of chunk 1 sees rows kept from chunks 0 and 1 only, and only outside its window
    chunk = 24
    O3, S3 = orc.tca_prefill_chunked(Q, K, V, b, w, p, 0.5, chunk=chunk)
    for h in range(Hq):
        parts = []
        for c0 in range(0, L, chunk):
            c1 = min(L, c0 + chunk)
            parts.append(c0 + orc.select(Q[h, c1 - 1], K[0, c0:c1], b, p[h], 0.5).S)
        assert list(S3[h]) == list(np.concatenate(parts))
        assert len(S3[h]) == sum(orc.selected_rows(b, (min(L, c0 + chunk) - c0) // b, p[h]) for c0 in range(0, L, chunk))
        i = 40                                                     # in chunk 1 = [24, 48)
        upto = np.concatenate(parts[:2])
        keys = [int(j) for j in upto if j <= i - w] + list(range(i - w + 1, i + 1))
        ref = scipy_softmax(K[0][keys] @ Q[h, i] / math.sqrt(d)) @ V[0][keys]
        np.testing.assert_allclose(O3[h, i], ref, rtol=1e-12)
    # chunk not a multiple of b is rejected
    with pytest.raises(ValueError):
        orc.tca_prefill_chunked(Q, K, V, b, w, p, 0.5, chunk=10)


# ------------------------------------------------- group-shared selection --
def test_group_shared_hand_worked():
    sbar, h, t, S = read_rows("group_shared_b2_L4.txt")
    X = np.log(np.array([[4.0, 1.0, 3.0, 2.0], [1.0, 2.0, 3.0, 4.0]]))
    np.testing.assert_allclose(orc.group_scores_from_logits(X), sbar, atol=1e-15)
    np.testing.assert_allclose(orc.block_metric_of_scores(np.array(sbar), 2, 0.5), h, atol=1e-15)
    # through select_shared: d = 4, K = identity rows, so that q_g . k_i = q_g[i]; scale 1
    sel = orc.select_shared(X, np.eye(4), 2, np.array([0.5, 0.5]), 0.5, scale=1.0)
    np.testing.assert_allclose(sel.h, h, atol=1e-15)
    assert list(sel.t) == [int(v) for v in t] and list(sel.S) == [int(v) for v in S]
    np.testing.assert_allclose(np.exp(sel.x), sbar, atol=1e-15)


def test_group_shared_reduces_to_per_head_selection():
    rng = np.random.default_rng(21)
    L, d, b = 75, 8, 8
    K = rng.standard_normal((L, d))
    q = 2 * rng.standard_normal((3, d))
    p = rng.dirichlet(np.ones(4))
    for metric in ("hhi", "entropy"):
        one = orc.select(q[0], K, b, p, 0.4, metric=metric)
        # a group of one head, and a group of identical heads, are that head
        for grp in (q[:1], np.repeat(q[:1], 3, axis=0)):
            sh = orc.select_shared(grp, K, b, p, 0.4, metric=metric)
            assert list(sh.S) == list(one.S) and list(sh.t) == list(one.t)
            np.testing.assert_allclose(sh.h, one.h, rtol=1e-12, atol=1e-15)
    # the metric written on scores equals the one written on logits
    x = orc.last_query_logits(q[1], K)
    for metric in ("hhi", "entropy"):
        np.testing.assert_allclose(orc.block_metric_of_scores(orc.softmax(x), b, 0.3, metric),
                                   orc.block_metric(x, b, 0.3, metric), rtol=1e-12)


def test_group_shared_invariants_and_brute_force():
    rng = np.random.default_rng(22)
    L, d, b, G = 53, 6, 4, 3
    K = rng.standard_normal((L, d))
    q = 3 * rng.standard_normal((G, d))
    p = np.array([0.3, 0.45, 0.25])
    sel = orc.select_shared(q, K, b, p, 0.5)
    m = L // b
    assert len(sel.S) == orc.selected_rows(b, m, p)
    assert abs(np.exp(sel.x).sum() - 1.0) < 1e-13                      # a mean of distributions is one
    # the order of the heads inside the group does not matter
    sel2 = orc.select_shared(q[[2, 0, 1]], K, b, p, 0.5)
    assert list(sel2.S) == list(sel.S)
    # brute force with python loops and library softmax
    sc = 1.0 / math.sqrt(d)
    sbar = [0.0] * L
    for g in range(G):
        sg = scipy_softmax([sum(q[g][e] * K[i][e] for e in range(d)) * sc for i in range(L)])
        for i in range(L):
            sbar[i] += sg[i] / G
    hb = []
    for j in range(m):
        blk = sbar[j * b:(j + 1) * b]
        hb.append(0.5 * sum(blk) + 0.5 * (1.0 - sum(v * v for v in blk) / sum(blk) ** 2))
    np.testing.assert_allclose(sel.h, hb, rtol=1e-12)
    order = sorted(range(m), key=lambda j: (hb[j], j))
    psi = list(orc.psi_list(b, m, p))
    expect = []
    for r, j in enumerate(order):
        best = sorted(range(b), key=lambda i: (-sbar[j * b + i], i))[:psi[r]]
        expect += [j * b + i for i in best]
    assert sorted(expect) == list(sel.S)
    # it is not the per-head selection of any single head, nor the selection by mean logits
    assert any(list(orc.select(q[g], K, b, p, 0.5).S) != list(sel.S) for g in range(G))
    assert list(orc.select(q.mean(axis=0), K, b, p, 0.5).S) != list(sel.S)


def test_group_shared_attention_decode_and_calibration():
    rng = np.random.default_rng(23)
    Hq, Hkv, L, d, b, w = 4, 2, 40, 8, 4, 8
    Q = rng.standard_normal((Hq, L, d))
    K = rng.standard_normal((Hkv, L, d))
    V = rng.standard_normal((Hkv, L, d))
    p = rng.dirichlet(np.ones(3), size=Hkv)
    O, sels = orc.tca_prefill(Q, K, V, b, w, p, 0.5, share=True)
    assert len(sels) == Hkv
    # every query head attends to its group's set: the row recomputed from Eq. 2
    for h in range(Hq):
        np.testing.assert_allclose(O[h, 33], orc.attention_row(Q[h, 33], 33, K[h // 2], V[h // 2], sels[h // 2].S, w),
                                   rtol=1e-13)
    # full budget: dense attention, shared or not
    full = np.tile(np.array([0.0, 0.0, 1.0]), (Hkv, 1))
    Od, _ = orc.tca_prefill(Q, K, V, b, w, full, 0.5, share=True)
    for h in range(Hq):
        np.testing.assert_allclose(Od[h], orc.dense_causal_attention(Q[h], K[h // 2], V[h // 2]), rtol=1e-12)
    # one chunk = Alg. 2; two chunks: the second chunk's set comes from its own keys and last queries
    Oc, Sc = orc.tca_prefill_chunked(Q, K, V, b, w, p, 0.5, chunk=L, share=True)
    np.testing.assert_allclose(Oc, O, rtol=1e-13)
    Oc2, Sc2 = orc.tca_prefill_chunked(Q, K, V, b, w, p, 0.5, chunk=20, share=True)
    for g in range(Hkv):
        first = orc.select_shared(Q[2 * g:2 * g + 2, 19], K[g, :20], b, p[g], 0.5).S
        second = 20 + orc.select_shared(Q[2 * g:2 * g + 2, 39], K[g, 20:40], b, p[g], 0.5).S
        assert list(Sc2[g]) == list(first) + list(second)
    # decode: the step that follows prefill reproduces the last prefill row; a completed block is
    # ranked by the group mean of the block-normalised scores
    cache = orc.HeadCache(S=[s.S.copy() for s in sels], K=K[:, : L - 1].copy(), V=V[:, : L - 1].copy())
    before = [s.copy() for s in cache.S]
    out = orc.decode_step(cache, Q[:, L - 1], K[:, L - 1], V[:, L - 1], b, w, p, share=True)
    np.testing.assert_allclose(out, O[:, L - 1], rtol=1e-12)
    j = (L - 1) // b
    for g in range(Hkv):
        sb = np.mean([scipy_softmax(K[g, j * b:(j + 1) * b] @ Q[h, L - 1] / math.sqrt(d)) for h in (2 * g, 2 * g + 1)], axis=0)
        t = orc.decode_budget(b, p[g])
        keep = sorted(j * b + i for i in sorted(range(b), key=lambda i: (-sb[i], i))[:t])
        assert list(cache.S[g]) == list(before[g]) + keep
    # calibration: a group of identical heads calibrates like the single head
    Qs = np.repeat(Q[:1], 2, axis=0)
    one = orc.calibrate(Qs[:1], K[:1], b, 5, 1.0, 0.6, 0.5)[0]
    grp = orc.calibrate(Qs, K[:1], b, 5, 1.0, 0.6, 0.5, share=True)[0]
    assert grp.index == one.index and list(grp.n) == list(one.n)
    np.testing.assert_allclose(grp.a, one.a, rtol=1e-12)
    # and for distinct heads a_i is the sum over the shared set of the group-mean column means
    cal = orc.calibrate(Q[:2], K[:1], b, 5, 1.0, 0.6, 0.5, share=True)[0]
    cands = orc.candidates(b, 5, 1.0)
    S2 = orc.select_shared(Q[:2, L - 1], K[0], b, cands[2], 0.5).S
    cm = 0.5 * (orc.column_means(orc.dense_causal_probs(Q[0], K[0])) + orc.column_means(orc.dense_causal_probs(Q[1], K[0])))
    assert abs(cal.a[2] - cm[S2].sum()) < 1e-13


# --------------------------------------------------------------------------
# Layer integration (extensions): FP8 cache rows, rotary embedding, several layers
# --------------------------------------------------------------------------
def _fp8_fixture():
    vals, rounds, row = [], [], {}
    for line in open(os.path.join(GOLD, "fp8_e4m3_codes.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "round":
            rounds.append((float(t[1]), int(t[2], 16)))
        elif t[0] in ("row", "scale", "codes"):
            row[t[0]] = [int(v, 16) if t[0] == "codes" else float(v) for v in t[1:]]
        else:
            vals.append((int(t[0], 16), float(t[1])))
    return vals, rounds, row


def test_fp8_format_against_hand_values_and_the_library_type():
    import torch
    vals, rounds, row = _fp8_fixture()
    table = orc.fp8_e4m3_values()
    for code, v in vals:
        assert table[code] == v, hex(code)
    assert np.isnan(table[0x7F]) and np.isnan(table[0xFF]) and np.nanmax(table) == 448.0
    # the whole table against the library's float8 type
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.nan_to_num(table, nan=-1.0), np.nan_to_num(lib, nan=-1.0))
    for y, code in rounds:
        assert int(orc.fp8_e4m3_encode(np.float32(y))) == code, y
    # rounding of many numbers against the library's conversion (which does not saturate: clip first)
    rng = np.random.default_rng(5)
    y = np.concatenate([(rng.standard_normal(50000) * s).astype(np.float32) for s in (1e-3, 0.05, 1.0, 30.0, 200.0)])
    ref = torch.from_numpy(np.clip(y, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = orc.fp8_e4m3_encode(y)
    nz = y != 0                                           # the sign of a zero is not a matter of rounding
    assert np.array_equal(got[nz], ref[nz])
    # every representable value encodes to itself
    finite = ~np.isnan(table)
    assert np.array_equal(orc.fp8_e4m3_encode(table[finite].astype(np.float32))[1:], np.arange(256)[finite][1:])
    # a planted mistake (ties rounded away from zero instead of to even) fails the fixture
    away = lambda y: int(orc.fp8_e4m3_encode(np.float32(np.nextafter(np.float32(y), np.float32(1e9)))))
    assert away(1.0625) != dict(rounds)[1.0625]


def test_fp8_rows_scale_rule_and_error_bound():
    _, _, row = _fp8_fixture()
    codes, scale = orc.quantize_rows_fp8(np.array([row["row"]]))
    assert codes[0].tolist() == row["codes"] and float(scale[0]) == row["scale"][0]
    assert np.array_equal(orc.roundtrip_rows_fp8(np.array([row["row"]]))[0], np.array(row["row"]))
    rng = np.random.default_rng(6)
    X = rng.standard_normal((200, 128)) * rng.uniform(0.01, 50, size=(200, 1))
    X[7] = 0.0
    codes, scale = orc.quantize_rows_fp8(X)
    assert codes.dtype == np.uint8 and scale.dtype == np.float32 and scale[7] == 1.0 and not codes[7].any()
    amax = np.abs(X.astype(np.float32)).max(axis=1)
    big = np.abs(X.astype(np.float32)) == amax[:, None]
    assert np.all((codes[big & (amax[:, None] > 0)] & 0x7F) == 0x7E)        # the row's largest entry sits at +-448
    R = orc.dequantize_rows_fp8(codes, scale)
    # normal range: half a unit of a 3-bit mantissa (2^-4 relative); below 2^-6 * scale: half a subnormal step
    err = np.abs(R - X.astype(np.float32))
    bound = np.maximum(np.abs(X) * 2.0 ** -4, scale[:, None] * 2.0 ** -10) * (1 + 1e-6)
    assert np.all(err <= bound)
    assert np.all(np.sign(R) * np.sign(X) >= 0)


def test_decode_step_with_an_fp8_cache_reads_dequantised_rows():
    """The cache mode is Eq. 2 over rows that went through the FP8 store: checked against the plain
    attention routine fed rows converted by the library's float8 type with the row scales."""
    import torch
    rng = np.random.default_rng(8)
    Hq, Hkv, d, L, b, w = 2, 1, 16, 40, 4, 8
    Q, K, V = rng.standard_normal((Hq, L, d)), rng.standard_normal((Hkv, L, d)) * 3, rng.standard_normal((Hkv, L, d))
    P = np.stack([orc.config_from_budget(b, 1.0, 0.5)] * Hq)
    sels = orc.select_all_heads(Q[:, L - 1], K, b, P, 0.5)
    cache = orc.cache_after_prefill(K, V, sels, kv_quant="fp8")
    q, kn, vn = rng.standard_normal((Hq, d)), rng.standard_normal((Hkv, d)), rng.standard_normal((Hkv, d))
    out = orc.decode_step(cache, q, kn, vn, b, w, P, kv_quant="fp8")

    def lib_roundtrip(X):
        X32 = torch.from_numpy(np.asarray(X, np.float32))
        amax = X32.abs().amax(dim=-1, keepdim=True)
        scale = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
        return ((X32 / scale).clamp(-448, 448).to(torch.float8_e4m3fn).to(torch.float64) * scale.to(torch.float64)).numpy()

    Kq = np.concatenate([lib_roundtrip(K), lib_roundtrip(kn)[:, None]], axis=1)
    Vq = np.concatenate([lib_roundtrip(V), lib_roundtrip(vn)[:, None]], axis=1)
    for h in range(Hq):
        ref = orc.attention_row(q[h], L, Kq[0], Vq[0], sels[h].S, w)
        np.testing.assert_allclose(out[h], ref, rtol=1e-12, atol=1e-14)
    assert cache.length == L + 1 and np.array_equal(cache.K[0, L], Kq[0, L])
    # and it differs from the unquantised step by no more than the rows' rounding allows
    plain = orc.decode_step(orc.cache_after_prefill(K, V, sels), q, kn, vn, b, w, P)
    assert 0 < np.abs(plain - out).max() < 0.5


def test_rope_hand_example_complex_rotation_and_invariants():
    rows = [list(map(float, l.split())) for l in open(os.path.join(GOLD, "rope_d4.txt")) if l.strip() and not l.startswith("#")]
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    np.testing.assert_allclose(orc.rope_rotate(x, [2], pairing="half")[0], rows[0], atol=5e-10)
    np.testing.assert_allclose(orc.rope_rotate(x, [2], pairing="interleaved")[0], rows[1], atol=5e-10)
    rng = np.random.default_rng(9)
    n, d = 7, 16
    X, pos = rng.standard_normal((3, n, d)), rng.integers(0, 5000, size=n)
    R = orc.rope_rotate(X, pos)
    # the rotation written with complex numbers: (a + ib) e^{i t f}
    f = 10000.0 ** (-2.0 * np.arange(d // 2) / d)
    z = (X[..., : d // 2] + 1j * X[..., d // 2:]) * np.exp(1j * pos[:, None] * f[None, :])
    np.testing.assert_allclose(R[..., : d // 2], z.real, atol=1e-12)
    np.testing.assert_allclose(R[..., d // 2:], z.imag, atol=1e-12)
    np.testing.assert_allclose(np.linalg.norm(R, axis=-1), np.linalg.norm(X, axis=-1), rtol=1e-13)
    assert np.array_equal(orc.rope_rotate(X, np.zeros(n)), X)
    # q_m . k_n depends on m - n only; rotating by a then by b is rotating by a + b
    q, k = rng.standard_normal((1, d)), rng.standard_normal((1, d))
    d1 = orc.rope_rotate(q, [37]) @ orc.rope_rotate(k, [30]).T
    d2 = orc.rope_rotate(q, [1007]) @ orc.rope_rotate(k, [1000]).T
    np.testing.assert_allclose(d1, d2, rtol=1e-10)
    np.testing.assert_allclose(orc.rope_rotate(orc.rope_rotate(q, [11]), [31]), orc.rope_rotate(q, [42]), atol=1e-12)
    # the two pairings are one rotation seen through a permutation of the coordinates
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])
    np.testing.assert_allclose(orc.rope_rotate(X, pos, pairing="interleaved")[..., perm], orc.rope_rotate(X[..., perm], pos), atol=1e-12)


def test_qkv_project_hand_example_selector_weights_and_brute_force():
    rows = np.array([list(map(float, l.split())) for l in open(os.path.join(GOLD, "qkv_project_d2.txt"))
                     if l.strip() and not l.startswith("#")])
    X = np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 2.0]])
    W = np.array([[1, 0, 0], [0, 1, 0], [1, 1, 1], [2, 0, -1], [0, 0, 1], [1, -1, 0], [0.5, 0.5, 0], [-1, 2, 1]], float)
    bias = np.array([0.5, 0, 0, 0, 0, 0, 0, -1.0])
    for off, bs in ((0, None), (8, bias)):
        Q, K, V = orc.qkv_project(X, W, 2, 1, 2, bias=bs)
        assert Q.shape == (2, 2, 2) and K.shape == (1, 2, 2) and V.shape == (1, 2, 2)
        got = np.concatenate([Q.reshape(4, 2), K.reshape(2, 2), V.reshape(2, 2)])
        np.testing.assert_array_equal(got, rows[off:off + 8])
    # weights that pick single hidden features: every output is an entry of X, by name
    rng = np.random.default_rng(21)
    n, hidden, Hq, Hkv, d = 5, 40, 3, 1, 4
    X = rng.standard_normal((n, hidden))
    pick = rng.permutation(hidden)[: (Hq + 2 * Hkv) * d]
    W = np.zeros(((Hq + 2 * Hkv) * d, hidden))
    W[np.arange(len(pick)), pick] = 1.0
    Q, K, V = orc.qkv_project(X, W, Hq, Hkv, d)
    for h in range(Hq):
        for e in range(d):
            assert np.array_equal(Q[h, :, e], X[:, pick[h * d + e]])
    for e in range(d):
        assert np.array_equal(K[0, :, e], X[:, pick[Hq * d + e]])
        assert np.array_equal(V[0, :, e], X[:, pick[(Hq + Hkv) * d + e]])
    # the definition, one multiply-add at a time
    W = rng.standard_normal(((Hq + 2 * Hkv) * d, hidden))
    bias = rng.standard_normal((Hq + 2 * Hkv) * d)
    Q, K, V = orc.qkv_project(X, W, Hq, Hkv, d, bias=bias)
    heads = [("q", h) for h in range(Hq)] + [("k", 0), ("v", 0)]
    for f0, (kind, h) in enumerate(heads):
        out = {"q": Q, "k": K, "v": V}[kind][h]
        for t in range(n):
            for e in range(d):
                acc = bias[f0 * d + e]
                for c in range(hidden):
                    acc += X[t, c] * W[f0 * d + e, c]
                assert abs(out[t, e] - acc) < 1e-12
    # attention over projected rows is what the method's Eq. 1 is written for: Q K^T of head h uses
    # that head's W_Q and its KV head's W_K
    S = Q[1] @ K[0].T
    Wq1, Wk = W[d:2 * d], W[Hq * d:(Hq + 1) * d]
    np.testing.assert_allclose(S, (X @ Wq1.T + bias[d:2 * d]) @ (X @ Wk.T + bias[Hq * d:(Hq + 1) * d]).T, rtol=1e-12)


def test_calibrate_layers_is_alg1_layer_by_layer():
    rng = np.random.default_rng(10)
    Hq, Hkv, d, L, b, M = 2, 1, 8, 64, 4, 5
    Qs = [rng.standard_normal((Hq, L, d)) * g for g in (0.5, 3.0, 8.0)]
    Ks = [rng.standard_normal((Hkv, L, d)) for _ in range(3)]
    out = orc.calibrate_layers(Qs, Ks, b, M, 1.0, 0.9, 0.5)
    assert len(out) == 3 and all(len(layer) == Hq for layer in out)
    for l in range(3):
        for h in range(Hq):
            one = orc.calibrate_head(Qs[l][h], Ks[l][0], b, orc.candidates(b, M, 1.0), 0.9, 0.5)
            assert out[l][h].index == one.index and np.array_equal(out[l][h].p, one.p)
    # sharper queries concentrate attention: the peaked layer never needs a larger candidate than the flat one
    assert max(c.index for c in out[2]) <= max(c.index for c in out[0])
