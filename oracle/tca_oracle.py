"""Plain fp64 CPU oracle for the hot path of TCA-Attention (arxiv 2512.09238).

THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path (the HIP library and its
Python binding) never does and shares no code, table or constant with it.

Everything here is numpy in float64, written to be read next to the paper:
one function per equation / algorithm step, no blocking, no fusion, no
reordering beyond what the step states.  Index conventions are 0-based:
position j of the paper's 1..L is j-1 here; "the last query" is row L-1.

Readings of the paper where it is silent or ambiguous (each is the default
here and the only behaviour the GPU path implements):

  * one selection per *query* head; under GQA query head h reads KV head
    h // (Hq // Hkv)  (Sec. IV: "independently and in parallel to all heads").
  * the local subset of query i is the sliding window (i-w, i]; causal mask
    everywhere; a global row j is visible to query i only if j <= i-w, which
    realises "no overlap between the global and local subsets" (Sec. IV).
  * sum_k floor(m p_k) can fall short of m: the missing blocks are the
    lowest-ranked ones and receive the minimum budget k=1  (Eq. 7).
  * block with the r-th smallest h receives the r-th entry of the ascending
    list Psi, so the densest blocks get the largest budgets (Eq. 7 gloss).
  * ties (equal h, equal score) go to the lower index.
  * s is normalised over all L keys, the tail L mod b included (Eq. 5); the
    concentration term of Eq. 6 is evaluated with the block's own maximum so
    it stays defined when the block's mass underflows.
  * sigma of Eq. 3 is a parameter (the paper never prints its value).
  * Eq. 4: the column count ||A_:,k||_0 is the structural causal count L-k;
    S_i is the global subset only; a_i is not renormalised.
  * an empty valid set in Alg. 1 returns the last (largest) candidate, flagged.
  * decode (Sec. IV-B last paragraph): blocks are aligned to absolute
    positions; a block is scored, with the query of the step that completes
    it, over its b rows, and its top t = floor(sum_k k p_k) rows join the
    global subset; they become visible once they leave the window.
  * chunked prefill is not in the paper; `tca_prefill_chunked` states the rule
    used (each chunk scored by its own last query over its own keys).
  * group-shared selection (share=True; an extension for GQA, not in the paper):
    one index set per KV head, chosen by the mean over the group's query heads of
    their Eq. 5 scores; Eq. 6-8 then run on that mean score unchanged, and every
    query head of the group attends to the shared set.  See the section
    "Group-shared selection" below.

  * layer integration around the path (extensions, not in the paper, which takes Q, K, V as
    given, post position encoding): rotary position embedding of Q and K (`rope_rotate`, the
    published RoFormer rotation), an FP8 E4M3 decode cache with one scale per row
    (`quantize_rows_fp8`; `kv_quant="fp8"` in the cache routines), and calibration of several
    layers (`calibrate_layers`: Alg. 1 once per layer).  See "Layer integration" below.

Functions pinned by tests/test_oracle_pins.py; none is "parity unpinned"
except the readings listed above, which are choices rather than facts.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Eq. 3 : log-Gaussian configuration candidates
# --------------------------------------------------------------------------
def retain_counts(b: int) -> np.ndarray:
    """The set K = {1, 2, 4, ..., b} of allowed per-block retain counts (Sec. IV-A)."""
    if b < 1 or (b & (b - 1)) != 0:
        raise ValueError("block size must be a power of two")
    return 2 ** np.arange(int(math.log2(b)) + 1, dtype=np.int64)


def config_from_mu(b: int, mu: float, sigma: float) -> np.ndarray:
    """Eq. 3: p_k = Phi[log2 k] / sum Phi, Phi[x] = exp(-(x-mu)^2 / (2 sigma^2))."""
    x = np.log2(retain_counts(b).astype(F64))
    e = -((x - mu) ** 2) / (2.0 * sigma * sigma)
    phi = np.exp(e - e.max())          # common factor cancels in the ratio; avoids 0/0 for tiny sigma
    return phi / phi.sum()


def candidate_mus(b: int, M: int) -> np.ndarray:
    """mu^i = log2(1 + (i-1)(b-1)/(M-1)), i = 1..M  (text below Eq. 3)."""
    if M == 1:
        return np.array([0.0])
    i = np.arange(1, M + 1, dtype=F64)
    return np.log2(1.0 + (i - 1.0) * (b - 1.0) / (M - 1.0))


def candidates(b: int, M: int, sigma: float) -> np.ndarray:
    """The candidate set C = {p^1..p^M} of Eq. 3, shape [M, log2(b)+1]."""
    return np.stack([config_from_mu(b, mu, sigma) for mu in candidate_mus(b, M)])


def mean_budget(b: int, p: np.ndarray) -> float:
    """sum_k k p_k : average number of tokens kept per block (Sec. IV-B, decode)."""
    return float(np.dot(retain_counts(b).astype(F64), np.asarray(p, F64)))


def config_from_budget(b: int, sigma: float, frac: float) -> np.ndarray:
    """Configuration whose mean budget sum_k k p_k equals frac*b (reading: the
    workloads state a budget as a fraction of L, the paper as a vector p).

    Bisection on mu in [0, log2 b] at fixed sigma; the mean is increasing in mu.
    frac >= 1 gives the one-hot vector at k=b; a target above the largest
    reachable mean gives the mu = log2 b configuration; a target below the
    smallest reachable mean gives the one-hot vector at k=1.
    """
    nk = len(retain_counts(b))
    target = frac * b
    lo, hi = 0.0, float(math.log2(b))
    if frac >= 1.0:
        p = np.zeros(nk)
        p[-1] = 1.0
        return p
    if target >= mean_budget(b, config_from_mu(b, hi, sigma)):
        return config_from_mu(b, hi, sigma)
    if target < mean_budget(b, config_from_mu(b, lo, sigma)):
        p = np.zeros(nk)
        p[0] = 1.0
        return p
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if mean_budget(b, config_from_mu(b, mid, sigma)) < target:
            lo = mid
        else:
            hi = mid
    return config_from_mu(b, 0.5 * (lo + hi), sigma)


# --------------------------------------------------------------------------
# Eq. 7 : rank -> budget map Psi
# --------------------------------------------------------------------------
def psi_counts(m: int, p: np.ndarray) -> np.ndarray:
    """Number of entries of each value in Psi: c_k = floor(m p_k) (Eq. 7).

    A guard of 1e-9 keeps floor() stable when m p_k is an integer up to
    rounding.  Blocks left over (m - sum c_k) get the minimum budget k=1.
    """
    p = np.asarray(p, F64)
    c = np.floor(m * p + 1e-9).astype(np.int64)
    c[0] += m - int(c.sum())
    return c


def psi_list(b: int, m: int, p: np.ndarray) -> np.ndarray:
    """Psi written out: ascending list of m per-block budgets (Eq. 7)."""
    return np.repeat(retain_counts(b), psi_counts(m, p))


def selected_rows(b: int, m: int, p: np.ndarray) -> int:
    """|S| = sum_k k c_k: fixed by (m, p), independent of the data."""
    return int(np.dot(retain_counts(b), psi_counts(m, p)))


def decode_budget(b: int, p: np.ndarray) -> int:
    """t = floor(sum_k k p_k): rows kept from a block completed during decoding."""
    return int(math.floor(mean_budget(b, p) + 1e-9))


# --------------------------------------------------------------------------
# Eq. 5 : token importance from the last query
# --------------------------------------------------------------------------
def default_scale(d: int) -> float:
    return 1.0 / math.sqrt(d)


def last_query_logits(q_last: np.ndarray, K: np.ndarray, scale: float | None = None) -> np.ndarray:
    """x_j = q_L . k_j / sqrt(d_h) for every key j (the argument of Eq. 5)."""
    q = np.asarray(q_last, F64)
    K = np.asarray(K, F64)
    sc = default_scale(K.shape[1]) if scale is None else scale
    # row-by-row products summed along d: the same reduction for every row,
    # so identical rows give identical logits.
    return (K * q[None, :]).sum(axis=1) * sc


def softmax(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, F64)
    e = np.exp(x - x.max())
    return e / e.sum()


def token_scores(q_last: np.ndarray, K: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Eq. 5: s = softmax(Q_L K^T / sqrt(d_h)) over all L keys."""
    return softmax(last_query_logits(q_last, K, scale))


# --------------------------------------------------------------------------
# Eq. 6 : block redundancy metric
# --------------------------------------------------------------------------
def block_metric(x: np.ndarray, b: int, alpha: float, metric: str = "hhi") -> np.ndarray:
    """h_j = (1-alpha) sum_{B_j} s + alpha (1 - sum s^2 / (sum s)^2)  (Eq. 6).

    x: logits of all L keys.  The first term uses s normalised over all L keys.
    The ratio in the second term is invariant to the normaliser, so it is
    evaluated from exp(x - max of the block).

    metric="entropy": the concentration index of the appendix ablation ("Ablations on
    Concentration Index"), which the paper names but does not write out.  Reading:
    the second term becomes the entropy of the scores renormalised inside the block,
    divided by ln b so that it spans [0, 1] like 1 - HHI does:
        h_j = (1-alpha) sum_{B_j} s + alpha * ( -sum_i t_i ln t_i ) / ln b,  t_i = s_i / sum_{B_j} s.
    """
    if metric not in ("hhi", "entropy"):
        raise ValueError(metric)
    x = np.asarray(x, F64)
    L = x.shape[0]
    m = L // b
    s = softmax(x)
    h = np.empty(m, F64)
    for j in range(m):
        blk = slice(j * b, (j + 1) * b)
        mass = s[blk].sum()
        e = np.exp(x[blk] - x[blk].max())
        if metric == "hhi":
            spread = 1.0 - (e * e).sum() / (e.sum() ** 2)
        else:
            t = e / e.sum()
            nz = t > 0.0                          # 0 ln 0 = 0
            spread = -(t[nz] * np.log(t[nz])).sum() / np.log(b)
        h[j] = (1.0 - alpha) * mass + alpha * spread
    return h


def block_ranks(h: np.ndarray) -> np.ndarray:
    """rank_j = position of block j in ascending order of h, ties to the lower j
    (I = SortIndex(h), Sec. IV-B)."""
    order = np.argsort(np.asarray(h, F64), kind="stable")
    rank = np.empty_like(order)
    rank[order] = np.arange(len(order))
    return rank


def block_budgets(b: int, h: np.ndarray, p: np.ndarray) -> np.ndarray:
    """t_j = Psi[rank_j] (Eq. 7): the r-th smallest h takes the r-th entry of Psi."""
    m = len(h)
    if m == 0:
        return np.zeros(0, np.int64)
    return psi_list(b, m, p)[block_ranks(h)]


# --------------------------------------------------------------------------
# Eq. 8 : per-block top-t
# --------------------------------------------------------------------------
def top_t(x_block: np.ndarray, t: int) -> np.ndarray:
    """Positions (within the block) of the t largest scores, ties to the lower
    position; returned ascending (Eq. 8).  softmax is monotone, so ranking the
    logits ranks s."""
    order = np.argsort(-np.asarray(x_block, F64), kind="stable")
    return np.sort(order[:t])


@dataclass
class Selection:
    """Everything Alg. 2 lines 1-6 produce for one head."""
    S: np.ndarray                 # selected positions, ascending (global subset)
    x: np.ndarray                 # logits of the last query, all L keys
    h: np.ndarray                 # Eq. 6 per block
    t: np.ndarray                 # Eq. 7 per block


def select(q_last, K, b: int, p, alpha: float, scale: float | None = None, metric: str = "hhi") -> Selection:
    """Alg. 2 lines 1-6 for one head: scores, blocks, metric, ranking, budgets, top-t."""
    K = np.asarray(K, F64)
    L = K.shape[0]
    m = L // b
    x = last_query_logits(q_last, K, scale)
    h = block_metric(x, b, alpha, metric)
    t = block_budgets(b, h, p)
    parts = [j * b + top_t(x[j * b:(j + 1) * b], int(t[j])) for j in range(m)]
    S = np.concatenate(parts).astype(np.int64) if parts else np.zeros(0, np.int64)
    return Selection(S=S, x=x, h=h, t=t)


def kv_head_of(h: int, n_q_heads: int, n_kv_heads: int) -> int:
    return h // (n_q_heads // n_kv_heads)


def select_all_heads(q_last, K, b, p, alpha, scale=None, metric: str = "hhi") -> list[Selection]:
    """q_last [Hq,d], K [Hkv,L,d], p [Hq,nk]: one independent selection per query head."""
    Hq, Hkv = q_last.shape[0], K.shape[0]
    return [select(q_last[h], K[kv_head_of(h, Hq, Hkv)], b, p[h], alpha, scale, metric) for h in range(Hq)]


# --------------------------------------------------------------------------
# Group-shared selection for GQA (extension; the paper applies Eq. 5-8 per head)
# --------------------------------------------------------------------------
def group_scores_from_logits(X: np.ndarray) -> np.ndarray:
    """sbar_i = (1/G) sum_g softmax(X_g)_i : the mean of the group's Eq. 5 scores.
    X [G, L] holds the last-query logits of the G query heads that share one KV head."""
    X = np.asarray(X, F64)
    return np.stack([softmax(X[g]) for g in range(X.shape[0])]).sum(axis=0) / X.shape[0]


def block_metric_of_scores(s: np.ndarray, b: int, alpha: float, metric: str = "hhi") -> np.ndarray:
    """Eq. 6 written on scores rather than logits:
    h_j = (1-alpha) sum_{B_j} s + alpha (1 - sum s^2 / (sum s)^2), or with the entropy of
    s / sum_{B_j} s over ln b as the second term.  s must not underflow to zero over a whole block."""
    if metric not in ("hhi", "entropy"):
        raise ValueError(metric)
    s = np.asarray(s, F64)
    m = s.shape[0] // b
    h = np.empty(m, F64)
    for j in range(m):
        sb = s[j * b:(j + 1) * b]
        mass = sb.sum()
        if metric == "hhi":
            spread = 1.0 - (sb * sb).sum() / (mass * mass)
        else:
            t = sb / mass
            nz = t > 0.0
            spread = -(t[nz] * np.log(t[nz])).sum() / np.log(b)
        h[j] = (1.0 - alpha) * mass + alpha * spread
    return h


def select_shared(q_group, K, b: int, p, alpha: float, scale: float | None = None,
                  metric: str = "hhi") -> Selection:
    """Alg. 2 lines 1-6 for one KV head shared by the query heads q_group [G, d]:
    the token score is the group mean of Eq. 5; Eq. 6, 7, 8 as for a single head.
    Selection.x holds ln(sbar) (the quantity comparable to a logit)."""
    K = np.asarray(K, F64)
    q_group = np.asarray(q_group, F64)
    L = K.shape[0]
    m = L // b
    X = np.stack([last_query_logits(q_group[g], K, scale) for g in range(q_group.shape[0])])
    sbar = group_scores_from_logits(X)
    h = block_metric_of_scores(sbar, b, alpha, metric)
    t = block_budgets(b, h, p)
    parts = [j * b + top_t(sbar[j * b:(j + 1) * b], int(t[j])) for j in range(m)]
    S = np.concatenate(parts).astype(np.int64) if parts else np.zeros(0, np.int64)
    with np.errstate(divide="ignore"):
        return Selection(S=S, x=np.log(sbar), h=h, t=t)


def select_all_groups(q_last, K, b, p, alpha, scale=None, metric: str = "hhi") -> list[Selection]:
    """q_last [Hq,d], K [Hkv,L,d], p [Hkv,nk]: one selection per KV head."""
    Hq, Hkv = q_last.shape[0], K.shape[0]
    G = Hq // Hkv
    return [select_shared(q_last[g * G:(g + 1) * G], K[g], b, p[g], alpha, scale, metric) for g in range(Hkv)]


# --------------------------------------------------------------------------
# Eq. 1 and Eq. 2 : attention
# --------------------------------------------------------------------------
def dense_causal_attention(Q, K, V, scale: float | None = None) -> np.ndarray:
    """Eq. 1 for one head with the causal mask of an autoregressive model."""
    Q, K, V = (np.asarray(a, F64) for a in (Q, K, V))
    L, d = Q.shape
    sc = default_scale(d) if scale is None else scale
    out = np.empty((L, V.shape[1]), F64)
    for i in range(L):
        a = softmax(K[: i + 1] @ Q[i] * sc)
        out[i] = a @ V[: i + 1]
    return out


def visible_keys(i: int, S: np.ndarray, w: int) -> np.ndarray:
    """Key positions query i attends to (Eq. 2): the global rows that have left
    its window, then the window (i-w, i] itself."""
    S = np.asarray(S, np.int64)
    glob = S[S <= i - w]
    local = np.arange(max(0, i - w + 1), i + 1, dtype=np.int64)
    return np.concatenate([glob, local])


def attention_row(q_i, i: int, K, V, S, w: int, scale: float | None = None) -> np.ndarray:
    """Eq. 2 for the query at position i: softmax over [K^G; K^L] times [V^G; V^L]."""
    q_i, K, V = (np.asarray(a, F64) for a in (q_i, K, V))
    sc = default_scale(K.shape[1]) if scale is None else scale
    T = visible_keys(i, S, w)
    a = softmax(K[T] @ q_i * sc)
    return a @ V[T]


def tca_attention(Q, K, V, S, w: int, scale: float | None = None, q_pos0: int = 0) -> np.ndarray:
    """Eq. 2 for every query of one head (Alg. 2 line 7).  Q row r sits at
    position q_pos0 + r."""
    Q = np.asarray(Q, F64)
    return np.stack([attention_row(Q[r], q_pos0 + r, K, V, S, w, scale) for r in range(Q.shape[0])])


def tca_prefill(Q, K, V, b: int, w: int, p, alpha: float, scale: float | None = None, share: bool = False):
    """Alg. 2 for all heads.  Q [Hq,L,d], K,V [Hkv,L,d], p [Hq,nk] (share: [Hkv,nk]).
    Returns (O [Hq,L,d], list of Selection: one per query head, or per KV head when share)."""
    Hq, L, _ = Q.shape
    Hkv = K.shape[0]
    q_last = np.asarray(Q)[:, L - 1, :]
    sels = select_all_groups(q_last, K, b, p, alpha, scale) if share else select_all_heads(q_last, K, b, p, alpha, scale)
    O = np.stack([
        tca_attention(Q[h], K[kv_head_of(h, Hq, Hkv)], V[kv_head_of(h, Hq, Hkv)],
                      sels[kv_head_of(h, Hq, Hkv) if share else h].S, w, scale)
        for h in range(Hq)
    ])
    return O, sels


def tca_prefill_chunked(Q, K, V, b: int, w: int, p, alpha: float, chunk: int, scale: float | None = None,
                        share: bool = False):
    """Chunked prefill.  NOT in the paper: a serving extension, defined here as
    follows.  The sequence arrives in chunks of `chunk` tokens (a multiple of b).
    For the chunk covering positions [c0, c1): the chunk's last query scores the
    chunk's own keys only (Eq. 5 restricted to [c0, c1)), Eq. 6-8 run over the
    chunk's full blocks with the head's configuration, and the kept positions
    are appended to the head's global subset; then every query of the chunk
    attends (Eq. 2) to the global subset as it stands - rows kept from earlier
    chunks and from this one, visible once they have left the query's window -
    plus its window.  With one chunk covering the sequence this is Alg. 2.

    Q [Hq,L,d], K,V [Hkv,L,d], p [Hq,nk].  Returns (O [Hq,L,d], list of index sets).
    share: one set per KV head (p [Hkv,nk]), each chunk scored by the group mean of its last queries.
    """
    Q, K, V = (np.asarray(a, F64) for a in (Q, K, V))
    Hq, L, _ = Q.shape
    Hkv = K.shape[0]
    if chunk % b != 0:
        raise ValueError("chunk must be a multiple of the block size")
    G = Hq // Hkv
    S = [np.zeros(0, np.int64) for _ in range(Hkv if share else Hq)]
    O = np.empty((Hq, L, V.shape[2]), F64)
    for c0 in range(0, L, chunk):
        c1 = min(L, c0 + chunk)
        for n in range(len(S)):
            if share:
                sel = select_shared(Q[n * G:(n + 1) * G, c1 - 1], K[n, c0:c1], b, p[n], alpha, scale)
            else:
                sel = select(Q[n, c1 - 1], K[kv_head_of(n, Hq, Hkv), c0:c1], b, p[n], alpha, scale)
            S[n] = np.concatenate([S[n], c0 + sel.S]).astype(np.int64)
        for h in range(Hq):
            g = kv_head_of(h, Hq, Hkv)
            O[h, c0:c1] = tca_attention(Q[h, c0:c1], K[g, :c1], V[g, :c1], S[g if share else h], w, scale, q_pos0=c0)
    return O, S


# --------------------------------------------------------------------------
# Decode stage (Sec. IV-B, "Online Token Selection in Decoding Stage")
# --------------------------------------------------------------------------
@dataclass
class HeadCache:
    """KV cache of one sequence: per query head the global subset (positions,
    ascending), plus every dense row seen so far so the window can be read from
    it (a real cache keeps only the last w of them)."""
    S: list = field(default_factory=list)      # [Hq] int64 arrays ([Hkv] with group-shared selection)
    K: np.ndarray | None = None                # [Hkv, T, d] all rows so far
    V: np.ndarray | None = None

    @property
    def length(self) -> int:
        return 0 if self.K is None else self.K.shape[1]


def cache_after_prefill(K, V, sels: list[Selection], kv_quant: str | None = None) -> HeadCache:
    """State after Alg. 2: global = S (all of it), local = the dense rows.
    kv_quant="fp8": the cache stores every row as FP8 E4M3 codes with one scale per row; what the
    decode steps read is the dequantised row (quantisation is per row, so quantising all rows and
    reading those in S or in the window is the same as quantising only what the cache keeps)."""
    K, V = np.asarray(K, F64), np.asarray(V, F64)
    if kv_quant == "fp8":
        K, V = roundtrip_rows_fp8(K), roundtrip_rows_fp8(V)
    elif kv_quant is not None:
        raise ValueError(kv_quant)
    return HeadCache(S=[s.S.copy() for s in sels], K=K.copy(), V=V.copy())


def decode_step(cache: HeadCache, q, k_new, v_new, b: int, w: int, p, scale: float | None = None,
                share: bool = False, kv_quant: str | None = None) -> np.ndarray:
    """One generated token.  q [Hq,d]; k_new, v_new [Hkv,d] are the rows of the
    token at position T = cache.length, appended before attending.

    Attention: Eq. 2 for a single query at position T.
    Selection: if T is the last position of a block, that block's b rows are
    scored with this step's query (Eq. 5 restricted to the block) and the top
    t = floor(sum_k k p_k) positions are appended to the head's global subset.
    share: cache.S and p are per KV head; the block's rows are ranked by the group
    mean of the heads' scores, each normalised over the block.
    kv_quant="fp8": the new rows enter the cache as FP8 codes with a scale per row; attention and
    the scoring of a completed block read the dequantised rows.
    """
    q = np.asarray(q, F64)
    Hq, d = q.shape
    Hkv = np.asarray(k_new).shape[0]
    T = cache.length
    k_new = np.asarray(k_new, F64)[:, None, :]
    v_new = np.asarray(v_new, F64)[:, None, :]
    if kv_quant == "fp8":
        k_new, v_new = roundtrip_rows_fp8(k_new), roundtrip_rows_fp8(v_new)
    elif kv_quant is not None:
        raise ValueError(kv_quant)
    cache.K = k_new if cache.K is None else np.concatenate([cache.K, k_new], axis=1)
    cache.V = v_new if cache.V is None else np.concatenate([cache.V, v_new], axis=1)
    out = np.empty((Hq, cache.V.shape[2]), F64)
    for h in range(Hq):
        g = kv_head_of(h, Hq, Hkv)
        out[h] = attention_row(q[h], T, cache.K[g], cache.V[g], cache.S[g if share else h], w, scale)
    if (T + 1) % b == 0:
        j = T // b
        G = Hq // Hkv
        for n in range(len(cache.S)):
            if share:
                X = np.stack([last_query_logits(q[h], cache.K[n, j * b:(j + 1) * b], scale)
                              for h in range(n * G, (n + 1) * G)])
                x = group_scores_from_logits(X)
            else:
                x = last_query_logits(q[n], cache.K[kv_head_of(n, Hq, Hkv), j * b:(j + 1) * b], scale)
            keep = j * b + top_t(x, decode_budget(b, p[n]))
            cache.S[n] = np.concatenate([cache.S[n], keep]).astype(np.int64)
    return out


# --------------------------------------------------------------------------
# Alg. 1 and Eq. 4 : offline head-specific sparsity determination
# --------------------------------------------------------------------------
def dense_causal_probs(Q, K, scale: float | None = None) -> np.ndarray:
    """A = softmax(Q K^T / sqrt(d_h)) with the causal mask, [L, L] (Alg. 1 line 1)."""
    Q, K = np.asarray(Q, F64), np.asarray(K, F64)
    L, d = Q.shape
    sc = default_scale(d) if scale is None else scale
    A = np.zeros((L, L), F64)
    for i in range(L):
        A[i, : i + 1] = softmax(K[: i + 1] @ Q[i] * sc)
    return A


def column_means(A: np.ndarray) -> np.ndarray:
    """Inner term of Eq. 4: mean of column k of A over the rows that can see
    key k, i.e. the L-k rows j >= k (0-based)."""
    L = A.shape[0]
    return np.array([A[k:, k].sum() / (L - k) for k in range(L)], F64)


def cumulative_score(abar: np.ndarray, S: np.ndarray) -> float:
    """Eq. 4: a_i = sum over the selected tokens of their column mean."""
    return float(abar[np.asarray(S, np.int64)].sum())


@dataclass
class Calibration:
    index: int            # chosen candidate, 0-based
    p: np.ndarray         # chosen configuration
    a: np.ndarray         # a_i for every candidate
    n: np.ndarray         # |S_i| for every candidate
    fallback: bool        # True if no candidate reached tau


def calibrate_head(Q, K, b: int, cands: np.ndarray, tau: float, alpha: float,
                   scale: float | None = None) -> Calibration:
    """Alg. 1 for one head on one calibration sequence."""
    Q = np.asarray(Q, F64)
    L = Q.shape[0]
    abar = column_means(dense_causal_probs(Q, K, scale))
    a = np.empty(len(cands), F64)
    n = np.empty(len(cands), np.int64)
    for i, p in enumerate(cands):
        S = select(Q[L - 1], K, b, p, alpha, scale).S
        a[i] = cumulative_score(abar, S)
        n[i] = len(S)
    valid = [i for i in range(len(cands)) if a[i] >= tau]
    if valid:
        best = min(valid, key=lambda i: (n[i], i))
        return Calibration(best, cands[best].copy(), a, n, False)
    last = len(cands) - 1
    return Calibration(last, cands[last].copy(), a, n, True)


def calibrate_group(Qg, K, b: int, cands: np.ndarray, tau: float, alpha: float,
                    scale: float | None = None) -> Calibration:
    """Alg. 1 for one KV head with group-shared selection: Qg [G,L,d].  The importance of
    key k is the mean over the group of the heads' column means (Eq. 4 inner term), the
    candidate sets come from `select_shared`."""
    Qg = np.asarray(Qg, F64)
    G, L, _ = Qg.shape
    abar = np.stack([column_means(dense_causal_probs(Qg[g], K, scale)) for g in range(G)]).sum(axis=0) / G
    a = np.empty(len(cands), F64)
    n = np.empty(len(cands), np.int64)
    for i, p in enumerate(cands):
        S = select_shared(Qg[:, L - 1], K, b, p, alpha, scale).S
        a[i] = cumulative_score(abar, S)
        n[i] = len(S)
    valid = [i for i in range(len(cands)) if a[i] >= tau]
    if valid:
        best = min(valid, key=lambda i: (n[i], i))
        return Calibration(best, cands[best].copy(), a, n, False)
    last = len(cands) - 1
    return Calibration(last, cands[last].copy(), a, n, True)


def calibrate(Q, K, b: int, M: int, sigma: float, tau: float, alpha: float,
              scale: float | None = None, share: bool = False) -> list[Calibration]:
    """Alg. 1 for all heads.  Q [Hq,L,d], K [Hkv,L,d].  share: one result per KV head."""
    Hq, Hkv = Q.shape[0], K.shape[0]
    cands = candidates(b, M, sigma)
    if share:
        G = Hq // Hkv
        return [calibrate_group(Q[g * G:(g + 1) * G], K[g], b, cands, tau, alpha, scale) for g in range(Hkv)]
    return [calibrate_head(Q[h], K[kv_head_of(h, Hq, Hkv)], b, cands, tau, alpha, scale) for h in range(Hq)]


# --------------------------------------------------------------------------
# Theorem 1 quantities
# --------------------------------------------------------------------------
def theorem_quantities(q_i, i: int, K, V, S, w: int, scale: float | None = None):
    """For query i: gamma_i (dense causal softmax mass on omitted keys), the
    l1 distance between the dense and the sparse distributions, and both
    outputs (Theorem 1 and its proof)."""
    q_i, K, V = (np.asarray(a, F64) for a in (q_i, K, V))
    sc = default_scale(K.shape[1]) if scale is None else scale
    s_full = softmax(K[: i + 1] @ q_i * sc)
    T = visible_keys(i, S, w)
    keep = np.zeros(i + 1, bool)
    keep[T] = True
    gamma = float(s_full[~keep].sum())
    s_sparse = np.zeros(i + 1, F64)
    s_sparse[T] = softmax(K[T] @ q_i * sc)
    l1 = float(np.abs(s_full - s_sparse).sum())
    return gamma, l1, s_full @ V[: i + 1], s_sparse @ V[: i + 1]


# --------------------------------------------------------------------------
# Layer integration (extensions around the path; none of this is in the paper)
# --------------------------------------------------------------------------
# FP8 E4M3 (OCP 8-bit floating point, "E4M3": 1 sign, 4 exponent bits with bias 7, 3 mantissa
# bits; no infinities; S.1111.111 is NaN; largest finite value 448 = 1.75 * 2^8; subnormals
# m/8 * 2^-6).  A cache row x of d numbers is stored as d codes and one float32 scale:
#     amax = max_i |x_i|,  scale = amax / 448 (1 if amax = 0),  code_i = RNE_e4m3(x_i / scale)
# with the two divisions in float32 (the decision of a code is taken in the precision the
# kernel takes it in); the row read back is code_i * scale, exact in float64.
FP8_MAX = 448.0


def fp8_e4m3_values() -> np.ndarray:
    """The 256 codes' values in float64, written out from the format definition (NaN for 0x7f, 0xff)."""
    out = np.empty(256, F64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e, m = (code >> 3) & 0xF, code & 0x7
        if e == 0xF and m == 0x7:
            out[code] = np.nan
        elif e == 0:
            out[code] = sign * (m / 8.0) * 2.0 ** -6
        else:
            out[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return out


def fp8_e4m3_encode(y) -> np.ndarray:
    """Round-to-nearest-even of float32 numbers to E4M3 codes, saturating at +-448.  Done by
    search over the table of values, not by bit manipulation: the nearest representable value
    wins, a tie goes to the code with an even mantissa field."""
    y = np.asarray(y, np.float32).astype(F64)
    vals = fp8_e4m3_values()
    pos_codes = np.arange(0, 0x7F)                       # 0 .. 448, ascending in value
    pos_vals = vals[pos_codes]
    a = np.minimum(np.abs(y), FP8_MAX)
    hi = np.searchsorted(pos_vals, a, side="left")       # first value >= a
    hi = np.minimum(hi, len(pos_vals) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - pos_vals[lo], pos_vals[hi] - a
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (pos_codes[hi] % 2 == 0))
    code = np.where(take_hi, pos_codes[hi], pos_codes[lo]).astype(np.uint8)
    return np.where(np.signbit(y), code | 0x80, code).astype(np.uint8)


def quantize_rows_fp8(X):
    """Rows along the last axis -> (codes uint8, same shape; scales float32, one per row)."""
    X32 = np.asarray(X, np.float32)
    amax = np.max(np.abs(X32), axis=-1)
    scale = np.where(amax > 0, amax / np.float32(FP8_MAX), np.float32(1.0)).astype(np.float32)
    y = (X32 / scale[..., None]).astype(np.float32)
    return fp8_e4m3_encode(y), scale


def dequantize_rows_fp8(codes, scales) -> np.ndarray:
    return fp8_e4m3_values()[np.asarray(codes, np.uint8)] * np.asarray(scales, F64)[..., None]


def roundtrip_rows_fp8(X) -> np.ndarray:
    """What an FP8 cache returns for the rows X."""
    return dequantize_rows_fp8(*quantize_rows_fp8(X))


def rope_rotate(X, positions, base: float = 10000.0, pairing: str = "half") -> np.ndarray:
    """Rotary position embedding (the RoFormer rotation) of the rows of X [..., n, d] at the given
    positions [n]: the pair (x_a, x_b) of a row at position t is turned by the angle
    t * base^(-2 i / d), i = 0 .. d/2-1.  pairing="half": pair i is (i, i + d/2) (the layout of
    Llama-family checkpoints); "interleaved": pair i is (2i, 2i+1) (the original paper's)."""
    X = np.asarray(X, F64)
    d = X.shape[-1]
    t = np.asarray(positions, F64)
    inv_freq = base ** (-2.0 * np.arange(d // 2, dtype=F64) / d)
    ang = t[:, None] * inv_freq[None, :]                 # [n, d/2]
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(X)
    if pairing == "half":
        a, b = X[..., : d // 2], X[..., d // 2:]
        out[..., : d // 2] = a * c - b * s
        out[..., d // 2:] = b * c + a * s
    elif pairing == "interleaved":
        a, b = X[..., 0::2], X[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = b * c + a * s
    else:
        raise ValueError(pairing)
    return out


def qkv_project(X, W, n_q_heads: int, n_kv_heads: int, d: int, bias=None):
    """The projections that produce what the method takes as given (Sec. III: Q = X W_Q,
    K = X W_K, V = X W_V, per head): X [n, hidden] are the layer's input rows; W [(Hq + 2 Hkv) d,
    hidden] holds one row per output feature, the Hq query heads first, then the Hkv key heads,
    then the Hkv value heads, d rows each (so W_Q of head h is W[h d : (h+1) d].T); bias, if
    given, [(Hq + 2 Hkv) d] is added to the features.  Returns Q [Hq, n, d], K [Hkv, n, d],
    V [Hkv, n, d]."""
    X, W = np.asarray(X, F64), np.asarray(W, F64)
    n, Hq, Hkv = X.shape[0], n_q_heads, n_kv_heads
    assert W.shape == ((Hq + 2 * Hkv) * d, X.shape[1])
    Y = X @ W.T                                          # [n, features]
    if bias is not None:
        Y = Y + np.asarray(bias, F64)[None, :]
    Y = Y.reshape(n, Hq + 2 * Hkv, d).transpose(1, 0, 2)  # [head, n, d]
    return Y[:Hq].copy(), Y[Hq:Hq + Hkv].copy(), Y[Hq + Hkv:].copy()


def calibrate_layers(Qs, Ks, b: int, M: int, sigma: float, tau: float, alpha: float, share: bool = False):
    """Alg. 1 applied to every layer of a model in turn (Sec. IV-A: the determination is made
    once per model, for all heads of all layers): Qs[l] [Hq, L, d], Ks[l] [Hkv, L, d] are the
    calibration sample's queries and keys at layer l.  Returns one list of Calibration per layer."""
    return [calibrate(Qs[l], Ks[l], b, M, sigma, tau, alpha, share=share) for l in range(len(Qs))]
