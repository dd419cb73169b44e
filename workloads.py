"""Seeded synthetic inputs for the TCA hot path.

This module holds input generation only: random draws, the structure the
workload descriptions ask for (centroid copies, low-rank keys, near-duplicate
rows, per-head query gains, budget fractions) and the one rounding to the
storage type.  It contains none of the method's arithmetic and is the only
module both the CPU oracle's tests and the GPU path's tests/benchmark share.

Storage types: "f32" arrays are numpy float32; "bf16" arrays are numpy uint16
holding bfloat16 bit patterns (round-to-nearest-even from float32).  `to_f64`
widens either exactly.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------- dtypes --
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float array once to the storage type."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored array (float32, or uint16 bf16 bits) to float64."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# ------------------------------------------------------------- generators --
def keys_centroid(rng, L: int, d: int, n_centroids: int = 64, copy_frac: float = 0.5,
                  noise_std: float = 0.05) -> np.ndarray:
    """Half the rows are copies of seeded centroids plus small noise, the rest
    N(0,1): clustered, partly redundant keys."""
    cent = rng.standard_normal((n_centroids, d), dtype=np.float32)
    K = rng.standard_normal((L, d), dtype=np.float32)
    n_copy = int(round(copy_frac * L))
    rows = rng.permutation(L)[:n_copy]
    which = rng.integers(0, n_centroids, size=n_copy)
    K[rows] = cent[which] + noise_std * rng.standard_normal((n_copy, d), dtype=np.float32)
    return K


def keys_lowrank(rng, L: int, d: int, rank: int = 32, noise_std: float = 0.1,
                 dup_frac: float = 0.3, dup_noise_std: float = 0.01) -> np.ndarray:
    """Low-rank signal plus noise; a seeded fraction of rows is replaced by a
    copy of an earlier row of the base matrix plus tiny noise (near duplicates)."""
    U = rng.standard_normal((L, rank), dtype=np.float32)
    W = rng.standard_normal((d, rank), dtype=np.float32)
    K = (U @ W.T) / np.float32(np.sqrt(rank))
    K += np.float32(noise_std) * rng.standard_normal((L, d), dtype=np.float32)
    n_dup = int(round(dup_frac * L))
    rows = np.sort(rng.permutation(np.arange(1, L))[:n_dup]) if L > 1 else np.zeros(0, np.int64)
    src = (rng.random(len(rows)) * rows).astype(np.int64)          # uniform in [0, row)
    base = K.copy()
    K[rows] = base[src] + np.float32(dup_noise_std) * rng.standard_normal((len(rows), d), dtype=np.float32)
    return K


def head_gains(rng, Hq: int, lo: float = 1.0, hi: float = 8.0) -> np.ndarray:
    """Per-head query gain, log-uniform: small gain = near-uniform attention,
    large gain = peaked attention."""
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=Hq)).astype(np.float32)


def budget_fractions(seed: int, Hq: int, lo: float = 0.05, hi: float = 0.5) -> np.ndarray:
    """Per-head budget as a fraction of L, uniform in [lo, hi]."""
    return np.random.default_rng(seed).uniform(lo, hi, size=Hq)


def prefill_inputs(kind: str, Hq: int, Hkv: int, d: int, L: int, dtype: str, seed: int) -> dict:
    """Q [Hq,L,d], K,V [Hkv,L,d] in storage type `dtype`.

    kind "centroid": Q,V ~ N(0,1); K from `keys_centroid`.
    kind "lowrank" : Q ~ g_h N(0,1) with per-head gains; V ~ N(0,1); K from `keys_lowrank`.
    """
    rng = np.random.default_rng(seed)
    if kind == "centroid":
        K = np.stack([keys_centroid(rng, L, d) for _ in range(Hkv)])
        gains = np.ones(Hq, np.float32)
    elif kind == "lowrank":
        K = np.stack([keys_lowrank(rng, L, d) for _ in range(Hkv)])
        gains = head_gains(rng, Hq)
    else:
        raise ValueError(kind)
    V = rng.standard_normal((Hkv, L, d), dtype=np.float32)
    Q = np.empty((Hq, L, d), np.uint16 if dtype == "bf16" else np.float32)
    for h in range(Hq):                       # per head: bounds the float32 scratch
        Q[h] = store(gains[h] * rng.standard_normal((L, d), dtype=np.float32), dtype)
    return {"Q": Q, "K": store(K, dtype), "V": store(V, dtype), "gains": gains}


def decode_inputs(Hq: int, Hkv: int, d: int, n_steps: int, dtype: str, seed: int, batch: int = 1,
                  gains: np.ndarray | None = None) -> dict:
    """Per decode step: q [steps,B,Hq,d], k_new,v_new [steps,B,Hkv,d] ~ N(0,1) (q times head gain)."""
    rng = np.random.default_rng(seed)
    g = np.ones(Hq, np.float32) if gains is None else gains
    q = rng.standard_normal((n_steps, batch, Hq, d), dtype=np.float32) * g[None, None, :, None]
    k = rng.standard_normal((n_steps, batch, Hkv, d), dtype=np.float32)
    v = rng.standard_normal((n_steps, batch, Hkv, d), dtype=np.float32)
    return {"q": store(q, dtype), "k_new": store(k, dtype), "v_new": store(v, dtype)}


def compacted_cache_inputs(Hq: int, Hkv: int, d: int, T0: int, w: int, b: int, n_rows: np.ndarray,
                           dtype: str, seed: int) -> dict:
    """A cache as it stands after T0 tokens without running prefill: per head
    `n_rows[h]` global rows at ascending random positions < T0 (rows themselves
    from the low-rank generator), plus the last w dense rows per KV head.

    Returns idx (list of int32 arrays), Kg/Vg (lists, stored dtype), ringK/ringV
    [Hkv,w,d] holding positions T0-w..T0-1 in position order.
    """
    rng = np.random.default_rng(seed)
    idx, Kg, Vg = [], [], []
    for h in range(Hq):
        n = int(n_rows[h])
        pos = np.sort(rng.choice(T0, size=n, replace=False)).astype(np.int32) if n else np.zeros(0, np.int32)
        idx.append(pos)
        Kg.append(store(keys_lowrank(rng, max(n, 2), d)[:n], dtype))
        Vg.append(store(rng.standard_normal((n, d), dtype=np.float32), dtype))
    ringK = store(np.stack([keys_lowrank(rng, w, d) for _ in range(Hkv)]), dtype)
    ringV = store(rng.standard_normal((Hkv, w, d), dtype=np.float32), dtype)
    return {"idx": idx, "Kg": Kg, "Vg": Vg, "ringK": ringK, "ringV": ringV}


# ------------------------------------------------ the named configurations --
CONFIGS = {
    # small fp32 case: whole oracle in seconds.  b and w are scaled down with L
    # (the paper's b=128, w=4096 would make L=1024 dense).
    1: dict(kind="centroid", Hq=4, Hkv=1, d=64, L=1024, dtype="f32", b=32, w=128, alpha=0.5, sigma=1.0,
            budget=0.25),
    # Llama-3-8B-shaped layer, 32K
    2: dict(kind="lowrank", Hq=32, Hkv=8, d=128, L=32768, dtype="bf16", b=128, w=4096, alpha=0.5, sigma=1.0),
    # same at 128K, budgets from calibration on a separate 8K sample
    3: dict(kind="lowrank", Hq=32, Hkv=8, d=128, L=131072, dtype="bf16", b=128, w=4096, alpha=0.5, sigma=1.0,
            L_cal=8192, M=14, tau=0.9),
    # decode at 128K, batch 16
    4: dict(kind="lowrank", Hq=32, Hkv=8, d=128, L=131072, dtype="bf16", b=128, w=4096, alpha=0.5, sigma=1.0,
            batch=16, steps=64),
}


def data_seed(cfg_id: int) -> int:
    return 1000 + cfg_id


def budget_seed(cfg_id: int) -> int:
    return 2000 + cfg_id


def calib_seed(cfg_id: int) -> int:
    return 3000 + cfg_id


def projection_inputs(Hq: int, Hkv: int, d: int, hidden: int, n: int, dtype: str, seed: int) -> dict:
    """Inputs of the Q / K / V projections in front of the path: n rows of hidden states of unit
    scale (what a normalisation layer hands on), one weight row per output feature of scale
    1/sqrt(hidden) (outputs of unit scale), a bias of scale 0.1; each rounded once to the storage type."""
    rng = np.random.default_rng(seed)
    n_feat = (Hq + 2 * Hkv) * d
    return {"X": store(rng.standard_normal((n, hidden), dtype=np.float32), dtype),
            "W": store(rng.standard_normal((n_feat, hidden), dtype=np.float32) / np.float32(hidden ** 0.5), dtype),
            "bias": store(np.float32(0.1) * rng.standard_normal(n_feat, dtype=np.float32), dtype)}


def device_projection_inputs(Hq: int, Hkv: int, d: int, hidden: int, n: int, seed: int, device="cuda:0"):
    """The recipe of `projection_inputs` in bf16, drawn on the GPU with a seeded torch generator."""
    import torch
    g = torch.Generator(device=device).manual_seed(seed)
    n_feat = (Hq + 2 * Hkv) * d
    X = torch.empty(n, hidden, device=device, dtype=torch.bfloat16)
    for r0 in range(0, n, 16384):                        # in slabs: no fp32 copy of the whole array
        r1 = min(n, r0 + 16384)
        X[r0:r1] = torch.randn(r1 - r0, hidden, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    W = (torch.randn(n_feat, hidden, generator=g, device=device, dtype=torch.float32) / hidden ** 0.5).to(torch.bfloat16)
    bias = (0.1 * torch.randn(n_feat, generator=g, device=device, dtype=torch.float32)).to(torch.bfloat16)
    return {"X": X, "W": W, "bias": bias}


# ------------------------------------------- device-side generation (large) --
def device_lowrank_inputs(Hq: int, Hkv: int, d: int, L: int, seed: int, device="cuda:0", rank: int = 32,
                          noise_std: float = 0.1, dup_frac: float = 0.3, dup_noise_std: float = 0.01):
    """The "lowrank" recipe of `prefill_inputs`, drawn on the GPU with a seeded torch
    generator (for workloads too large to build on the host in reasonable time).
    Returns bf16 torch tensors Q [Hq,L,d], K,V [Hkv,L,d] and the per-head gains."""
    import torch
    g = torch.Generator(device=device).manual_seed(seed)
    rn = lambda *shape: torch.randn(*shape, generator=g, device=device, dtype=torch.float32)
    K = torch.empty(Hkv, L, d, device=device, dtype=torch.bfloat16)
    for kv in range(Hkv):
        U, W = rn(L, rank), rn(d, rank)
        base = (U @ W.T) / rank ** 0.5 + noise_std * rn(L, d)
        n_dup = int(round(dup_frac * L))
        rows = torch.randperm(L - 1, generator=g, device=device)[:n_dup] + 1
        src = (torch.rand(n_dup, generator=g, device=device) * rows).long()
        out = base.clone()
        out[rows] = base[src] + dup_noise_std * rn(n_dup, d)
        K[kv] = out.to(torch.bfloat16)
    V = rn(Hkv, L, d).to(torch.bfloat16)
    gains = torch.exp(torch.rand(Hq, generator=g, device=device) * float(np.log(8.0)))
    Q = torch.empty(Hq, L, d, device=device, dtype=torch.bfloat16)
    for h in range(Hq):
        Q[h] = (gains[h] * rn(L, d)).to(torch.bfloat16)
    return {"Q": Q, "K": K, "V": V, "gains": gains}


CONFIGS[5] = dict(kind="lowrank", Hq=64, Hkv=8, d=128, dtype="bf16", b=128, w=4096, alpha=0.5, sigma=1.0,
                  n_seqs=8, len_lo=4096, len_hi=131072, chunk=8192, L_cal=8192, M=14, tau=0.9)


def config5_lengths(seed: int = 1005) -> list:
    """8 sequence lengths, log-uniform in [4096, 131072]."""
    c = CONFIGS[5]
    rng = np.random.default_rng(seed)
    return [int(x) for x in np.exp(rng.uniform(np.log(c["len_lo"]), np.log(c["len_hi"]), size=c["n_seqs"]))]
