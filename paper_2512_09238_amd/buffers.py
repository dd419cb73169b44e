"""Device-memory plumbing (torch): storage-type conversion of host arrays,
workspaces, the flat global buffers and the decode cache.  No method arithmetic."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as tb


def torch_dtype(prm) -> torch.dtype:
    return torch.bfloat16 if prm.dtype == tb.TCA_BF16 else torch.float32


def to_device(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """numpy float32 -> float32 tensor; numpy uint16 (bf16 bit patterns) -> bfloat16 tensor."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def workspace(nbytes: int, device="cuda:0") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class GlobalBuffers:
    """idx / Kg / Vg / n_rows for one sequence with capacities `cap`, one per selection head."""

    def __init__(self, prm, cap, device="cuda:0"):
        cap = np.asarray(cap, np.int64)
        self.offs = np.concatenate([[0], np.cumsum(cap)]).astype(np.int64)
        total = max(int(self.offs[-1]), 1)
        d = prm.head_dim
        self.idx = torch.zeros(total, dtype=torch.int32, device=device)
        self.Kg = torch.zeros(total, d, dtype=torch_dtype(prm), device=device)
        self.Vg = torch.zeros(total, d, dtype=torch_dtype(prm), device=device)
        self.n_rows = torch.zeros(tb.tca_selection_heads(prm), dtype=torch.int32, device=device)


class DecodeCache:
    """Batch of per-sequence caches sharing one capacity layout."""

    def __init__(self, prm, batch, cap, device="cuda:0", kv_format=tb.TCA_KV_NATIVE):
        cap = np.asarray(cap, np.int64)
        self.offs = np.concatenate([[0], np.cumsum(cap)]).astype(np.int64)
        self.cap_rows = int(self.offs[-1])
        self.max_head_rows = int(cap.max()) if len(cap) else 0
        rows = max(self.cap_rows, 1)
        d, w, Hkv, Hq = prm.head_dim, prm.window, prm.n_kv_heads, tb.tca_selection_heads(prm)
        fp8 = kv_format == tb.TCA_KV_FP8
        dt = torch.uint8 if fp8 else torch_dtype(prm)       # FP8 rows: one code byte per element, scales beside them
        self.kv_format = kv_format
        self.idx = torch.zeros(batch, rows, dtype=torch.int32, device=device)
        self.Kg = torch.zeros(batch, rows, d, dtype=dt, device=device)
        self.Vg = torch.zeros(batch, rows, d, dtype=dt, device=device)
        self.n_rows = torch.zeros(batch, Hq, dtype=torch.int32, device=device)
        self.ringK = torch.zeros(batch, Hkv, w, d, dtype=dt, device=device)
        self.ringV = torch.zeros(batch, Hkv, w, d, dtype=dt, device=device)
        self.length = torch.zeros(batch, dtype=torch.int64, device=device)
        self.batch = batch
        self.Kg_scale = self.Vg_scale = self.ringK_scale = self.ringV_scale = None
        if fp8:
            self.Kg_scale = torch.zeros(batch, rows, dtype=torch.float32, device=device)
            self.Vg_scale = torch.zeros(batch, rows, dtype=torch.float32, device=device)
            self.ringK_scale = torch.zeros(batch, Hkv, w, dtype=torch.float32, device=device)
            self.ringV_scale = torch.zeros(batch, Hkv, w, dtype=torch.float32, device=device)
        self.view = tb.make_cache(batch, self.cap_rows, self.idx, self.Kg, self.Vg, self.n_rows,
                                  self.ringK, self.ringV, self.length, kv_format, self.Kg_scale, self.Vg_scale,
                                  self.ringK_scale, self.ringV_scale)
