"""Plumbing shared by the GPU parity tests: run the C-ABI path on workload
arrays, and compare a GPU index set with the oracle's under the stated rule
(identical wherever the decision margin exceeds 1e-6 relative)."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl
from oracle import tca_oracle as orc

MARGIN = 1e-6
TOL = {"bf16": 2e-2, "f32": 1e-4}      # max-abs output tolerance per storage type


def params_for(tb, Hq, Hkv, d, b, w, dtype, alpha=0.5, metric="hhi", share=False):
    return tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16 if dtype == "bf16" else tb.TCA_F32, alpha, 0.0,
                          tb.TCA_METRIC_ENTROPY if metric == "entropy" else tb.TCA_METRIC_HHI,
                          tb.TCA_SHARE_GROUP if share else tb.TCA_SHARE_HEAD)


def gpu_select(tb, bufs_mod, prm, x, P, L=None, pos0=0, gb=None):
    """tca_select on the arrays of workload dict x.  Returns (GlobalBuffers, device K, V, Q)."""
    Kd, Vd = bufs_mod.to_device(x["K"]), bufs_mod.to_device(x["V"])
    Qd = bufs_mod.to_device(x["Q"])
    L = x["K"].shape[1] if L is None else L
    n_tokens = L - pos0
    total, rows = tb.tca_select_rows(prm, n_tokens // prm.block, P)
    if gb is None:
        gb = bufs_mod.GlobalBuffers(prm, rows)
    q_last = Qd[:, L - 1, :].contiguous()
    ws = bufs_mod.workspace(tb.tca_select_workspace_bytes(prm, n_tokens))
    tb.tca_select(prm, q_last, Kd, Vd, x["K"].shape[1], pos0, n_tokens, P, gb.offs, gb.n_rows, gb.idx,
                  gb.Kg, gb.Vg, ws)
    torch.cuda.synchronize()
    return gb, Qd, Kd, Vd


def head_indices(gb, h):
    n = int(gb.n_rows[h].item())
    o = int(gb.offs[h])
    return gb.idx[o:o + n].cpu().numpy().astype(np.int64)


def selection_mismatch_is_sub_margin(sel: orc.Selection, got: np.ndarray, b: int, p) -> bool:
    """True if `got` differs from the oracle's set only through decisions whose
    margin is below MARGIN: the gap between the t-th and (t+1)-th logit of a
    block (relative to max(1,|x|)), or the gap in h between blocks on either
    side of a boundary of Psi."""
    m = len(sel.t)
    got_t = np.bincount(got // b, minlength=m)[:m]
    order = np.argsort(sel.h, kind="stable")
    hs = sel.h[order]
    psi = orc.psi_list(b, m, p)
    close_blocks = set()
    for r in range(1, m):
        if psi[r] != psi[r - 1]:
            gap = abs(hs[r] - hs[r - 1]) / max(1.0, abs(hs[r]))
            if gap <= MARGIN:
                # every block tied (within the margin) with the boundary pair may swap groups
                lo = r - 1
                while lo > 0 and abs(hs[lo] - hs[lo - 1]) <= MARGIN * max(1.0, abs(hs[lo])):
                    lo -= 1
                hi = r
                while hi < m - 1 and abs(hs[hi + 1] - hs[hi]) <= MARGIN * max(1.0, abs(hs[hi])):
                    hi += 1
                close_blocks.update(order[lo:hi + 1].tolist())
    for j in range(m):
        gj = got[(got >= j * b) & (got < (j + 1) * b)]
        if got_t[j] != sel.t[j]:
            if j not in close_blocks:
                return False
            t = int(got_t[j])
            if t not in orc.retain_counts(b):
                return False
        else:
            t = int(sel.t[j])
        xb = sel.x[j * b:(j + 1) * b]
        want = j * b + orc.top_t(xb, t)
        if not np.array_equal(np.sort(gj), want):
            srt = np.sort(xb)[::-1]
            if t >= b:
                return False
            gap = (srt[t - 1] - srt[t]) / max(1.0, abs(srt[t - 1]))
            if gap > MARGIN:
                return False
            # the two sets may differ only in elements tied with the threshold
            diff = np.setxor1d(gj, want)
            if np.any(np.abs(sel.x[diff] - srt[t - 1]) > MARGIN * max(1.0, abs(srt[t - 1]))):
                return False
    return True


def assert_selection(sel: orc.Selection, got: np.ndarray, b: int, p, tag=""):
    assert np.all(np.diff(got) > 0), f"{tag}: indices not strictly ascending"
    if np.array_equal(got, sel.S):
        return True
    assert len(got) == len(sel.S), f"{tag}: {len(got)} rows, oracle {len(sel.S)}"
    assert selection_mismatch_is_sub_margin(sel, got, b, p), f"{tag}: index set differs beyond the margin"
    return False


def oracle_rows(x, P, prm_dict, S_list, rows, heads=None):
    """Oracle outputs for the given query rows (positions) of each head, using the index sets S_list
    (one per query head, or one per KV head for a shared selection)."""
    Qf, Kf, Vf = x["Q"], wl.to_f64(x["K"]), wl.to_f64(x["V"])
    Hq, Hkv = Qf.shape[0], Kf.shape[0]
    heads = range(Hq) if heads is None else heads
    per = Hq // len(S_list)
    out = {}
    for h in heads:
        g = orc.kv_head_of(h, Hq, Hkv)
        q = wl.to_f64(Qf[h][rows])
        out[h] = np.stack([orc.attention_row(q[n], int(i), Kf[g], Vf[g], S_list[h // per], prm_dict["w"])
                           for n, i in enumerate(rows)])
    return out
