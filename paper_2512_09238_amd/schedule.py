"""Host-side scheduling of chunked prefill and of a ragged mixed batch (prefill
chunks interleaved with decode steps).  Plumbing only: every step of the method
runs in libtca kernels through the C ABI; this module decides what to call when
and owns the device buffers (torch).

Chunked prefill is a serving extension, not part of the paper's method: the
chunk covering [c0, c1) is scored by its own last query over its own keys
(`tca_select` with pos0 = c0), its kept rows are appended to the head's global
region, and its queries attend to the region as it stands plus their window
(`tca_prefill` with q_pos0 = c0).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as tb
from . import buffers as bufs


def chunk_bounds(L: int, chunk: int):
    return [(c0, min(L, c0 + chunk)) for c0 in range(0, L, chunk)]


def chunked_rows(prm, L: int, chunk: int, P) -> np.ndarray:
    """Rows each head's global region receives from a chunked prefill of L tokens."""
    rows = np.zeros(tb.tca_selection_heads(prm), np.int64)
    for c0, c1 in chunk_bounds(L, chunk):
        rows += tb.tca_select_rows(prm, (c1 - c0) // prm.block, P)[1]
    return rows


class Workspaces:
    """Scratch buffers sized for chunks of at most `chunk` tokens and decode batches of `batch`."""

    def __init__(self, prm, chunk: int, cap_rows: int, batch: int, max_head_rows: int, device="cuda:0"):
        self.select = bufs.workspace(tb.tca_select_workspace_bytes(prm, chunk), device)
        self.prefill = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, chunk, cap_rows), device)
        self.decode = bufs.workspace(tb.tca_decode_workspace_bytes(prm, batch, max_head_rows), device)


def prefill_chunk(prm, Q, K, V, L_alloc: int, c0: int, c1: int, P, offs, n_rows, idx, Kg, Vg, O, ws: Workspaces):
    """One chunk: selection over [c0, c1) then attention for the queries of [c0, c1).
    Q, O: [Hq, L_alloc, d] tensors of the whole sequence; K, V: [Hkv, L_alloc, d]."""
    n = c1 - c0
    q_last = Q[:, c1 - 1].contiguous()
    tb.tca_select(prm, q_last, K, V, L_alloc, c0, n, P, offs, n_rows, idx, Kg, Vg, ws.select)
    Qc = Q[:, c0:c1].contiguous()
    Oc = torch.empty_like(Qc)
    tb.tca_prefill(prm, Qc, c0, n, K, V, L_alloc, idx, Kg, Vg, offs, n_rows, Oc, None, ws.prefill)
    O[:, c0:c1] = Oc


class MixedBatch:
    """Ragged batch: sequences are prefilled chunk by chunk, round-robin over the
    unfinished ones; after every chunk, one decode step runs for all sequences
    that have finished prefill.  Cache slots are assigned in the order in which
    sequences will finish, so the decoding set is always slots [0, n_done)."""

    def __init__(self, prm, lengths, chunk: int, P, device="cuda:0"):
        self.prm, self.chunk, self.P = prm, chunk, np.ascontiguousarray(P, np.float64)
        self.lengths = [int(x) for x in lengths]
        B = len(self.lengths)
        # simulate the round-robin schedule on the host to learn the completion order
        left = [len(chunk_bounds(L, chunk)) for L in self.lengths]
        order, events, turn = [], [], 0
        pending = [i for i in range(B)]
        while pending:
            i = pending[turn % len(pending)]
            k = len(chunk_bounds(self.lengths[i], chunk)) - left[i]
            events.append((i, k))
            left[i] -= 1
            if left[i] == 0:
                order.append(i)
                pending.remove(i)
            else:
                turn += 1
        self.events = events                    # (sequence, chunk index) in execution order
        self.slot_of = {seq: s for s, seq in enumerate(order)}
        self.seq_of_slot = order
        t_dec = np.array([tb.tca_decode_budget(prm.block, p) for p in self.P])
        cap = np.zeros(tb.tca_selection_heads(prm), np.int64)
        # at most one decode step per chunk event, each can complete at most one block per sequence
        extra = t_dec * (len(events) // prm.block + 2)
        for L in self.lengths:
            cap = np.maximum(cap, chunked_rows(prm, L, chunk, self.P) + extra)
        self.cache = bufs.DecodeCache(prm, B, cap, device)
        self.ws = Workspaces(prm, chunk, self.cache.cap_rows, B, self.cache.max_head_rows, device)
        self.n_done = 0
        self.decode_calls = 0

    def cache_slices(self, seq):
        s = self.slot_of[seq]
        c = self.cache
        return c.n_rows[s], c.idx[s], c.Kg[s], c.Vg[s]

    def run(self, seqs, decode_inputs=None, on_decode=None):
        """seqs[i] = dict(Q, K, V, O) device tensors of sequence i.  decode_inputs(step, slots) ->
        (q, k_new, v_new) for the sequences in cache slots [0, len(slots)); on_decode(step, slots, O)."""
        prm = self.prm
        for (i, k) in self.events:
            L = self.lengths[i]
            c0, c1 = chunk_bounds(L, self.chunk)[k]
            sq = seqs[i]
            n_rows, idx, Kg, Vg = self.cache_slices(i)
            prefill_chunk(prm, sq["Q"], sq["K"], sq["V"], sq["K"].shape[1], c0, c1, self.P, self.cache.offs,
                          n_rows, idx, Kg, Vg, sq["O"], self.ws)
            if c1 == L:                           # prefill finished: hand the window over to the decode cache
                tb.tca_cache_load_window(prm, self.cache.view, self.slot_of[i], sq["K"], sq["V"], sq["K"].shape[1], L)
                self.n_done += 1
            if self.n_done and decode_inputs is not None:
                slots = list(range(self.n_done))
                q, kn, vn = decode_inputs(self.decode_calls, slots)
                Od = torch.empty_like(q)
                view = tb.make_cache(self.n_done, self.cache.cap_rows, self.cache.idx, self.cache.Kg, self.cache.Vg,
                                     self.cache.n_rows, self.cache.ringK, self.cache.ringV, self.cache.length)
                tb.tca_decode(prm, view, self.cache.offs, q, kn, vn, self.P, Od, self.ws.decode)
                if on_decode is not None:
                    on_decode(self.decode_calls, slots, Od)
                self.decode_calls += 1
