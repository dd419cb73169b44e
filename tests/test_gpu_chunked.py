"""GPU parity for chunked prefill and the ragged mixed batch (prefill chunks
interleaved with decode steps).  Chunked prefill is a serving extension that
the paper does not describe; the oracle's `tca_prefill_chunked` states the rule."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import tca_oracle as orc
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    import paper_2512_09238_amd.binding as tb
    import paper_2512_09238_amd.buffers as bufs
    import paper_2512_09238_amd.schedule as sched
    return tb, bufs, sched


CASES = [
    # kind, Hq, Hkv, d, L, dtype, b, w, chunk, seed
    ("lowrank", 4, 2, 64, 700, "f32", 32, 64, 256, 81),
    ("lowrank", 16, 2, 128, 2500, "bf16", 128, 512, 1024, 82),     # G = 8, ragged last chunk
    ("centroid", 2, 1, 128, 1024, "bf16", 64, 128, 2048, 83),      # one chunk covers the sequence
]


def _draw_chunked(rng):
    G, Hkv = int(rng.integers(1, 9)), int(rng.integers(1, 3))
    d = int(rng.choice([64, 128]))
    b = int(2 ** rng.integers(2, 8))
    w = b * int(rng.integers(1, 5))
    chunk = b * int(rng.integers(1, 9))                 # chunks are whole blocks; the last one may be ragged
    L = int(rng.integers(chunk + 1, min(5 * chunk + 40, 1300) + chunk))
    return (str(rng.choice(["lowrank", "centroid"])), G * Hkv, Hkv, d, L, str(rng.choice(["bf16", "f32"])), b, w,
            chunk, int(rng.integers(1000, 9999)))


CASES = CASES + [_draw_chunked(np.random.default_rng(700 + i)) for i in range(16)]


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"{c[0]}-Hq{c[1]}-d{c[3]}-L{c[4]}-{c[5]}-b{c[6]}-w{c[7]}-chunk{c[8]}")
def test_chunked_prefill_matches_oracle(mods, case):
    tb, bufs, sched = mods
    kind, Hq, Hkv, d, L, dtype, b, w, chunk, seed = case
    print("case", case, flush=True)
    x = wl.prefill_inputs(kind, Hq, Hkv, d, L, dtype, seed)
    fr = wl.budget_fractions(seed + 1, Hq)
    P_gpu = np.stack([tb.tca_config_from_budget(b, 1.0, f) for f in fr])
    P_orc = np.stack([orc.config_from_budget(b, 1.0, f) for f in fr])
    prm = H.params_for(tb, Hq, Hkv, d, b, w, dtype)
    rows = sched.chunked_rows(prm, L, chunk, P_gpu)
    gb = bufs.GlobalBuffers(prm, rows)
    Qd, Kd, Vd = (bufs.to_device(x[k]) for k in ("Q", "K", "V"))
    O = torch.full_like(Qd, float("nan"))
    ws = sched.Workspaces(prm, chunk, int(gb.offs[-1]), 1, int(rows.max()))
    for c0, c1 in sched.chunk_bounds(L, chunk):
        sched.prefill_chunk(prm, Qd, Kd, Vd, L, c0, c1, P_gpu, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, O, ws)
    torch.cuda.synchronize()
    Oref, S = orc.tca_prefill_chunked(wl.to_f64(x["Q"]), wl.to_f64(x["K"]), wl.to_f64(x["V"]), b, w, P_orc, 0.5, chunk)
    for h in range(Hq):
        assert np.array_equal(H.head_indices(gb, h), S[h]), f"head {h}"
    Og = bufs.to_host_f64(O)
    assert not np.isnan(Og).any()
    err = np.abs(Og - Oref).max()
    print("max abs err", err, flush=True)
    assert err <= H.TOL[dtype]
    if chunk >= L:      # one chunk = Alg. 2
        O1, _ = orc.tca_prefill(wl.to_f64(x["Q"]), wl.to_f64(x["K"]), wl.to_f64(x["V"]), b, w, P_orc, 0.5)
        assert np.abs(Og - O1).max() <= H.TOL[dtype]


def test_mixed_batch_prefill_chunks_interleaved_with_decode(mods):
    """Three ragged sequences: round-robin chunks, a decode step for the finished
    ones after every chunk.  Each sequence is independent, so the oracle replays
    it alone: chunked prefill, then its decode steps in order."""
    tb, bufs, sched = mods
    Hq, Hkv, d, b, w, chunk = 8, 2, 64, 32, 128, 256
    lengths = [300, 1100, 700]
    seed = 91
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    fr = wl.budget_fractions(seed, Hq)
    P_gpu = np.stack([tb.tca_config_from_budget(b, 1.0, f) for f in fr])
    P_orc = np.stack([orc.config_from_budget(b, 1.0, f) for f in fr])
    xs = [wl.prefill_inputs("lowrank", Hq, Hkv, d, L, "bf16", seed + 1 + i) for i, L in enumerate(lengths)]
    mb = sched.MixedBatch(prm, lengths, chunk, P_gpu)
    n_calls = len(mb.events)
    dec = wl.decode_inputs(Hq, Hkv, d, n_calls, "bf16", seed + 9, batch=len(lengths))
    seqs = []
    for x in xs:
        Qd = bufs.to_device(x["Q"])
        seqs.append(dict(Q=Qd, K=bufs.to_device(x["K"]), V=bufs.to_device(x["V"]), O=torch.full_like(Qd, float("nan"))))
    outs = {}

    def decode_inputs(step, slots):
        n = len(slots)
        return tuple(bufs.to_device(dec[k][step, :n]) for k in ("q", "k_new", "v_new"))

    def on_decode(step, slots, Od):
        outs[step] = (list(slots), Od.clone())

    mb.run(seqs, decode_inputs, on_decode)
    torch.cuda.synchronize()
    assert mb.n_done == len(lengths) and len(outs) >= 2
    worst_p, worst_d = 0.0, 0.0
    for i, (x, L) in enumerate(zip(xs, lengths)):
        Qf, Kf, Vf = (wl.to_f64(x[k]) for k in ("Q", "K", "V"))
        Oref, S = orc.tca_prefill_chunked(Qf, Kf, Vf, b, w, P_orc, 0.5, chunk)
        worst_p = max(worst_p, np.abs(bufs.to_host_f64(seqs[i]["O"]) - Oref).max())
        slot = mb.slot_of[i]
        oc = orc.HeadCache(S=[s.copy() for s in S], K=Kf.copy(), V=Vf.copy())
        for step in sorted(outs):
            slots, Od = outs[step]
            if slot not in slots:
                continue
            ref = orc.decode_step(oc, wl.to_f64(dec["q"][step, slot]), wl.to_f64(dec["k_new"][step, slot]),
                                  wl.to_f64(dec["v_new"][step, slot]), b, w, P_orc)
            worst_d = max(worst_d, np.abs(Od[slot].double().cpu().numpy() - ref).max())
        for h in range(Hq):
            o, n = int(mb.cache.offs[h]), int(mb.cache.n_rows[slot, h].item())
            assert np.array_equal(mb.cache.idx[slot, o:o + n].cpu().numpy(), oc.S[h]), (i, h)
        assert int(mb.cache.length[slot].item()) == oc.length
    print("max abs err prefill", worst_p, "decode", worst_d, flush=True)
    assert worst_p <= H.TOL["bf16"] and worst_d <= H.TOL["bf16"]
