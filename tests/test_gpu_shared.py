"""GPU parity for group-shared selection under GQA (tca_params.share = TCA_SHARE_GROUP): one index
set per KV head, tokens scored by the mean over the group's query heads of their Eq. 5 scores.
An extension, not in the paper; the oracle's `select_shared` states the rule.  Same bars as the
per-head tests: index sets identical (sub-margin ties excepted), outputs within max-abs 2e-2
(bf16) / 1e-4 (fp32)."""
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


def configs(tb, b, fracs):
    return (np.stack([tb.tca_config_from_budget(b, 1.0, f) for f in fracs]),
            np.stack([orc.config_from_budget(b, 1.0, f) for f in fracs]))


SELECT_CASES = [
    # kind, Hq, Hkv, d, L, dtype, b, w, seed
    ("centroid", 4, 1, 64, 1024, "f32", 32, 128, 1001),          # config 1's shapes
    ("lowrank", 8, 2, 128, 4096 + 77, "bf16", 128, 512, 111),     # several tiles + ragged tail
    ("lowrank", 6, 2, 64, 1000, "bf16", 8, 64, 112),              # G=3, small blocks
    ("centroid", 7, 1, 128, 2048 + 5, "f32", 256, 256, 113),      # G=7, largest block
    ("lowrank", 2, 2, 128, 300, "bf16", 2, 16, 114),              # G=1: the shared path is the per-head path
    ("lowrank", 16, 2, 64, 640, "f32", 64, 128, 115),             # G=8
    ("lowrank", 4, 1, 64, 8192 + 1, "bf16", 2, 16, 116),          # 4096 blocks
    ("lowrank", 128, 16, 64, 512, "bf16", 32, 64, 117),           # 128 query heads
]


@pytest.mark.parametrize("metric", ["hhi", "entropy"])
@pytest.mark.parametrize("case", SELECT_CASES, ids=lambda c: f"{c[0]}-Hq{c[1]}-Hkv{c[2]}-d{c[3]}-L{c[4]}-{c[5]}-b{c[6]}")
def test_shared_select_matches_oracle(mods, case, metric):
    tb, bufs, _ = mods
    kind, Hq, Hkv, d, L, dtype, b, w, seed = case
    print("case", case, metric, flush=True)
    x = wl.prefill_inputs(kind, Hq, Hkv, d, L, dtype, seed)
    P_gpu, P_orc = configs(tb, b, wl.budget_fractions(seed + 1, Hkv))
    prm = H.params_for(tb, Hq, Hkv, d, b, w, dtype, metric=metric, share=True)
    assert tb.tca_selection_heads(prm) == Hkv
    gb, *_ = H.gpu_select(tb, bufs, prm, x, P_gpu)
    assert gb.n_rows.numel() == Hkv and len(gb.offs) == Hkv + 1
    sels = orc.select_all_groups(wl.to_f64(x["Q"][:, L - 1]), wl.to_f64(x["K"]), b, P_orc, 0.5, metric=metric)
    differs = False
    for g in range(Hkv):
        got = H.head_indices(gb, g)
        H.assert_selection(sels[g], got, b, P_orc[g], tag=f"kv head {g}")
        o = int(gb.offs[g])
        assert torch.equal(gb.Kg[o:o + len(got)].cpu(), bufs.to_device(x["K"][g][got], "cpu"))
        assert torch.equal(gb.Vg[o:o + len(got)].cpu(), bufs.to_device(x["V"][g][got], "cpu"))
        one = orc.select(wl.to_f64(x["Q"][g * (Hq // Hkv), L - 1]), wl.to_f64(x["K"][g]), b, P_orc[g], 0.5, metric=metric)
        differs |= not np.array_equal(one.S, sels[g].S)
    if Hq > Hkv and L // b >= 8:
        assert differs, "the shared sets equal the first head's own sets: the group mean is not exercised"


PREFILL_CASES = [
    ("centroid", 4, 1, 64, 1024, "f32", 32, 128, 1001),
    ("lowrank", 8, 2, 128, 1500, "bf16", 128, 256, 131),
    ("lowrank", 6, 2, 64, 700, "bf16", 16, 64, 132),
    ("lowrank", 8, 2, 128, 4096 + 100, "bf16", 128, 1024, 134),    # many key tiles, ragged query tile
    ("lowrank", 128, 16, 64, 300, "bf16", 32, 64, 137),            # 128 query heads, G=8
]


@pytest.mark.parametrize("case", PREFILL_CASES, ids=lambda c: f"{c[0]}-Hq{c[1]}-d{c[3]}-L{c[4]}-{c[5]}-b{c[6]}-w{c[7]}")
def test_shared_prefill_matches_oracle_every_row(mods, case):
    tb, bufs, _ = mods
    kind, Hq, Hkv, d, L, dtype, b, w, seed = case
    print("case", case, flush=True)
    G = Hq // Hkv
    x = wl.prefill_inputs(kind, Hq, Hkv, d, L, dtype, seed)
    P_gpu, P_orc = configs(tb, b, wl.budget_fractions(seed + 1, Hkv))
    prm = H.params_for(tb, Hq, Hkv, d, b, w, dtype, share=True)
    gb, Qd, Kd, Vd = H.gpu_select(tb, bufs, prm, x, P_gpu)
    O = torch.full_like(Qd, float("nan"))
    lse = torch.full((Hq, L), float("nan"), dtype=torch.float32, device="cuda")
    ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, lse, ws)
    torch.cuda.synchronize()
    Qf, Kf, Vf = wl.to_f64(x["Q"]), wl.to_f64(x["K"]), wl.to_f64(x["V"])
    Oref, sels = orc.tca_prefill(Qf, Kf, Vf, b, w, P_orc, 0.5, share=True)
    for g in range(Hkv):
        got = H.head_indices(gb, g)
        if not H.assert_selection(sels[g], got, b, P_orc[g], tag=f"kv head {g}"):
            for h in range(g * G, (g + 1) * G):
                Oref[h] = orc.tca_attention(Qf[h], Kf[g], Vf[g], got, w)
    Og = bufs.to_host_f64(O)
    assert not np.isnan(Og).any(), "some output rows were never written"
    err = np.abs(Og - Oref).max()
    print("max abs err", err, flush=True)
    assert err <= H.TOL[dtype]
    lg = lse.cpu().numpy()
    for h in (0, Hq - 1):
        g = h // G
        for i in (0, w, L - 1):
            T = orc.visible_keys(i, H.head_indices(gb, g), w)
            lref = np.log(np.exp(Kf[g][T] @ Qf[h, i] / np.sqrt(d)).sum())
            assert abs(lg[h, i] - lref) <= (5e-2 if dtype == "bf16" else 1e-3)


DECODE_CASES = [
    # Hq, Hkv, d, L, dtype, b, w, steps, seed
    (4, 1, 64, 1024, "f32", 32, 128, 40, 1001),
    (8, 2, 128, 1500 + 100, "bf16", 128, 256, 140, 151),
    (6, 2, 64, 90, "bf16", 8, 32, 30, 152),          # G=3
    (128, 16, 64, 200, "bf16", 16, 64, 20, 153),     # 128 query heads, G=8
    (10, 2, 128, 400, "f32", 16, 64, 20, 154),       # G=5, fp32, d=128
]


@pytest.mark.parametrize("case", DECODE_CASES, ids=lambda c: f"Hq{c[0]}-Hkv{c[1]}-d{c[2]}-L{c[3]}-{c[4]}-b{c[5]}-w{c[6]}-n{c[7]}")
def test_shared_decode_after_prefill_matches_oracle(mods, case):
    tb, bufs, _ = mods
    Hq, Hkv, d, L, dtype, b, w, steps, seed = case
    print("case", case, flush=True)
    kind = "centroid" if dtype == "f32" else "lowrank"
    x = wl.prefill_inputs(kind, Hq, Hkv, d, L, dtype, seed)
    P_gpu, P_orc = configs(tb, b, wl.budget_fractions(seed + 1, Hkv))
    prm = H.params_for(tb, Hq, Hkv, d, b, w, dtype, share=True)
    _, rows = tb.tca_select_rows(prm, L // b, P_gpu)
    extra = np.array([tb.tca_decode_budget(b, p) for p in P_gpu]) * ((L + steps) // b - L // b + 1)
    cache = bufs.DecodeCache(prm, 1, rows + extra)
    assert cache.n_rows.shape == (1, Hkv)
    Kd, Vd, Qd = bufs.to_device(x["K"]), bufs.to_device(x["V"]), bufs.to_device(x["Q"])
    ws = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
    tb.tca_select(prm, Qd[:, L - 1].contiguous(), Kd, Vd, L, 0, L, P_gpu, cache.offs, cache.n_rows[0],
                  cache.idx[0], cache.Kg[0], cache.Vg[0], ws)
    tb.tca_cache_load_window(prm, cache.view, 0, Kd, Vd, L, L)
    torch.cuda.synchronize()
    Qf, Kf, Vf = wl.to_f64(x["Q"]), wl.to_f64(x["K"]), wl.to_f64(x["V"])
    sels = orc.select_all_groups(Qf[:, L - 1], Kf, b, P_orc, 0.5)
    for g in range(Hkv):
        o, n = int(cache.offs[g]), int(cache.n_rows[0, g].item())
        assert np.array_equal(cache.idx[0, o:o + n].cpu().numpy(), sels[g].S)
    ocache = orc.cache_after_prefill(Kf, Vf, sels)

    dec = wl.decode_inputs(Hq, Hkv, d, steps, dtype, seed + 2, batch=1, gains=x["gains"])
    qd, kd, vd = (bufs.to_device(dec[k]) for k in ("q", "k_new", "v_new"))
    wsd = bufs.workspace(tb.tca_decode_workspace_bytes(prm, 1, cache.max_head_rows))
    O = torch.empty(steps, 1, Hq, d, dtype=qd.dtype, device="cuda")
    for s in range(steps):
        tb.tca_decode(prm, cache.view, cache.offs, qd[s], kd[s], vd[s], P_gpu, O[s], wsd)
    torch.cuda.synchronize()
    Og = bufs.to_host_f64(O)
    worst = 0.0
    for s in range(steps):
        ref = orc.decode_step(ocache, wl.to_f64(dec["q"][s, 0]), wl.to_f64(dec["k_new"][s, 0]),
                              wl.to_f64(dec["v_new"][s, 0]), b, w, P_orc, share=True)
        worst = max(worst, np.abs(Og[s, 0] - ref).max())
    print("max abs err over steps", worst, flush=True)
    assert worst <= H.TOL[dtype]
    assert int(cache.length[0].item()) == L + steps
    for g in range(Hkv):
        o, n = int(cache.offs[g]), int(cache.n_rows[0, g].item())
        assert np.array_equal(cache.idx[0, o:o + n].cpu().numpy(), ocache.S[g]), f"kv head {g}"
        kref = torch.from_numpy(ocache.K[g][ocache.S[g]]).to(cache.Kg.dtype)
        assert torch.equal(cache.Kg[0, o:o + n].cpu(), kref)


def test_shared_decode_from_empty_cache_batched(mods):
    tb, bufs, _ = mods
    Hq, Hkv, d, b, w, steps, B = 8, 2, 64, 8, 16, 50, 3
    P_gpu, P_orc = configs(tb, b, [0.3, 0.7])
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "f32", share=True)
    cap = np.array([tb.tca_decode_budget(b, p) for p in P_gpu]) * (steps // b + 1)
    cache = bufs.DecodeCache(prm, B, cap)
    dec = wl.decode_inputs(Hq, Hkv, d, steps, "f32", 161, batch=B)
    qd, kd, vd = (bufs.to_device(dec[k]) for k in ("q", "k_new", "v_new"))
    wsd = bufs.workspace(tb.tca_decode_workspace_bytes(prm, B, cache.max_head_rows))
    O = torch.empty(steps, B, Hq, d, dtype=torch.float32, device="cuda")
    for s in range(steps):
        tb.tca_decode(prm, cache.view, cache.offs, qd[s], kd[s], vd[s], P_gpu, O[s], wsd)
    torch.cuda.synchronize()
    Og = bufs.to_host_f64(O)
    for sq in range(B):
        oc = orc.HeadCache(S=[np.zeros(0, np.int64) for _ in range(Hkv)])
        for s in range(steps):
            ref = orc.decode_step(oc, dec["q"][s, sq], dec["k_new"][s, sq], dec["v_new"][s, sq], b, w, P_orc, share=True)
            assert np.abs(Og[s, sq] - ref).max() <= 1e-4, (sq, s)
        for g in range(Hkv):
            o, n = int(cache.offs[g]), int(cache.n_rows[sq, g].item())
            assert np.array_equal(cache.idx[sq, o:o + n].cpu().numpy(), oc.S[g])


@pytest.mark.parametrize("case", [("lowrank", 4, 2, 64, 512, "f32", 16, 6, 171),
                                  ("lowrank", 8, 2, 128, 640 + 13, "bf16", 32, 14, 172)],
                         ids=lambda c: f"{c[0]}-Hq{c[1]}-d{c[3]}-L{c[4]}-{c[5]}-b{c[6]}-M{c[7]}")
def test_shared_calibrate_budgets_matches_oracle(mods, case):
    tb, bufs, _ = mods
    kind, Hq, Hkv, d, L, dtype, b, M, seed = case
    x = wl.prefill_inputs(kind, Hq, Hkv, d, L, dtype, seed)
    prm = H.params_for(tb, Hq, Hkv, d, b, b, dtype, share=True)
    Qd, Kd = bufs.to_device(x["Q"]), bufs.to_device(x["K"])
    ws = bufs.workspace(tb.tca_calibrate_workspace_bytes(prm, L, M))
    Qf, Kf = wl.to_f64(x["Q"]), wl.to_f64(x["K"])
    ref0 = orc.calibrate(Qf, Kf, b, M, 1.0, 0.0, 0.5, share=True)
    a_ref = np.stack([c.a for c in ref0])
    n_ref = np.stack([c.n for c in ref0])
    for tau in (0.0, float(np.median(a_ref)), 0.9):
        got = tb.tca_calibrate_budgets(prm, Qd, Kd, L, M, 1.0, tau, ws)
        assert got["a"].shape == (Hkv, M)
        np.testing.assert_allclose(got["a"], a_ref, rtol=1e-9, atol=1e-12)
        assert np.array_equal(got["n"], n_ref)
        ref = orc.calibrate(Qf, Kf, b, M, 1.0, tau, 0.5, share=True)
        for g in range(Hkv):
            if np.min(np.abs(a_ref[g] - tau)) > 1e-9 * max(1.0, abs(tau)):
                assert got["cand_idx"][g] == ref[g].index, (tau, g)
                assert bool(got["fallback"][g]) == ref[g].fallback


def test_shared_chunked_prefill_matches_oracle(mods):
    tb, bufs, sched = mods
    kind, Hq, Hkv, d, L, dtype, b, w, chunk, seed = ("lowrank", 16, 2, 128, 2500, "bf16", 128, 512, 1024, 182)
    x = wl.prefill_inputs(kind, Hq, Hkv, d, L, dtype, seed)
    P_gpu, P_orc = configs(tb, b, wl.budget_fractions(seed + 1, Hkv))
    prm = H.params_for(tb, Hq, Hkv, d, b, w, dtype, share=True)
    rows = sched.chunked_rows(prm, L, chunk, P_gpu)
    gb = bufs.GlobalBuffers(prm, rows)
    Qd, Kd, Vd = (bufs.to_device(x[k]) for k in ("Q", "K", "V"))
    O = torch.full_like(Qd, float("nan"))
    ws = sched.Workspaces(prm, chunk, int(gb.offs[-1]), 1, int(rows.max()))
    for c0, c1 in sched.chunk_bounds(L, chunk):
        sched.prefill_chunk(prm, Qd, Kd, Vd, L, c0, c1, P_gpu, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, O, ws)
    torch.cuda.synchronize()
    Oref, S = orc.tca_prefill_chunked(wl.to_f64(x["Q"]), wl.to_f64(x["K"]), wl.to_f64(x["V"]), b, w, P_orc, 0.5, chunk,
                                      share=True)
    for g in range(Hkv):
        assert np.array_equal(H.head_indices(gb, g), S[g]), f"kv head {g}"
    Og = bufs.to_host_f64(O)
    assert not np.isnan(Og).any()
    assert np.abs(Og - Oref).max() <= H.TOL[dtype]


def test_shared_prefill_full_size_sampled_rows(mods):
    """Config 3 (128K tokens, Hq=32, Hkv=8) with one selection per KV head, as bench.py --shared
    runs it: index sets compared in full, outputs on sampled rows of every query head."""
    tb, bufs, _ = mods
    c = wl.CONFIGS[3]
    Hq, Hkv, d, L, b, w = c["Hq"], c["Hkv"], c["d"], c["L"], c["b"], c["w"]
    G = Hq // Hkv
    x = wl.prefill_inputs(c["kind"], Hq, Hkv, d, L, "bf16", wl.data_seed(3))
    P_gpu, P_orc = configs(tb, b, wl.budget_fractions(wl.budget_seed(3), Hkv))
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16", share=True)
    gb, Qd, Kd, Vd = H.gpu_select(tb, bufs, prm, x, P_gpu)
    O = torch.full_like(Qd, float("nan"))
    ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
    torch.cuda.synchronize()
    print("gpu done", flush=True)
    Kf, Vf = wl.to_f64(x["K"]), wl.to_f64(x["V"])
    sels = orc.select_all_groups(wl.to_f64(x["Q"][:, L - 1]), Kf, b, P_orc, c["alpha"])
    S_used = []
    for g in range(Hkv):
        got = H.head_indices(gb, g)
        H.assert_selection(sels[g], got, b, P_orc[g], tag=f"kv head {g}")
        S_used.append(got)
    rng = np.random.default_rng(199)
    pos = np.unique(np.concatenate([[0, b, w - 1, w, w + 1, L // 2, L - 1], rng.integers(0, L, size=8)])).astype(np.int64)
    Og = O[:, torch.from_numpy(pos).cuda()].double().cpu().numpy()
    worst = 0.0
    for h in range(Hq):
        qh = wl.to_f64(x["Q"][h][pos])
        for n, i in enumerate(pos):
            ref = orc.attention_row(qh[n], int(i), Kf[h // G], Vf[h // G], S_used[h // G], w)
            worst = max(worst, float(np.abs(ref - Og[h, n]).max()))
    print("max abs err on", len(pos) * Hq, "rows:", worst, flush=True)
    assert worst <= H.TOL["bf16"]


def test_shared_decode_full_size_sampled_heads(mods):
    """Config 4 (batch 16 at 128K context) with one selection per KV head: sampled (sequence,
    query head) outputs against the oracle, and the rows appended by a block that completes."""
    tb, bufs, _ = mods
    c = wl.CONFIGS[4]
    Hq, Hkv, d, T0, b, w, B = c["Hq"], c["Hkv"], c["d"], c["L"], c["b"], c["w"], c["batch"]
    G = Hq // Hkv
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16", share=True)
    fr = wl.budget_fractions(wl.budget_seed(4), Hkv)
    P_gpu, P_orc = configs(tb, b, fr)
    n_glob = np.round(fr * (T0 - w)).astype(np.int64)
    t_dec = np.array([tb.tca_decode_budget(b, p) for p in P_gpu])
    cache = bufs.DecodeCache(prm, B, n_glob + 2 * t_dec)
    gen = torch.Generator(device="cuda").manual_seed(wl.data_seed(4) + 1)
    rng = np.random.default_rng(wl.data_seed(4) + 1)
    pend = rng.integers(0, b, size=B)
    pend[3] = b - 1                                    # sequence 3 completes a block at this step
    lengths = T0 + pend
    for s in range(B):
        cache.Kg[s].copy_(torch.randn(cache.Kg[s].shape, generator=gen, device="cuda", dtype=torch.float32))
        cache.Vg[s].copy_(torch.randn(cache.Vg[s].shape, generator=gen, device="cuda", dtype=torch.float32))
        for g in range(Hkv):
            o = int(cache.offs[g])
            pos = np.sort(rng.choice(T0 - w, size=int(n_glob[g]), replace=False)).astype(np.int32)
            cache.idx[s, o:o + len(pos)] = torch.from_numpy(pos).cuda()
    cache.n_rows.copy_(torch.from_numpy(np.tile(n_glob.astype(np.int32), (B, 1))))
    cache.ringK.copy_(torch.randn(cache.ringK.shape, generator=gen, device="cuda", dtype=torch.float32))
    cache.ringV.copy_(torch.randn(cache.ringV.shape, generator=gen, device="cuda", dtype=torch.float32))
    cache.length.copy_(torch.from_numpy(lengths.astype(np.int64)))
    q = torch.randn(B, Hq, d, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    kn = torch.randn(B, Hkv, d, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    vn = torch.randn(B, Hkv, d, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    O = torch.full((B, Hq, d), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = bufs.workspace(tb.tca_decode_workspace_bytes(prm, B, cache.max_head_rows))
    groups = [(0, 0), (3, 1), (3, 7), (9, 4), (15, 7)]           # (sequence, KV head)
    before = {}
    for (s, g) in groups:
        o, n = int(cache.offs[g]), int(n_glob[g])
        before[(s, g)] = dict(idx=cache.idx[s, o:o + n].cpu().numpy().astype(np.int64),
                              Kg=cache.Kg[s, o:o + n].double().cpu().numpy(), Vg=cache.Vg[s, o:o + n].double().cpu().numpy(),
                              ringK=cache.ringK[s, g].double().cpu().numpy(), ringV=cache.ringV[s, g].double().cpu().numpy())
    tb.tca_decode(prm, cache.view, cache.offs, q, kn, vn, P_gpu, O, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(O.float()).any()
    assert cache.length.cpu().tolist() == (lengths + 1).tolist()
    worst = 0.0
    for (s, g) in groups:
        T = int(lengths[s])
        bf = before[(s, g)]
        Kfull = np.zeros((T + 1, d)); Vfull = np.zeros((T + 1, d))
        Kfull[bf["idx"]] = bf["Kg"]; Vfull[bf["idx"]] = bf["Vg"]
        for p in range(T - w + 1, T):
            Kfull[p] = bf["ringK"][p % w]; Vfull[p] = bf["ringV"][p % w]
        Kfull[T] = kn[s, g].double().cpu().numpy(); Vfull[T] = vn[s, g].double().cpu().numpy()
        qg = q[s, g * G:(g + 1) * G].double().cpu().numpy()
        for j in range(G):
            ref = orc.attention_row(qg[j], T, Kfull, Vfull, bf["idx"], w)
            worst = max(worst, float(np.abs(ref - O[s, g * G + j].double().cpu().numpy()).max()))
        o = int(cache.offs[g])
        n_now = int(cache.n_rows[s, g].item())
        if (T + 1) % b == 0:
            blk = T // b
            X = np.stack([orc.last_query_logits(qg[j], Kfull[blk * b:(blk + 1) * b]) for j in range(G)])
            keep = blk * b + orc.top_t(orc.group_scores_from_logits(X), orc.decode_budget(b, P_orc[g]))
            assert n_now == n_glob[g] + len(keep)
            assert np.array_equal(cache.idx[s, o + int(n_glob[g]):o + n_now].cpu().numpy(), keep)
            assert np.array_equal(cache.Kg[s, o + int(n_glob[g]):o + n_now].double().cpu().numpy(), Kfull[keep])
        else:
            assert n_now == n_glob[g]
    print("max abs err on sampled (sequence, head) pairs:", worst, flush=True)
    assert worst <= H.TOL["bf16"]


def test_shared_mixed_batch_and_graph_replay(mods):
    """The ragged mixed batch (chunks interleaved with decode steps) with one selection per KV
    head, each sequence replayed alone by the oracle; then one more decode step of the whole
    batch captured into a HIP graph and replayed against the eager result."""
    tb, bufs, sched = mods
    Hq, Hkv, d, b, w, chunk = 8, 2, 64, 32, 128, 256
    lengths = [300, 1100, 700]
    seed = 191
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16", share=True)
    P_gpu, P_orc = configs(tb, b, wl.budget_fractions(seed, Hkv))
    xs = [wl.prefill_inputs("lowrank", Hq, Hkv, d, L, "bf16", seed + 1 + i) for i, L in enumerate(lengths)]
    mb = sched.MixedBatch(prm, lengths, chunk, P_gpu)
    n_calls = len(mb.events)
    dec = wl.decode_inputs(Hq, Hkv, d, n_calls + 1, "bf16", seed + 9, batch=len(lengths))
    seqs = []
    for x in xs:
        Qd = bufs.to_device(x["Q"])
        seqs.append(dict(Q=Qd, K=bufs.to_device(x["K"]), V=bufs.to_device(x["V"]), O=torch.full_like(Qd, float("nan"))))
    outs = {}
    mb.run(seqs, lambda step, slots: tuple(bufs.to_device(dec[k][step, :len(slots)]) for k in ("q", "k_new", "v_new")),
           lambda step, slots, Od: outs.__setitem__(step, (list(slots), Od.clone())))
    torch.cuda.synchronize()
    assert mb.n_done == len(lengths)
    worst_p, worst_d = 0.0, 0.0
    for i, (x, L) in enumerate(zip(xs, lengths)):
        Qf, Kf, Vf = (wl.to_f64(x[k]) for k in ("Q", "K", "V"))
        Oref, S = orc.tca_prefill_chunked(Qf, Kf, Vf, b, w, P_orc, 0.5, chunk, share=True)
        worst_p = max(worst_p, np.abs(bufs.to_host_f64(seqs[i]["O"]) - Oref).max())
        slot = mb.slot_of[i]
        oc = orc.HeadCache(S=[s_.copy() for s_ in S], K=Kf.copy(), V=Vf.copy())
        for step in sorted(outs):
            slots, Od = outs[step]
            if slot in slots:
                ref = orc.decode_step(oc, wl.to_f64(dec["q"][step, slot]), wl.to_f64(dec["k_new"][step, slot]),
                                      wl.to_f64(dec["v_new"][step, slot]), b, w, P_orc, share=True)
                worst_d = max(worst_d, np.abs(Od[slot].double().cpu().numpy() - ref).max())
        for g in range(Hkv):
            o, n = int(mb.cache.offs[g]), int(mb.cache.n_rows[slot, g].item())
            assert np.array_equal(mb.cache.idx[slot, o:o + n].cpu().numpy(), oc.S[g]), (i, g)
    print("max abs err prefill", worst_p, "decode", worst_d, flush=True)
    assert worst_p <= H.TOL["bf16"] and worst_d <= H.TOL["bf16"]

    # one more step of the full batch: eager on a copy of the cache state, then from a graph
    c = mb.cache
    order = mb.seq_of_slot
    q1, k1, v1 = (bufs.to_device(np.ascontiguousarray(dec[k][n_calls][order])) for k in ("q", "k_new", "v_new"))
    state = [t.clone() for t in (c.idx, c.Kg, c.Vg, c.n_rows, c.ringK, c.ringV, c.length)]
    O_eager = torch.empty_like(q1)
    tb.tca_decode(prm, c.view, c.offs, q1, k1, v1, P_gpu, O_eager, mb.ws.decode)
    torch.cuda.synchronize()
    after = [t.clone() for t in (c.idx, c.n_rows, c.length)]
    for t, s0 in zip((c.idx, c.Kg, c.Vg, c.n_rows, c.ringK, c.ringV, c.length), state):
        t.copy_(s0)
    O_graph = torch.empty_like(q1)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        tb.tca_decode(prm, c.view, c.offs, q1, k1, v1, P_gpu, O_graph, mb.ws.decode)
    for rep in range(3):
        for t, s0 in zip((c.idx, c.Kg, c.Vg, c.n_rows, c.ringK, c.ringV, c.length), state):
            t.copy_(s0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O_graph, O_eager), f"replay {rep}"
        assert all(torch.equal(a, t) for a, t in zip(after, (c.idx, c.n_rows, c.length)))


@pytest.mark.parametrize("share", [False, True], ids=["per_head", "shared"])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128)])
def test_decode_with_rising_and_falling_logits(mods, share, dtype, d):
    """One decode step over a hand-filled cache whose key magnitudes ramp up, then down, along the
    stored rows, so that the split-K kernels raise their softmax reference many times (and then
    stop raising it) inside one slot, in several slots and in the ring."""
    tb, bufs, _ = mods
    Hq, Hkv, b, w, T0 = 8, 2, 16, 256, 6000
    G = Hq // Hkv
    Hs = Hkv if share else Hq
    prm = H.params_for(tb, Hq, Hkv, d, b, w, dtype, share=share)
    P_gpu, _ = configs(tb, b, [0.5] * Hs)
    rng = np.random.default_rng(211)
    n_glob = rng.integers(1500, 3500, size=Hs)
    cache = bufs.DecodeCache(prm, 1, n_glob + 64)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    T = T0 + 3                                              # no block completes at this step
    idx_h, Kg_h, Vg_h = [], [], []
    for n_ in range(Hs):
        n = int(n_glob[n_])
        pos = np.sort(rng.choice(T0 - w, size=n, replace=False)).astype(np.int32)
        ramp = np.concatenate([np.linspace(0.05, 4.0, n // 2), np.linspace(4.0, 0.05, n - n // 2)])[:, None]
        Kg = torch.from_numpy(rng.standard_normal((n, d)) * ramp).to(dt)
        Vg = torch.from_numpy(rng.standard_normal((n, d))).to(dt)
        o = int(cache.offs[n_])
        cache.idx[0, o:o + n] = torch.from_numpy(pos).cuda()
        cache.Kg[0, o:o + n] = Kg.cuda()
        cache.Vg[0, o:o + n] = Vg.cuda()
        idx_h.append(pos.astype(np.int64)); Kg_h.append(Kg.double().numpy()); Vg_h.append(Vg.double().numpy())
    cache.n_rows.copy_(torch.from_numpy(n_glob.astype(np.int32))[None])
    ramp_w = np.linspace(0.05, 3.0, w)[None, :, None]
    ringK = torch.from_numpy(rng.standard_normal((Hkv, w, d)) * ramp_w).to(dt)
    ringV = torch.from_numpy(rng.standard_normal((Hkv, w, d))).to(dt)
    cache.ringK[0] = ringK.cuda(); cache.ringV[0] = ringV.cuda()
    cache.length.fill_(T)
    q = torch.from_numpy(2.0 * rng.standard_normal((1, Hq, d))).to(dt).cuda()
    kn = torch.from_numpy(rng.standard_normal((1, Hkv, d))).to(dt).cuda()
    vn = torch.from_numpy(rng.standard_normal((1, Hkv, d))).to(dt).cuda()
    O = torch.full((1, Hq, d), float("nan"), dtype=dt, device="cuda")
    ws = bufs.workspace(tb.tca_decode_workspace_bytes(prm, 1, cache.max_head_rows))
    tb.tca_decode(prm, cache.view, cache.offs, q, kn, vn, P_gpu, O, ws)
    torch.cuda.synchronize()
    worst = 0.0
    for h in range(Hq):
        g, n_ = h // G, (h // G if share else h)
        Kfull = np.zeros((T + 1, d)); Vfull = np.zeros((T + 1, d))
        Kfull[idx_h[n_]] = Kg_h[n_]; Vfull[idx_h[n_]] = Vg_h[n_]
        for p in range(T - w + 1, T):
            Kfull[p] = ringK[g, p % w].double().numpy(); Vfull[p] = ringV[g, p % w].double().numpy()
        Kfull[T] = kn[0, g].double().cpu().numpy(); Vfull[T] = vn[0, g].double().cpu().numpy()
        ref = orc.attention_row(q[0, h].double().cpu().numpy(), T, Kfull, Vfull, idx_h[n_], w)
        worst = max(worst, float(np.abs(ref - O[0, h].double().cpu().numpy()).max()))
    print("max abs err", worst, flush=True)
    assert worst <= H.TOL[dtype]
