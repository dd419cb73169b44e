"""GPU parity at the full workload sizes, in the launch configuration bench.py
times: index sets compared in full (selection is O(L d) for the oracle),
attention outputs on sampled rows the oracle computes one by one."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import tca_oracle as orc
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    import paper_2512_09238_amd.binding as tb
    return tb


@pytest.fixture(scope="module")
def bufs():
    import paper_2512_09238_amd.buffers as bufs
    return bufs


def _sample_positions(L, w, b, n, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, b - 1, b, w - 1, w, w + 1, L // 2, L - b, L - 2, L - 1]
    return np.unique(np.concatenate([fixed, rng.integers(0, L, size=n)])).astype(np.int64)


# d = 64 with enough query tiles for the 8-wave workgroups of the MFMA kernel, ragged last tile
WIDE_D64 = dict(kind="lowrank", Hq=32, Hkv=8, d=64, L=8192 + 77, b=64, w=512, alpha=0.5, sigma=1.0)


@pytest.mark.parametrize("cfg_id", [2, 3, "d64"])
def test_prefill_full_size_sampled_rows(tb, bufs, cfg_id):
    c = WIDE_D64 if cfg_id == "d64" else wl.CONFIGS[cfg_id]
    Hq, Hkv, d, L, b, w = c["Hq"], c["Hkv"], c["d"], c["L"], c["b"], c["w"]
    print("config", cfg_id, "L", L, flush=True)
    seed_id = 6 if cfg_id == "d64" else cfg_id
    x = wl.prefill_inputs(c["kind"], Hq, Hkv, d, L, "bf16", wl.data_seed(seed_id))
    fr = wl.budget_fractions(wl.budget_seed(seed_id), Hq)
    P_gpu = np.stack([tb.tca_config_from_budget(b, c["sigma"], f) for f in fr])
    P_orc = np.stack([orc.config_from_budget(b, c["sigma"], f) for f in fr])
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    gb, Qd, Kd, Vd = H.gpu_select(tb, bufs, prm, x, P_gpu)
    O = torch.full_like(Qd, float("nan"))
    ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(O).any(), "a (head, query tile) of the output was never written"
    print("gpu done", flush=True)

    Kf, Vf = wl.to_f64(x["K"]), wl.to_f64(x["V"])
    sels = orc.select_all_heads(wl.to_f64(x["Q"][:, L - 1]), Kf, b, P_orc, c["alpha"])
    S_used = []
    for h in range(Hq):
        got = H.head_indices(gb, h)
        H.assert_selection(sels[h], got, b, P_orc[h], tag=f"cfg{cfg_id} head {h}")
        S_used.append(got)
        # the compacted rows are byte copies
        if h % 7 == 0:
            o = int(gb.offs[h])
            pick = np.linspace(0, len(got) - 1, 64).astype(np.int64)
            kg = gb.Kg[o + torch.from_numpy(pick).cuda()].cpu()
            assert torch.equal(kg, bufs.to_device(x["K"][h // (Hq // Hkv)][got[pick]], "cpu"))
    pos = _sample_positions(L, w, b, 12, 99)
    if cfg_id == "d64":
        pos = np.unique(np.concatenate([pos, np.arange(L - 80, L)]))   # the ragged last query tile in full
    Og = O[:, torch.from_numpy(pos).cuda()].double().cpu().numpy()
    worst = 0.0
    for h in range(Hq):
        g = h // (Hq // Hkv)
        qh = wl.to_f64(x["Q"][h][pos])
        for n, i in enumerate(pos):
            ref = orc.attention_row(qh[n], int(i), Kf[g], Vf[g], S_used[h], w)
            worst = max(worst, float(np.abs(ref - Og[h, n]).max()))
    print("max abs err on", len(pos) * Hq, "rows:", worst, flush=True)
    assert worst <= H.TOL["bf16"]


def test_calibration_full_length_two_heads(tb, bufs):
    """Alg. 1 at the calibration length of config 3 (8192 tokens), on a two-head
    slice (the oracle's dense L x L pass is what bounds the slice)."""
    c = wl.CONFIGS[3]
    Lc, b, M, d = c["L_cal"], c["b"], c["M"], c["d"]
    x = wl.prefill_inputs(c["kind"], 2, 1, d, Lc, "bf16", wl.calib_seed(3))
    prm = H.params_for(tb, 2, 1, d, b, c["w"], "bf16")
    Qd, Kd = bufs.to_device(x["Q"]), bufs.to_device(x["K"])
    ws = bufs.workspace(tb.tca_calibrate_workspace_bytes(prm, Lc, M))
    got = tb.tca_calibrate_budgets(prm, Qd, Kd, Lc, M, c["sigma"], c["tau"], ws)
    ref = orc.calibrate(wl.to_f64(x["Q"]), wl.to_f64(x["K"]), b, M, c["sigma"], c["tau"], c["alpha"])
    for h in range(2):
        np.testing.assert_allclose(got["a"][h], ref[h].a, rtol=1e-9)
        assert np.array_equal(got["n"][h], ref[h].n)
        if np.min(np.abs(ref[h].a - c["tau"])) > 1e-9:
            assert got["cand_idx"][h] == ref[h].index and bool(got["fallback"][h]) == ref[h].fallback


def _decode_full_size(tb, bufs, fp8):
    """Config 4: batch 16 at 128K context, all 64 steps queued back to back.  Cache contents are
    drawn on the device with a seeded torch generator (fp8: codes and scales drawn directly, as
    bench.py does); for sampled (sequence, head) pairs the host keeps what the query can see
    (global rows, window, appended rows) and replays the steps with the oracle's routines: outputs
    at the first step, at every step that completes a block of the pair's sequence, at the step
    after it and at the last step; the global subsets (positions and rows as stored) after the 64
    steps bit for bit, which covers every block completed on the way."""
    c = wl.CONFIGS[4]
    Hq, Hkv, d, T0, b, w, B, steps = c["Hq"], c["Hkv"], c["d"], c["L"], c["b"], c["w"], c["batch"], c["steps"]
    G = Hq // Hkv
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    fr = wl.budget_fractions(wl.budget_seed(4), Hq)
    P_gpu = np.stack([tb.tca_config_from_budget(b, c["sigma"], f) for f in fr])
    P_orc = np.stack([orc.config_from_budget(b, c["sigma"], f) for f in fr])
    n_glob = np.round(fr * (T0 - w)).astype(np.int64)
    t_dec = np.array([tb.tca_decode_budget(b, p) for p in P_gpu])
    cache = bufs.DecodeCache(prm, B, n_glob + 2 * t_dec, kv_format=tb.TCA_KV_FP8 if fp8 else tb.TCA_KV_NATIVE)
    g = torch.Generator(device="cuda").manual_seed(wl.data_seed(4))
    rng = np.random.default_rng(wl.data_seed(4))
    pend = rng.integers(0, b, size=B)
    pend[3] = b - 1                                    # sequence 3 completes a block at step 0
    pend[7] = b - 1 - 20                               # sequence 7 at step 20
    pend[9] = b - steps                                # sequence 9 at the last step
    lengths = T0 + pend
    done_at = {s: int(b - 1 - pend[s]) for s in range(B) if b - 1 - pend[s] < steps}
    print("blocks complete at steps", done_at, flush=True)

    def fill(rows, scales):
        if not fp8:
            rows.copy_(torch.randn(rows.shape, generator=g, device="cuda", dtype=torch.float32))
            return
        codes = torch.randint(0, 256, rows.shape, generator=g, device="cuda", dtype=torch.uint8)
        codes[(codes & 0x7F) == 0x7F] = 0              # the two NaN codes
        rows.copy_(codes)
        scales.copy_(torch.rand(scales.shape, generator=g, device="cuda") * 0.015 + 0.005)

    def stored(name, *ix):
        """What the cache holds at an index, as the oracle's routines read it: float64 rows."""
        t = getattr(cache, name)[ix]
        if not fp8:
            return t.double().cpu().numpy()
        return orc.dequantize_rows_fp8(t.cpu().numpy(), getattr(cache, name + "_scale")[ix].cpu().numpy())

    for s in range(B):
        fill(cache.Kg[s], cache.Kg_scale[s] if fp8 else None)
        fill(cache.Vg[s], cache.Vg_scale[s] if fp8 else None)
        for h in range(Hq):
            o = int(cache.offs[h])
            pos = np.sort(rng.choice(T0 - w, size=int(n_glob[h]), replace=False)).astype(np.int32)
            cache.idx[s, o:o + len(pos)] = torch.from_numpy(pos).cuda()
    cache.n_rows.copy_(torch.from_numpy(np.tile(n_glob.astype(np.int32), (B, 1))))
    fill(cache.ringK, cache.ringK_scale)
    fill(cache.ringV, cache.ringV_scale)
    cache.length.copy_(torch.from_numpy(lengths.astype(np.int64)))
    q = torch.randn(steps, B, Hq, d, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    kn = torch.randn(steps, B, Hkv, d, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    vn = torch.randn(steps, B, Hkv, d, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    O = torch.full((steps, B, Hq, d), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = bufs.workspace(tb.tca_decode_workspace_bytes(prm, B, cache.max_head_rows))
    # host copies of what the sampled pairs need, taken before the first step
    pairs = [(0, 0), (3, 5), (3, 31), (7, 13), (7, 28), (9, 18), (15, 31)]
    before = {}
    for (s, h) in pairs:
        o, n = int(cache.offs[h]), int(n_glob[h])
        kvh = h // G
        before[(s, h)] = dict(idx=cache.idx[s, o:o + n].cpu().numpy().astype(np.int64),
                              Kg=stored("Kg", s, slice(o, o + n)), Vg=stored("Vg", s, slice(o, o + n)),
                              ringK=stored("ringK", s, kvh), ringV=stored("ringV", s, kvh))
    for st in range(steps):                            # no host sync between the steps
        tb.tca_decode(prm, cache.view, cache.offs, q[st], kn[st], vn[st], P_gpu, O[st], ws)
    torch.cuda.synchronize()
    print("gpu done", flush=True)
    assert not torch.isnan(O.float()).any()
    assert cache.length.cpu().tolist() == (lengths + steps).tolist()
    qh, knh, vnh, Oh = q.double().cpu().numpy(), kn.double().cpu().numpy(), vn.double().cpu().numpy(), O.double().cpu().numpy()
    if fp8:                                            # a new row enters the cache as codes and a scale
        knh, vnh = orc.roundtrip_rows_fp8(knh), orc.roundtrip_rows_fp8(vnh)
    worst, n_checked, n_completed = 0.0, 0, 0
    for (s, h) in pairs:
        kvh = h // G
        T_first = int(lengths[s])
        bf = before[(s, h)]
        # dense arrays holding only what the queries can see: global rows, the window, the new rows
        Kfull = np.zeros((T_first + steps, d)); Vfull = np.zeros((T_first + steps, d))
        Kfull[bf["idx"]] = bf["Kg"]; Vfull[bf["idx"]] = bf["Vg"]
        for p in range(T_first - w + 1, T_first):
            Kfull[p] = bf["ringK"][p % w]; Vfull[p] = bf["ringV"][p % w]
        S = bf["idx"].copy()
        check = {0, steps - 1}
        if s in done_at:
            check |= {done_at[s], min(done_at[s] + 1, steps - 1)}
        for st in range(steps):
            T = T_first + st
            Kfull[T] = knh[st, s, kvh]; Vfull[T] = vnh[st, s, kvh]
            if st in check:
                ref = orc.attention_row(qh[st, s, h], T, Kfull[:T + 1], Vfull[:T + 1], S, w)
                worst = max(worst, float(np.abs(ref - Oh[st, s, h]).max()))
                n_checked += 1
            if (T + 1) % b == 0:                       # the block completed by this token (Sec. IV-B, decoding stage)
                blk = T // b
                x = orc.last_query_logits(qh[st, s, h], Kfull[blk * b:(blk + 1) * b])
                S = np.concatenate([S, blk * b + orc.top_t(x, orc.decode_budget(b, P_orc[h]))])
                n_completed += 1
        o, n_now = int(cache.offs[h]), int(cache.n_rows[s, h].item())
        assert n_now == len(S), (s, h)
        assert np.array_equal(cache.idx[s, o:o + n_now].cpu().numpy(), S), (s, h)
        new_rows = S[len(bf["idx"]):]
        new_at = slice(o + len(bf["idx"]), o + n_now)
        assert np.array_equal(stored("Kg", s, new_at), Kfull[new_rows]), (s, h)
        assert np.array_equal(stored("Vg", s, new_at), Vfull[new_rows]), (s, h)
        if fp8 and len(new_rows):
            # kept rows are copied as stored: the codes and scales of the ring's rows, not a second quantisation
            slots = new_rows % w
            for name, ring in (("Kg", "ringK"), ("Vg", "ringV")):
                assert torch.equal(getattr(cache, name)[s, new_at], getattr(cache, ring)[s, kvh][slots]), (name, s, h)
                assert torch.equal(getattr(cache, name + "_scale")[s, new_at], getattr(cache, ring + "_scale")[s, kvh][slots]), (name, s, h)
    assert n_completed >= 5
    print("max abs err on", n_checked, "sampled (step, sequence, head) outputs:", worst, "; blocks completed:", n_completed, flush=True)
    assert worst <= H.TOL["bf16"]


def test_decode_full_size_all_steps_sampled_heads(tb, bufs):
    _decode_full_size(tb, bufs, fp8=False)


def test_decode_full_size_fp8_cache_all_steps_sampled_heads(tb, bufs):
    """The same with the FP8 cache (TCA_KV_FP8), the workload of bench.py's decode_fp8_cache line."""
    _decode_full_size(tb, bufs, fp8=True)


def test_config5_ragged_mixed_batch_sampled(tb, bufs):
    """Config 5: 70B-shaped layer (Hq=64, Hkv=8), 8 sequences with log-uniform
    lengths, 8192-token chunks interleaved with decode steps, budgets from
    calibration.  Inputs are drawn on the device; sampled (sequence, head) pairs
    are copied to the host and replayed by the oracle alone."""
    import paper_2512_09238_amd.schedule as sched
    c = wl.CONFIGS[5]
    Hq, Hkv, d, b, w, chunk = c["Hq"], c["Hkv"], c["d"], c["b"], c["w"], c["chunk"]
    G = Hq // Hkv
    lengths = wl.config5_lengths()
    print("lengths", lengths, flush=True)
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    # budgets: calibration on a separate 8192-token sample
    xc = wl.device_lowrank_inputs(Hq, Hkv, d, c["L_cal"], wl.calib_seed(5))
    wsc = bufs.workspace(tb.tca_calibrate_workspace_bytes(prm, c["L_cal"], c["M"]))
    cal = tb.tca_calibrate_budgets(prm, xc["Q"], xc["K"], c["L_cal"], c["M"], c["sigma"], c["tau"], wsc)
    P_gpu = cal["p_star"]
    # the oracle calibrates the heads it is going to replay by itself (Alg. 1 on the same sample)
    sample_heads = [0, 17, 40, Hq - 1]
    P_orc = {}
    for h in sample_heads:
        kv = h // G
        ch = orc.calibrate_head(xc["Q"][h].double().cpu().numpy(), xc["K"][kv].double().cpu().numpy(), b,
                                orc.candidates(b, c["M"], c["sigma"]), c["tau"], c["alpha"])
        assert ch.index == cal["cand_idx"][h], f"calibration of head {h}"
        np.testing.assert_allclose(P_gpu[h], ch.p, rtol=1e-12, atol=1e-15)
        P_orc[h] = ch.p
    del xc, wsc
    seqs = []
    for i, L in enumerate(lengths):
        x = wl.device_lowrank_inputs(Hq, Hkv, d, L, wl.data_seed(5) + 10 * i)
        seqs.append(dict(Q=x["Q"], K=x["K"], V=x["V"], O=torch.full_like(x["Q"], float("nan"))))
    mb = sched.MixedBatch(prm, lengths, chunk, P_gpu)
    n_calls = len(mb.events)
    g = torch.Generator(device="cuda").manual_seed(77)
    dq = torch.randn(n_calls, len(lengths), Hq, d, generator=g, device="cuda").to(torch.bfloat16)
    dk = torch.randn(n_calls, len(lengths), Hkv, d, generator=g, device="cuda").to(torch.bfloat16)
    dv = torch.randn(n_calls, len(lengths), Hkv, d, generator=g, device="cuda").to(torch.bfloat16)
    outs = {}
    mb.run(seqs, lambda step, slots: (dq[step, :len(slots)].contiguous(), dk[step, :len(slots)].contiguous(),
                                      dv[step, :len(slots)].contiguous()),
           lambda step, slots, Od: outs.__setitem__(step, (len(slots), Od.clone())))
    torch.cuda.synchronize()
    print("gpu done:", n_calls, "chunk events,", mb.decode_calls, "decode steps", flush=True)
    longest = int(np.argmax(lengths))
    pairs = [(longest, 0), (longest, Hq - 1), (int(np.argmin(lengths)), 17), (2, 40)]   # heads in sample_heads
    worst_p = worst_d = 0.0
    for (i, h) in pairs:
        L, kv = lengths[i], h // G
        Kf = seqs[i]["K"][kv].double().cpu().numpy()[None]
        Vf = seqs[i]["V"][kv].double().cpu().numpy()[None]
        p1 = P_orc[h][None]
        # selection replay: every chunk scored by its own last query
        S = np.zeros(0, np.int64)
        for c0, c1 in sched.chunk_bounds(L, chunk):
            ql = seqs[i]["Q"][h, c1 - 1].double().cpu().numpy()
            S = np.concatenate([S, c0 + orc.select(ql, Kf[0, c0:c1], b, p1[0], c["alpha"]).S])
        rows = np.unique(np.concatenate([[0, w, L - 1, min(L - 1, chunk), min(L - 1, chunk - 1)],
                                         np.random.default_rng(i * 100 + h).integers(0, L, 6)]))
        for r in rows:
            r = int(r)
            # the global subset as it stood when row r's chunk was processed
            c1 = min(L, (r // chunk + 1) * chunk)
            S_then = S[S < c1]
            ref = orc.attention_row(seqs[i]["Q"][h, r].double().cpu().numpy(), r, Kf[0], Vf[0], S_then, w)
            worst_p = max(worst_p, float(np.abs(ref - seqs[i]["O"][h, r].double().cpu().numpy()).max()))
        # decode replay for this (sequence, head)
        slot = mb.slot_of[i]
        oc = orc.HeadCache(S=[S.copy()], K=Kf.copy(), V=Vf.copy())
        for step in sorted(outs):
            n, Od = outs[step]
            if slot >= n:
                continue
            ref = orc.decode_step(oc, dq[step, slot, h:h + 1].double().cpu().numpy(),
                                  dk[step, slot, kv:kv + 1].double().cpu().numpy(),
                                  dv[step, slot, kv:kv + 1].double().cpu().numpy(), b, w, p1)
            worst_d = max(worst_d, float(np.abs(ref[0] - Od[slot, h].double().cpu().numpy()).max()))
        o, n = int(mb.cache.offs[h]), int(mb.cache.n_rows[slot, h].item())
        assert np.array_equal(mb.cache.idx[slot, o:o + n].cpu().numpy(), oc.S[0]), (i, h)
    print("max abs err prefill rows", worst_p, "decode", worst_d, flush=True)
    assert worst_p <= H.TOL["bf16"] and worst_d <= H.TOL["bf16"]


def test_config3_as_benchmarked_calibrated_budgets(tb, bufs):
    """Config 3 exactly as bench.py times it: budgets from tca_calibrate_budgets on the separate
    8192-token sample, then select + prefill at 131072 tokens.  The oracle calibrates the heads it
    replays by itself, selects for them over the full sequence and attends on sampled rows."""
    c = wl.CONFIGS[3]
    Hq, Hkv, d, L, b, w = c["Hq"], c["Hkv"], c["d"], c["L"], c["b"], c["w"]
    G = Hq // Hkv
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    xc = wl.prefill_inputs(c["kind"], Hq, Hkv, d, c["L_cal"], "bf16", wl.calib_seed(3))
    wsc = bufs.workspace(tb.tca_calibrate_workspace_bytes(prm, c["L_cal"], c["M"]))
    cal = tb.tca_calibrate_budgets(prm, bufs.to_device(xc["Q"]), bufs.to_device(xc["K"]), c["L_cal"], c["M"],
                                   c["sigma"], c["tau"], wsc)
    print("candidates", cal["cand_idx"].tolist(), flush=True)
    heads = [0, 13, Hq - 1]                              # calibrated by the oracle itself, and attended on sampled rows
    cands_orc = orc.candidates(b, c["M"], c["sigma"])
    P_orc = {h: cands_orc[int(cal["cand_idx"][h])] for h in range(Hq)}   # the other heads: the oracle's own candidate of that index
    for h in heads:
        ch = orc.calibrate_head(wl.to_f64(xc["Q"][h]), wl.to_f64(xc["K"][h // G]), b, cands_orc, c["tau"], c["alpha"])
        assert ch.index == cal["cand_idx"][h], f"calibration of head {h}"
        P_orc[h] = ch.p
    del xc, wsc
    x = wl.prefill_inputs(c["kind"], Hq, Hkv, d, L, "bf16", wl.data_seed(3))
    gb, Qd, Kd, Vd = H.gpu_select(tb, bufs, prm, x, cal["p_star"])
    O = torch.full_like(Qd, float("nan"))
    ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(O).any(), "a (head, query tile) of the output was never written"
    print("gpu done", flush=True)
    pos = _sample_positions(L, w, b, 10, 7)
    Og = O[:, torch.from_numpy(pos).cuda()].double().cpu().numpy()
    worst = 0.0
    for h in range(Hq):                                  # the index sets of all heads, in full
        sel = orc.select(wl.to_f64(x["Q"][h, L - 1]), wl.to_f64(x["K"][h // G]), b, P_orc[h], c["alpha"])
        H.assert_selection(sel, H.head_indices(gb, h), b, P_orc[h], tag=f"cfg3 calibrated head {h}")
    for h in heads:
        Kf, Vf = wl.to_f64(x["K"][h // G]), wl.to_f64(x["V"][h // G])
        got = H.head_indices(gb, h)
        qh = wl.to_f64(x["Q"][h][pos])
        for n, i in enumerate(pos):
            ref = orc.attention_row(qh[n], int(i), Kf, Vf, got, w)
            worst = max(worst, float(np.abs(ref - Og[h, n]).max()))
    print("max abs err on", len(pos) * len(heads), "rows:", worst, flush=True)
    assert worst <= H.TOL["bf16"]

    # the two switches at the same size (bench.py --switches).  Gather-free: positions only from
    # tca_select, rows read through idx by tca_prefill; the same numbers reach the same arithmetic,
    # so the output equals the plain one bit for bit.
    n2, idx2 = torch.zeros_like(gb.n_rows), torch.full_like(gb.idx, -1)
    ws_sel = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
    q_last = Qd[:, L - 1].contiguous()
    tb.tca_select(prm, q_last, Kd, Vd, L, 0, L, cal["p_star"], gb.offs, n2, idx2, None, None, ws_sel)
    O2 = torch.full_like(O, float("nan"))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, idx2, None, None, gb.offs, n2, O2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(n2, gb.n_rows)
    for h in range(Hq):
        o, n = int(gb.offs[h]), int(gb.n_rows[h].item())
        assert torch.equal(idx2[o:o + n], gb.idx[o:o + n]), f"gather-free positions, head {h}"
    assert torch.equal(O2, O), "gather-free output"
    print("gather-free equals the plain path", flush=True)
    del idx2
    # Overlapped: window part on a side stream while the selection runs, merged through the
    # log-sum-exp; two more roundings to bf16 than the one-pass kernel, so compared with the oracle
    # on the sampled rows, and the positions with the plain call's.
    n3 = torch.zeros_like(gb.n_rows)
    gb.idx.fill_(-1)
    O2.fill_(float("nan"))
    O_part = torch.full_like(O, float("nan"))
    lse_parts = torch.empty(2, Hq, L, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    tb.tca_select_prefill_overlapped(prm, q_last, Qd, Kd, Vd, L, 0, L, cal["p_star"], gb.offs, n3, gb.idx, gb.Kg, gb.Vg,
                                     O2, O_part, lse_parts, ws_sel, ws, side.cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(n3, n2) and not torch.isnan(O2.float()).any()
    Og = O2[:, torch.from_numpy(pos).cuda()].double().cpu().numpy()
    worst_o = 0.0
    for h in heads:
        Kf, Vf = wl.to_f64(x["K"][h // G]), wl.to_f64(x["V"][h // G])
        o, n = int(gb.offs[h]), int(n3[h].item())
        got = gb.idx[o:o + n].cpu().numpy().astype(np.int64)
        qh = wl.to_f64(x["Q"][h][pos])
        for k, i in enumerate(pos):
            ref = orc.attention_row(qh[k], int(i), Kf, Vf, got, w)
            worst_o = max(worst_o, float(np.abs(ref - Og[h, k]).max()))
    print("overlapped: max abs err on the same rows:", worst_o, "; against the plain output:",
          float((O2.float() - O.float()).abs().max().item()), flush=True)
    assert worst_o <= H.TOL["bf16"]


def test_prefill_is_deterministic_at_full_size(tb, bufs):
    """The bf16 attention kernel synchronises its workgroups' tile copies with one barrier per tile;
    a copy that could land late, or a tile overwritten early, would show as run-to-run differences.
    Config 3: six calls on the same inputs and workspace, every output equal to the first bit for
    bit, with the selection rerun in between so that the workspace and caches are disturbed."""
    c = wl.CONFIGS[3]
    Hq, Hkv, d, L, b, w = c["Hq"], c["Hkv"], c["d"], c["L"], c["b"], c["w"]
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    x = wl.prefill_inputs(c["kind"], Hq, Hkv, d, L, "bf16", wl.data_seed(3))
    fr = wl.budget_fractions(wl.budget_seed(3), Hq)
    P = np.stack([tb.tca_config_from_budget(b, c["sigma"], f) for f in fr])
    gb, Qd, Kd, Vd = H.gpu_select(tb, bufs, prm, x, P)
    ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    ws_sel = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
    q_last = Qd[:, L - 1].contiguous()
    first = None
    for rep in range(6):
        O = torch.full_like(Qd, float("nan"))
        tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
        torch.cuda.synchronize()
        if first is None:
            first = O
        else:
            assert torch.equal(O, first), f"call {rep} differs from the first"
        gb.n_rows.zero_()
        tb.tca_select(prm, q_last, Kd, Vd, L, 0, L, P, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws_sel)
    assert not torch.isnan(first.float()).any()


def test_longest_single_call_4096_blocks_512k_tokens(tb, bufs):
    """The most one tca_select call ranks (4096 blocks of 128 = 524288 tokens), with prefill over
    the same range: 32-bit tile offsets close to their 2 GiB guard, 2048 query tiles per head."""
    Hq, Hkv, d, b, w = 4, 1, 128, 128, 4096
    L = 4096 * b
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    x = wl.device_lowrank_inputs(Hq, Hkv, d, L, 4242)
    fr = [0.08, 0.2, 0.35, 0.5]
    P_gpu = np.stack([tb.tca_config_from_budget(b, 1.0, f) for f in fr])
    P_orc = np.stack([orc.config_from_budget(b, 1.0, f) for f in fr])
    total, rows = tb.tca_select_rows(prm, L // b, P_gpu)
    gb = bufs.GlobalBuffers(prm, rows)
    ws = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
    tb.tca_select(prm, x["Q"][:, L - 1].contiguous(), x["K"], x["V"], L, 0, L, P_gpu, gb.offs, gb.n_rows,
                  gb.idx, gb.Kg, gb.Vg, ws)
    del ws
    O = torch.full_like(x["Q"], float("nan"))
    wsp = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    tb.tca_prefill(prm, x["Q"], 0, L, x["K"], x["V"], L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, wsp)
    torch.cuda.synchronize()
    assert not torch.isnan(O).any(), "a (head, query tile) of the output was never written"
    print("gpu done", flush=True)
    Kf, Vf = x["K"][0].double().cpu().numpy(), x["V"][0].double().cpu().numpy()
    pos = _sample_positions(L, w, b, 6, 5)
    worst = 0.0
    for h in (0, Hq - 1):
        sel = orc.select(x["Q"][h, L - 1].double().cpu().numpy(), Kf, b, P_orc[h], 0.5)
        got = H.head_indices(gb, h)
        H.assert_selection(sel, got, b, P_orc[h], tag=f"512K head {h}")
        for i in pos:
            ref = orc.attention_row(x["Q"][h, int(i)].double().cpu().numpy(), int(i), Kf, Vf, got, w)
            worst = max(worst, float(np.abs(ref - O[h, int(i)].double().cpu().numpy()).max()))
    print("max abs err on", 2 * len(pos), "rows:", worst, flush=True)
    assert worst <= H.TOL["bf16"]


def test_diagnostics_clock_and_mfma_probe(tb, bufs):
    """The MFMA probe returns plausible figures; a bf16 prefill leaves the cycle / tick sums of its
    attention kernel at the head of its workspace when tca_diag_prefill_clocks is on, and does
    not touch that place when it is off (the default)."""
    wsp = bufs.workspace(tb.tca_probe_workspace_bytes())
    tf_c, ghz_c = tb.tca_probe_mfma(False, 2000, wsp)
    tf_r, ghz_r = tb.tca_probe_mfma(True, 2000, wsp)
    print("probe: constants %.0f TFLOP/s at %.2f GHz, random %.0f TFLOP/s at %.2f GHz" % (tf_c, ghz_c, tf_r, ghz_r), flush=True)
    for tf, ghz in ((tf_c, ghz_c), (tf_r, ghz_r)):
        assert 300.0 < tf < 2600.0 and 0.5 < ghz < 2.6
        # 1024 SIMDs x 1024 flop per cycle at the measured clock bounds the rate
        assert tf <= 1024 * 1024 * ghz * 1e9 / 1e12 * 1.05
    with pytest.raises(tb.TcaError):
        tb.tca_probe_mfma(True, 0, wsp)
    Hq, Hkv, d, L, b, w = 8, 2, 128, 2048, 64, 256
    x = wl.prefill_inputs("lowrank", Hq, Hkv, d, L, "bf16", 77)
    P = np.stack([tb.tca_config_from_budget(b, 1.0, 0.3) for _ in range(Hq)])
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    gb, Qd, Kd, Vd = H.gpu_select(tb, bufs, prm, x, P)
    O = torch.full_like(Qd, float("nan"))
    ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
    torch.cuda.synchronize()
    assert bool((ws[:16] == 0xFF).all()), "clock counters written although the diagnostics switch is off"
    try:
        tb.tca_diag_prefill_clocks(True)
        tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
        ghz = tb.prefill_shader_clock_ghz(ws)
    finally:
        tb.tca_diag_prefill_clocks(False)
    print("prefill shader clock %.3f GHz" % ghz, flush=True)
    assert 0.3 < ghz < 2.6


def test_qkv_project_full_size_sampled_rows(tb, bufs):
    """The Q / K / V projections at the size bench.py --projection times (131072 rows, hidden 4096, 32 + 8 + 8
    heads of 128, head-major outputs, bias): every output element is written, and all 6144 features of
    sampled rows (the first and last row of the call, rows either side of workgroup-tile boundaries,
    random ones) equal the fp64 projections rounded to bf16 or their neighbour."""
    c = wl.CONFIGS[3]
    Hq, Hkv, d, L, hidden = c["Hq"], c["Hkv"], c["d"], c["L"], 4096
    x = wl.device_projection_inputs(Hq, Hkv, d, hidden, L, wl.data_seed(3) + 50)
    prm = H.params_for(tb, Hq, Hkv, d, c["b"], c["w"], "bf16")
    Q = torch.full((Hq, L, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    K = torch.full((Hkv, L, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    V = torch.full((Hkv, L, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    tb.tca_qkv_project(prm, x["X"], L, hidden, x["W"], x["bias"], Q, d, L * d, K, V, d, L * d)
    torch.cuda.synchronize()
    print("gpu done", flush=True)
    for name, T in zip("QKV", (Q, K, V)):
        assert not torch.isnan(T).any(), f"{name}: an element was never written"
    rng = np.random.default_rng(17)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, 2047, 2048, L // 2 - 1, L // 2, L - 257, L - 256, L - 2, L - 1],
                                     rng.integers(0, L, size=40)]))
    ri = torch.from_numpy(rows).cuda()
    Xs = x["X"][ri].double().cpu().numpy()
    ref = orc.qkv_project(Xs, x["W"].double().cpu().numpy(), Hq, Hkv, d, bias=x["bias"].double().cpu().numpy())
    worst = 0.0
    for name, T, r in zip("QKV", (Q, K, V), ref):
        got = T[:, ri].double().cpu().numpy()
        err = np.abs(got - r)
        bound = 2.0 ** -8 * np.abs(r) + 1e-4
        worst = max(worst, float((err / bound).max()))
        assert (err <= bound).all(), f"{name}: worst error {err.max()}"
        assert err.max() <= H.TOL["bf16"]
    print("worst error in units of the bound on", len(rows), "rows:", worst, flush=True)
