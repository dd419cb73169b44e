"""Benchmark of the TCA hot path on one MI355X.

A step = one pass of the prefill hot path over one 128K-token sequence:
tca_select (scores, block metric, ranking, budgets, top-t, compaction) followed
by tca_prefill (attention over the global and local subsets).  Inputs are
resident in HBM before the timed region.  The decode path (batch 16 at 128K
context) is timed in the same run and reported in the "decode" object.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
# HBM bytes per kernel launch on the default workload come from the counter runs summarised in this
# file (written by paper_2512_09238_amd.profile_summary); its figures are reported only while the
# kernel sources still hash to what was profiled, else `traffic` is null
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_config3.json")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def visible_pairs(idx_host, L, w):
    """(query, key) pairs of Eq. 2 for one head: global rows with idx <= i-w plus the window."""
    i = np.arange(L, dtype=np.int64)
    glob = np.searchsorted(idx_host, i - w, side="right").sum()
    local = np.minimum(i + 1, w).sum()
    return int(glob + local)


def bench_prefill(args, tb, bufs, wl, torch, share=False, x=None):
    """share: one selection per KV head (tca_params.share = TCA_SHARE_GROUP) on the same inputs."""
    cfg = dict(wl.CONFIGS[3])
    if args.L:
        cfg["L"] = args.L
    Hq, Hkv, d, L, b, w = cfg["Hq"], cfg["Hkv"], cfg["d"], cfg["L"], cfg["b"], cfg["w"]
    if x is None:
        log(f"[bench] generating config-3 inputs: Hq={Hq} Hkv={Hkv} d={d} L={L} bf16 ...")
        t0 = time.time()
        x = wl.prefill_inputs(cfg["kind"], Hq, Hkv, d, L, "bf16", wl.data_seed(3))
        log(f"[bench] inputs generated in {time.time() - t0:.1f}s")
    prm = tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16, cfg["alpha"], 0.0,
                         share=tb.TCA_SHARE_GROUP if share else tb.TCA_SHARE_HEAD)
    Hs = tb.tca_selection_heads(prm)
    GS = Hq // Hs

    budget_src = "uniform[0.05,0.5]"
    budget = ("frac", wl.budget_fractions(wl.budget_seed(3), Hs))
    fr = budget[1]
    P = np.stack([tb.tca_config_from_budget(b, cfg["sigma"], f) for f in fr])
    if args.calibrate:
        Lc = cfg["L_cal"]
        xc = wl.prefill_inputs(cfg["kind"], Hq, Hkv, d, Lc, "bf16", wl.calib_seed(3))
        Qc, Kc = bufs.to_device(xc["Q"]), bufs.to_device(xc["K"])
        wsc = bufs.workspace(tb.tca_calibrate_workspace_bytes(prm, Lc, cfg["M"]))
        t0 = time.time()
        cal = tb.tca_calibrate_budgets(prm, Qc, Kc, Lc, cfg["M"], cfg["sigma"], cfg["tau"], wsc)
        log(f"[bench] calibration on {Lc} tokens: {1e3 * (time.time() - t0):.1f} ms, candidates {cal['cand_idx'].tolist()}")
        P = cal["p_star"]
        budget = ("cand", cal["cand_idx"].astype(np.int64))
        budget_src = f"tca_calibrate_budgets(L_cal={Lc}, M={cfg['M']}, tau={cfg['tau']})"
        del Qc, Kc, wsc

    total, rows = tb.tca_select_rows(prm, L // b, P)
    gb = bufs.GlobalBuffers(prm, rows)
    Qd, Kd, Vd = bufs.to_device(x["Q"]), bufs.to_device(x["K"]), bufs.to_device(x["V"])
    q_last = Qd[:, L - 1].contiguous()
    O = torch.empty_like(Qd)
    ws_sel = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
    ws_pf = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
    log(f"[bench] realised budget {total / (Hs * L):.4f} of L per head on average; {total} global rows")

    def step(ev=None):
        gb.n_rows.zero_()
        if ev: ev[0].record()
        tb.tca_select(prm, q_last, Kd, Vd, L, 0, L, P, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws_sel)
        if ev: ev[1].record()
        tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws_pf)
        if ev: ev[2].record()

    for i in range(args.warmup):
        step()
        torch.cuda.synchronize()
        log(f"[bench] warmup {i + 1}/{args.warmup} done")
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    sel_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    pf_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    ms_per_step = 1e3 * wall / args.steps
    log(f"[bench] step {ms_per_step:.3f} ms (select {sel_ms:.3f} ms, prefill {pf_ms:.3f} ms)")
    # what the attention kernel's clock was, and what the matrix pipe sustains on this board with
    # constant and with random operands (register-only loop, no memory traffic)
    clock_ghz = tb.prefill_shader_clock_ghz(ws_pf)
    wsp = bufs.workspace(tb.tca_probe_workspace_bytes())
    probe_c = tb.tca_probe_mfma(False, 20000, wsp)
    probe_r = tb.tca_probe_mfma(True, 20000, wsp)
    log(f"[bench] shader clock during prefill_mfma_kernel {clock_ghz:.3f} GHz; MFMA probe: constants "
        f"{probe_c[0]:.0f} TFLOP/s at {probe_c[1]:.2f} GHz, random operands {probe_r[0]:.0f} TFLOP/s at {probe_r[1]:.2f} GHz")

    idx_host = gb.idx.cpu().numpy()
    n_rows = gb.n_rows.cpu().numpy()
    pairs = GS * sum(visible_pairs(idx_host[int(gb.offs[h]):int(gb.offs[h]) + int(n_rows[h])], L, w) for h in range(Hs))
    flops = 4.0 * d * pairs
    tflops = flops / (pf_ms * 1e-3) / 1e12
    e = 2
    sel_bytes = Hkv * L * d * e + Hs * L + 2 * int(n_rows.sum()) * (2 * d * e) + 4 * int(n_rows.sum())
    res = {
        "L": L, "ms_per_step": ms_per_step, "select_ms": sel_ms, "prefill_ms": pf_ms,
        "tokens_per_s": L / (ms_per_step * 1e-3), "pairs": pairs, "flops": flops, "tflops": tflops,
        "select_gbs": sel_bytes / (sel_ms * 1e-3) / 1e9, "select_bytes": sel_bytes,
        "budget_src": budget_src, "mean_budget": total / (Hs * L), "cfg": cfg, "global_rows": int(total),
        "clock_ghz": clock_ghz, "probe_const": probe_c, "probe_random": probe_r,
    }
    host = {"x": x, "P": P, "idx": idx_host, "offs": gb.offs, "n_rows": n_rows, "O": O, "prm": prm, "budget": budget}
    return res, host


def bench_projection(args, tb, bufs, wl, torch):
    """The Q / K / V projections in front of the path (tca_qkv_project) on the rows of config 3: hidden
    size 4096 (the model the configuration is shaped after), all 48 heads, head-major outputs.  Not
    part of the default step: the metric's workload starts from Q, K, V."""
    cfg = dict(wl.CONFIGS[3])
    if args.L:
        cfg["L"] = args.L
    Hq, Hkv, d, L, hidden = cfg["Hq"], cfg["Hkv"], cfg["d"], cfg["L"], 4096
    x = wl.device_projection_inputs(Hq, Hkv, d, hidden, L, wl.data_seed(3) + 50)
    prm = tb.make_params(Hq, Hkv, d, cfg["b"], cfg["w"], tb.TCA_BF16, cfg["alpha"], 0.0)
    Q = torch.empty(Hq, L, d, dtype=torch.bfloat16, device="cuda")
    K, V = torch.empty(Hkv, L, d, dtype=torch.bfloat16, device="cuda"), torch.empty(Hkv, L, d, dtype=torch.bfloat16, device="cuda")
    run = lambda: tb.tca_qkv_project(prm, x["X"], L, hidden, x["W"], x["bias"], Q, d, L * d, K, V, d, L * d)
    for _ in range(max(1, args.warmup)):
        run()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ev[0].record()
    for i in range(args.steps):
        run()
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]))
    flops = 2.0 * L * hidden * (Hq + 2 * Hkv) * d
    tflops = flops / (ms * 1e-3) / 1e12
    log(f"[bench] tca_qkv_project: {ms:.3f} ms for {L} rows x {hidden} -> {(Hq + 2 * Hkv) * d} features = {tflops:.0f} TFLOP/s")
    return {"what": f"tca_qkv_project, {L} rows, hidden {hidden}, {(Hq + 2 * Hkv) * d} output features, bf16, head-major outputs",
            "ms": ms, "flops": flops, "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": tflops / PEAK_BF16_TFLOPS, "bound": "mfma"}


def bench_switches(args, tb, bufs, wl, torch, host, cfg):
    """The two switches beside the plain path, on the same inputs and budgets (not part of the default
    run): gather-free prefill (no compacted copy of the kept rows) and the window part of the
    attention overlapped with the selection; each at the full length and on the last 8192-token
    chunk of the sequence with the earlier blocks already selected."""
    x, P, prm = host["x"], host["P"], host["prm"]
    Hq, Hkv, d, L, b = cfg["Hq"], cfg["Hkv"], cfg["d"], cfg["L"], cfg["b"]
    Hs = tb.tca_selection_heads(prm)
    Qd, Kd, Vd = bufs.to_device(x["Q"]), bufs.to_device(x["K"]), bufs.to_device(x["V"])
    side = torch.cuda.Stream()
    out = {}
    chunk = 8192
    for name, pos0 in (("full_length", 0), ("last_chunk_8192", L - chunk)):
        n = L - pos0
        _, rows_prev = tb.tca_select_rows(prm, pos0 // b, P)
        _, rows_new = tb.tca_select_rows(prm, n // b, P)
        gb = bufs.GlobalBuffers(prm, rows_prev + rows_new)
        ws_sel = bufs.workspace(tb.tca_select_workspace_bytes(prm, max(n, pos0)))
        ws_pf = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, n, int(gb.offs[-1])))
        if pos0:
            tb.tca_select(prm, Qd[:, pos0 - 1].contiguous(), Kd, Vd, L, 0, pos0, P, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws_sel)
        n_before = gb.n_rows.clone()
        q_last = Qd[:, L - 1].contiguous()
        Qc = Qd[:, pos0:].contiguous()
        O, O_part = torch.empty_like(Qc), torch.empty_like(Qc)
        lse_parts = torch.empty(2, Hq, n, dtype=torch.float32, device="cuda")

        def plain():
            tb.tca_select(prm, q_last, Kd, Vd, L, pos0, n, P, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws_sel)
            tb.tca_prefill(prm, Qc, pos0, n, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws_pf)

        def gather_free():
            tb.tca_select(prm, q_last, Kd, Vd, L, pos0, n, P, gb.offs, gb.n_rows, gb.idx, None, None, ws_sel)
            tb.tca_prefill(prm, Qc, pos0, n, Kd, Vd, L, gb.idx, None, None, gb.offs, gb.n_rows, O, None, ws_pf)

        def overlapped():
            tb.tca_select_prefill_overlapped(prm, q_last, Qc, Kd, Vd, L, pos0, n, P, gb.offs, gb.n_rows, gb.idx, gb.Kg,
                                             gb.Vg, O, O_part, lse_parts, ws_sel, ws_pf, side.cuda_stream)

        res = {}
        for label, fn in (("plain", plain), ("gather_free", gather_free), ("overlapped", overlapped)):
            if label == "gather_free" and pos0:
                continue            # the earlier chunks' rows would have to be kept as positions only as well: same kernel, not timed twice
            ms = []
            for it in range(4):
                gb.n_rows.copy_(n_before)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                torch.cuda.synchronize()
                ms.append(e0.elapsed_time(e1))
            res[label + "_ms"] = float(np.mean(ms[1:]))
        out[name] = res
        log(f"[bench] switches, {name}: " + ", ".join(f"{k} {v:.3f}" for k, v in res.items()))
        del gb, ws_sel, ws_pf, O, O_part, lse_parts, Qc
    return out


def cpu_baseline_prefill(host, cfg, wl, bufs, seconds=20.0, seed=5):
    """Times the oracle on the host: selection for every head in full, then
    Eq. 2 for a seeded sample of token positions (all heads each) until about
    `seconds` have elapsed.  Also returns the parity error on those rows."""
    from threadpoolctl import threadpool_info
    from oracle import tca_oracle as orc
    x = host["x"]
    Hq, Hkv, d, L, b, w = cfg["Hq"], cfg["Hkv"], cfg["d"], cfg["L"], cfg["b"], cfg["w"]
    Kf, Vf = wl.to_f64(x["K"]), wl.to_f64(x["V"])
    # the oracle derives its configurations itself, from the same fractions / candidate indices
    kind, val = host["budget"]
    if kind == "frac":
        Po = np.stack([orc.config_from_budget(b, cfg["sigma"], f) for f in val])
    else:
        Po = orc.candidates(b, cfg["M"], cfg["sigma"])[val]
    t0 = time.perf_counter()
    sels = orc.select_all_heads(wl.to_f64(x["Q"][:, L - 1]), Kf, b, Po, cfg["alpha"])
    t_sel = time.perf_counter() - t0
    same = all(np.array_equal(sels[h].S, host["idx"][int(host["offs"][h]):int(host["offs"][h]) + len(sels[h].S)])
               for h in range(Hq))
    rng = np.random.default_rng(seed)
    pos = np.concatenate([[L - 1, w - 1, w, 0], rng.integers(0, L, size=4096)])
    Og = host["O"]
    n_done, err = 0, 0.0
    t0 = time.perf_counter()
    for i in pos:
        i = int(i)
        for h in range(Hq):
            g = h // (Hq // Hkv)
            ref = orc.attention_row(wl.to_f64(x["Q"][h, i]), i, Kf[g], Vf[g], sels[h].S, w)
            err = max(err, float(np.abs(ref - Og[h, i].double().cpu().numpy()).max()))
        n_done += 1
        if time.perf_counter() - t0 > seconds:
            break
    t_att = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {
        "value": n_done / t_att, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": f"Eq. 2 for {n_done} seeded token positions x {Hq} heads in {t_att:.1f}s "
                  f"(full selection for all heads took {t_sel:.1f}s extra, amortised over L it adds "
                  f"{1e6 * t_sel / L:.1f} us/token); host has {os.cpu_count()} cpus",
        "index_sets_equal_gpu": bool(same), "max_abs_err_vs_gpu": err,
    }


def bench_decode(args, tb, bufs, wl, torch, share=False, fp8=False):
    """fp8: the cache rows are FP8 E4M3 codes with one scale per row (TCA_KV_FP8)."""
    cfg = dict(wl.CONFIGS[4])
    Hq, Hkv, d, T0, b, w, B, steps = (cfg[k] for k in ("Hq", "Hkv", "d", "L", "b", "w", "batch", "steps"))
    if args.decode_batch:
        B = args.decode_batch
    prm = tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16, cfg["alpha"], 0.0,
                         share=tb.TCA_SHARE_GROUP if share else tb.TCA_SHARE_HEAD)
    Hs = tb.tca_selection_heads(prm)
    fr = wl.budget_fractions(wl.budget_seed(4), Hs)
    P = np.stack([tb.tca_config_from_budget(b, cfg["sigma"], f) for f in fr])
    n_glob = np.round(fr * (T0 - w)).astype(np.int64)
    t_dec = np.array([tb.tca_decode_budget(b, p) for p in P])
    cap = n_glob + t_dec * (steps // b + 2)
    cache = bufs.DecodeCache(prm, B, cap, kv_format=tb.TCA_KV_FP8 if fp8 else tb.TCA_KV_NATIVE)
    g = torch.Generator(device="cuda").manual_seed(wl.data_seed(4))
    rng = np.random.default_rng(wl.data_seed(4))
    pend = rng.integers(0, b, size=B)                     # pending tokens of the open block
    lengths = T0 + pend

    def fill(rows, scales):
        if not fp8:
            rows.copy_(torch.randn(rows.shape, generator=g, device="cuda", dtype=torch.float32))
            return
        codes = torch.randint(0, 256, rows.shape, generator=g, device="cuda", dtype=torch.uint8)
        codes[(codes & 0x7F) == 0x7F] = 0                 # the two NaN codes
        rows.copy_(codes)
        scales.copy_(torch.rand(scales.shape, generator=g, device="cuda") * 0.015 + 0.005)

    for s in range(B):
        fill(cache.Kg[s], cache.Kg_scale[s] if fp8 else None)
        fill(cache.Vg[s], cache.Vg_scale[s] if fp8 else None)
        for h in range(Hs):
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
    O = torch.empty(steps, B, Hq, d, device="cuda", dtype=torch.bfloat16)
    ws = bufs.workspace(tb.tca_decode_workspace_bytes(prm, B, cache.max_head_rows))
    for s in range(2):                                    # warm-up steps (they advance the cache too)
        tb.tca_decode(prm, cache.view, cache.offs, q[s], kn[s], vn[s], P, O[s], ws)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for s in range(steps):
        tb.tca_decode(prm, cache.view, cache.offs, q[s], kn[s], vn[s], P, O[s], ws)
        ev[s + 1].record()
    torch.cuda.synchronize()
    us = np.array([ev[s].elapsed_time(ev[s + 1]) * 1e3 for s in range(steps)])
    row_bytes = (d + 4) if fp8 else 2 * d                 # a cache row: codes and a float scale, or bf16 elements
    bytes_step = B * (int(n_glob.sum()) * 2 * row_bytes + Hkv * w * 2 * row_bytes)
    res = {
        "kv_format": "fp8 e4m3 + scale per row" if fp8 else "bf16",
        "batch": B, "context": T0, "steps": steps, "us_per_step_mean": float(us.mean()),
        "us_per_step_p50": float(np.percentile(us, 50)), "us_per_step_p99": float(np.percentile(us, 99)),
        "algorithmic_bytes_per_step": bytes_step,
        "achieved_gbs": bytes_step / (us.mean() * 1e-6) / 1e9, "peak_gbs": PEAK_HBM_GBS,
        "frac": bytes_step / (us.mean() * 1e-6) / 1e9 / PEAK_HBM_GBS,
        "mean_budget": float(fr.mean()),
    }
    log(f"[bench] decode ({res['kv_format']}{', shared selection' if share else ''}): {res['us_per_step_mean']:.1f} us/step, {res['achieved_gbs']:.0f} GB/s")
    return res


def bench_mixed(args, tb, bufs, wl, torch):
    """Config 5 (not part of the default run): 8 sequences of ragged length prefilled in
    8192-token chunks, round-robin, with one decode step for the finished sequences after
    every chunk.  Wall time of the whole schedule, host scheduling included."""
    import paper_2512_09238_amd.schedule as sched
    c = wl.CONFIGS[5]
    Hq, Hkv, d, b, w, chunk = c["Hq"], c["Hkv"], c["d"], c["b"], c["w"], c["chunk"]
    lengths = wl.config5_lengths()
    prm = tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16, c["alpha"], 0.0)
    xc = wl.device_lowrank_inputs(Hq, Hkv, d, c["L_cal"], wl.calib_seed(5))
    wsc = bufs.workspace(tb.tca_calibrate_workspace_bytes(prm, c["L_cal"], c["M"]))
    cal = tb.tca_calibrate_budgets(prm, xc["Q"], xc["K"], c["L_cal"], c["M"], c["sigma"], c["tau"], wsc)
    del xc, wsc
    seqs = []
    for i, L in enumerate(lengths):
        x = wl.device_lowrank_inputs(Hq, Hkv, d, L, wl.data_seed(5) + 10 * i)
        seqs.append(dict(Q=x["Q"], K=x["K"], V=x["V"], O=torch.empty_like(x["Q"])))
    g = torch.Generator(device="cuda").manual_seed(77)
    best = None
    for rep in range(2):                       # the second pass has warm allocations
        mb = sched.MixedBatch(prm, lengths, chunk, cal["p_star"])
        n_calls = len(mb.events)
        dq = torch.randn(n_calls, len(lengths), Hq, d, generator=g, device="cuda").to(torch.bfloat16)
        dk = torch.randn(n_calls, len(lengths), Hkv, d, generator=g, device="cuda").to(torch.bfloat16)
        dv = torch.randn(n_calls, len(lengths), Hkv, d, generator=g, device="cuda").to(torch.bfloat16)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        mb.run(seqs, lambda step, slots: (dq[step, :len(slots)].contiguous(), dk[step, :len(slots)].contiguous(),
                                          dv[step, :len(slots)].contiguous()))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
        n_dec_steps, n_done = mb.decode_calls, mb.n_done
        del mb, dq, dk, dv
    total = int(sum(lengths))
    log(f"[bench] mixed batch: {total} prefill tokens in {len(lengths)} sequences, {n_dec_steps} decode steps: {1e3 * best:.1f} ms")
    return {"lengths": lengths, "chunk": chunk, "prefill_tokens": total, "decode_steps": n_dec_steps,
            "wall_ms": 1e3 * best, "prefill_tokens_per_s": total / best,
            "what": "config 5: Hq=64 Hkv=8 d=128 bf16, chunked prefill interleaved with decode, host scheduling included"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--L", type=int, default=0, help="override the sequence length (default: 131072)")
    ap.add_argument("--decode-batch", type=int, default=0)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle baseline leg")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--calibrate", action="store_true", default=True)
    ap.add_argument("--no-calibrate", dest="calibrate", action="store_false")
    ap.add_argument("--projection", action="store_true",
                    help="also time the Q / K / V projections in front of the path (tca_qkv_project, hidden size 4096)")
    ap.add_argument("--mixed", action="store_true", help="also time the config-5 ragged mixed batch (adds about a minute)")
    ap.add_argument("--prefill-variant", type=int, default=0,
                    help="workgroup shape of the bf16 prefill kernel (tca_diag_prefill_variant): 0 = automatic")
    ap.add_argument("--switches", action="store_true",
                    help="also time the gather-free prefill and the overlapped window part beside the plain path")
    ap.add_argument("--shared", action="store_true",
                    help="also time both workloads with one selection per KV head (tca_params.share), reported in 'shared_selection'")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build covers one GPU only (no sharding, no collectives); run with --gpus 1")

    import torch
    import paper_2512_09238_amd.binding as tb
    import paper_2512_09238_amd.buffers as bufs
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    tb.tca_diag_prefill_clocks(True)             # the attention kernel's shader clock is part of the report
    tb.tca_diag_prefill_variant(args.prefill_variant)
    log(f"[bench] device {props.name}: {props.multi_processor_count} CUs")

    if args.copy_probe:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b_ = torch.empty_like(a)
        a.fill_(1)
        torch.cuda.synchronize()
        b_.copy_(a)                      # the plain copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b_
        torch.cuda.empty_cache()

    res, host = bench_prefill(args, tb, bufs, wl, torch)
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline_prefill(host, res["cfg"], wl, bufs, seconds=args.cpu_seconds)
        log(f"[bench] oracle: {cpu['value']:.2f} tokens/s on {cpu['cores']} threads; "
            f"max abs err vs GPU on sampled rows {cpu['max_abs_err_vs_gpu']:.3e}; index sets equal: {cpu['index_sets_equal_gpu']}")
    switches = bench_switches(args, tb, bufs, wl, torch, host, res["cfg"]) if args.switches else None
    shared = None
    if args.shared:
        rs, hs_ = bench_prefill(args, tb, bufs, wl, torch, share=True, x=host["x"])
        del hs_
        shared = {"what": "the same workloads with tca_params.share = TCA_SHARE_GROUP: one selection per KV head",
                  "ms_per_step": rs["ms_per_step"], "select_ms": rs["select_ms"], "prefill_ms": rs["prefill_ms"],
                  "prefill_tflops": rs["tflops"], "global_rows": rs["global_rows"], "mean_budget_frac": rs["mean_budget"],
                  "select_gbs": rs["select_gbs"], "select_frac": rs["select_gbs"] / PEAK_HBM_GBS,
                  "per_head_global_rows": res["global_rows"]}
    del host
    torch.cuda.empty_cache()
    dec = None if args.no_decode else bench_decode(args, tb, bufs, wl, torch)
    dec_fp8 = None if args.no_decode else bench_decode(args, tb, bufs, wl, torch, fp8=True)
    if shared is not None and not args.no_decode:
        shared["decode"] = bench_decode(args, tb, bufs, wl, torch, share=True)
    mixed = bench_mixed(args, tb, bufs, wl, torch) if args.mixed else None
    projection = bench_projection(args, tb, bufs, wl, torch) if args.projection else None

    cfg = res["cfg"]
    import paper_2512_09238_amd.profile_summary as ps
    default_workload = res["L"] == 131072 and args.calibrate and args.prefill_variant == 0
    traffic_doc = ps.load_traffic(TRAFFIC_FILE) if default_workload else None
    prefill_traffic = ps.kernel_bytes(traffic_doc, "prefill_mfma_kernel")
    sel_traffic = None
    if traffic_doc is not None:
        parts = [ps.kernel_bytes(traffic_doc, k) for k in ("score_kernel", "gather_kernel")]   # assign_kernel: kilobytes
        sel_traffic = sum(parts) if all(v is not None for v in parts) else None
    out = {
        "metric": "prefill tokens/s at 128K context (select + compaction + sparse attention, one layer)",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": f"config 3: Llama-3-8B-shaped layer, Hq={cfg['Hq']} Hkv={cfg['Hkv']} d={cfg['d']} "
                        f"L={res['L']} bf16, b={cfg['b']} w={cfg['w']}, low-rank keys with 30% near-duplicates",
            "budgets": res["budget_src"], "mean_budget_frac": res["mean_budget"],
            "select_ms": res["select_ms"], "prefill_ms": res["prefill_ms"],
        },
        "roofline": {
            "kernel": "prefill_mfma_kernel", "bound": "mfma", "achieved": res["tflops"], "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": res["tflops"] / PEAK_BF16_TFLOPS,
            "traffic": prefill_traffic,
            "flops_per_launch": res["flops"], "visible_pairs": res["pairs"],
            "shader_clock_ghz": res["clock_ghz"],
            "mfma_probe": {
                "what": "register-only bf16 32x32x16 MFMA loop on every SIMD (tca_probe_mfma): TFLOP/s and shader clock",
                "constant_operands": {"tflops": res["probe_const"][0], "ghz": res["probe_const"][1]},
                "random_operands": {"tflops": res["probe_random"][0], "ghz": res["probe_random"][1]},
            },
            "frac_of_random_operand_probe": res["tflops"] / res["probe_random"][0] if res["probe_random"][0] else None,
        },
        "select_roofline": {
            "bound": "hbm", "achieved": res["select_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": res["select_gbs"] / PEAK_HBM_GBS, "bytes_per_launch": res["select_bytes"],
            "traffic": sel_traffic,
            "achieved_on_counted_traffic": sel_traffic / (res["select_ms"] * 1e-3) / 1e9 if sel_traffic else None,
        },
        "cpu_baseline": cpu,
        "decode": dec,
        "decode_fp8_cache": dec_fp8,
    }
    if switches is not None:
        out["switches"] = switches
    if mixed is not None:
        out["mixed_batch"] = mixed
    if projection is not None:
        out["qkv_project"] = projection
    if shared is not None:
        out["shared_selection"] = shared
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
