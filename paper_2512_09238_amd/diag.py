"""Diagnostics of the bf16 prefill kernel (not part of the hot path; uses include/tca_diag.h).

  python -m paper_2512_09238_amd.diag occupancy [--heads 32 16 8] [--variants 3 2] [--queries 2048] [--length 131072]

  python -m paper_2512_09238_amd.diag loop {prefill,tail,probe-random,probe-constant} [--seconds 10]
                                           [--heads 8] [--queries 2048] [--variant 3]

`loop`: keeps the GPU on one kind of work for some seconds, so that the board's energy counter can be
read meanwhile from another shell (`rocm-smi --showenergycounter` every few hundred milliseconds;
power = energy difference over time difference): `prefill` repeats config 3's tca_select + tca_prefill
(131072 tokens, budget 57 % for every head), `tail` the attention kernel alone on the last queries
of that sequence with few heads (the workload of `occupancy`: part of the chip, below the power
limit, in a chosen workgroup shape), the probes repeat tca_probe_mfma with operands of
random sign and magnitude, or constant.  Prints the start and end times of the loop, the mean step
time or rate, and the shader clock.

`occupancy`: the attention kernel on the last 2048 queries of a 131072-token sequence (config 3's
recipe, budget 57 % for every head) with 32, 16 and 8 query heads: 256, 128 and 64 workgroups of the
same work each, i.e. the whole chip, half and a quarter of it.  Prints per call the event-timed
duration, the mean workgroup duration and the shader clock, both from the kernel's own counters
(cycle counter and 100 MHz counter, tca_diag_prefill_clocks), the cycles per workgroup, how many of
them pass before the first tile step, and the tiles a workgroup walks.  Equal
cycles at different clocks separate what the code costs from what the power limit costs.
--variants names the workgroup shapes to run (tca_diag_prefill_variant: 1 = 4 waves x 32 queries,
2 = 4 x 64, 3 = 8 x 32, the shape of long calls and the default here).
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def occupancy(args):
    import torch
    import workloads as wl
    from paper_2512_09238_amd import binding as tb, buffers as bufs
    L, d, b, w, n = args.length, 128, 128, 4096, args.queries
    tb.tca_diag_prefill_clocks(True)
    try:
        for Hq in args.heads:
            Hkv = max(1, Hq // 4)
            x = wl.prefill_inputs("lowrank", Hq, Hkv, d, L, "bf16", wl.data_seed(3))
            prm = tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16, 0.5, 0.0, tb.TCA_METRIC_HHI, tb.TCA_SHARE_HEAD)
            P = np.stack([tb.tca_config_from_budget(b, 1.0, 0.57) for _ in range(Hq)])
            Qd, Kd, Vd = bufs.to_device(x["Q"]), bufs.to_device(x["K"]), bufs.to_device(x["V"])
            _, rows = tb.tca_select_rows(prm, L // b, P)
            gb = bufs.GlobalBuffers(prm, rows)
            ws_sel = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
            tb.tca_select(prm, Qd[:, L - 1].contiguous(), Kd, Vd, L, 0, L, P, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws_sel)
            ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, n, int(gb.offs[-1])))
            Qc = Qd[:, L - n:].contiguous()
            O = torch.empty_like(Qc)
            for variant in args.variants:
                tb.tca_diag_prefill_variant(variant)
                per_wg_queries = 128 if variant == 1 else 256
                nwg = Hq * (n // per_wg_queries)
                res = []
                for _ in range(args.repeats + 1):
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    tb.tca_prefill(prm, Qc, L - n, n, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
                    e1.record()
                    torch.cuda.synchronize()
                    c = ws[:16].view(torch.int64).cpu().numpy()
                    c4 = ws[:32].view(torch.int64).cpu().numpy()
                    res.append((e0.elapsed_time(e1), c[1] / nwg / 100.0, c[0] / (c[1] * 10.0), c[0] / nwg / 1e6,
                                c4[2] / nwg / 1e3, c4[3] / nwg))
                t, u, g, cyc, pro, tiles = (float(np.mean([r[i] for r in res[1:]])) for i in range(6))
                print(f"heads {Hq:3d}  shape {variant}  workgroups {nwg:4d}:  call {t:.3f} ms   workgroup {u:7.1f} us   "
                      f"clock {g:.2f} GHz   {cyc:.2f} M cycles per workgroup, {pro:.1f} K of them before the first of "
                      f"{tiles:.0f} tiles", flush=True)
            tb.tca_diag_prefill_variant(0)
            del gb, ws, ws_sel, Qd, Kd, Vd, Qc, O
            torch.cuda.empty_cache()
    finally:
        tb.tca_diag_prefill_variant(0)
        tb.tca_diag_prefill_clocks(False)


def loop(args):
    import time
    import torch
    import workloads as wl
    from paper_2512_09238_amd import binding as tb, buffers as bufs
    if args.what == "prefill":
        c = wl.CONFIGS[3]
        Hq, Hkv, d, L, b, w = c["Hq"], c["Hkv"], c["d"], c["L"], c["b"], c["w"]
        x = wl.prefill_inputs(c["kind"], Hq, Hkv, d, L, "bf16", wl.data_seed(3))
        prm = tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16, c["alpha"], 0.0, tb.TCA_METRIC_HHI, tb.TCA_SHARE_HEAD)
        P = np.stack([tb.tca_config_from_budget(b, 1.0, 0.57) for _ in range(Hq)])
        Qd, Kd, Vd = bufs.to_device(x["Q"]), bufs.to_device(x["K"]), bufs.to_device(x["V"])
        _, rows = tb.tca_select_rows(prm, L // b, P)
        gb = bufs.GlobalBuffers(prm, rows)
        ws_sel = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
        ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1])))
        q_last, O = Qd[:, L - 1].contiguous(), torch.empty_like(Qd)
        tb.tca_diag_prefill_clocks(True)

        def once():
            gb.n_rows.zero_()
            tb.tca_select(prm, q_last, Kd, Vd, L, 0, L, P, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws_sel)
            tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
            torch.cuda.synchronize()
            return tb.prefill_shader_clock_ghz(ws)
    elif args.what == "tail":
        # the last `queries` queries of the sequence with `heads` query heads: few workgroups of identical
        # work, below the power limit, in a forced workgroup shape
        Hq, d, L, b, w, n = args.heads, 128, 131072, 128, 4096, args.queries
        Hkv = max(1, Hq // 4)
        x = wl.prefill_inputs("lowrank", Hq, Hkv, d, L, "bf16", wl.data_seed(3))
        prm = tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16, 0.5, 0.0, tb.TCA_METRIC_HHI, tb.TCA_SHARE_HEAD)
        P = np.stack([tb.tca_config_from_budget(b, 1.0, 0.57) for _ in range(Hq)])
        Qd, Kd, Vd = bufs.to_device(x["Q"]), bufs.to_device(x["K"]), bufs.to_device(x["V"])
        _, rows = tb.tca_select_rows(prm, L // b, P)
        gb = bufs.GlobalBuffers(prm, rows)
        ws_sel = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
        tb.tca_select(prm, Qd[:, L - 1].contiguous(), Kd, Vd, L, 0, L, P, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws_sel)
        ws = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, n, int(gb.offs[-1])))
        Qc = Qd[:, L - n:].contiguous()
        O = torch.empty_like(Qc)
        tb.tca_diag_prefill_clocks(True)
        tb.tca_diag_prefill_variant(args.variant)

        def once():
            for _ in range(50):
                tb.tca_prefill(prm, Qc, L - n, n, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
            torch.cuda.synchronize()
            return tb.prefill_shader_clock_ghz(ws)
    else:
        wsp = bufs.workspace(tb.tca_probe_workspace_bytes())

        def once():
            return tb.tca_probe_mfma(args.what == "probe-random", 20000, wsp)
    once()
    t0, out = time.time(), []
    print(f"loop start {t0:.3f}", flush=True)
    while time.time() - t0 < args.seconds:
        out.append(once())
    t1 = time.time()
    if args.what in ("prefill", "tail"):
        per = 50 if args.what == "tail" else 1
        print(f"loop end {t1:.3f}: {len(out) * per} steps, {(t1 - t0) / (len(out) * per) * 1e3:.3f} ms per step, "
              f"shader clock {float(np.mean(out)):.2f} GHz", flush=True)
        tb.tca_diag_prefill_clocks(False)
        tb.tca_diag_prefill_variant(0)
    else:
        print(f"loop end {t1:.3f}: {len(out)} calls, {float(np.mean([o[0] for o in out])):.0f} TFLOP/s, "
              f"shader clock {float(np.mean([o[1] for o in out])):.2f} GHz", flush=True)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    o = sub.add_parser("occupancy")
    o.add_argument("--heads", type=int, nargs="+", default=[32, 16, 8])
    o.add_argument("--variants", type=int, nargs="+", default=[3], choices=[1, 2, 3])
    o.add_argument("--repeats", type=int, default=3)
    o.add_argument("--queries", type=int, default=2048, help="queries of the call: the last so many of the sequence")
    o.add_argument("--length", type=int, default=131072, help="tokens of the sequence")
    o.set_defaults(fn=occupancy)
    lp = sub.add_parser("loop")
    lp.add_argument("what", choices=["prefill", "tail", "probe-random", "probe-constant"])
    lp.add_argument("--seconds", type=float, default=10.0)
    lp.add_argument("--heads", type=int, default=8, help="tail: query heads (8 = a quarter of the chip)")
    lp.add_argument("--queries", type=int, default=2048, help="tail: queries of the call")
    lp.add_argument("--variant", type=int, default=3, choices=[1, 2, 3], help="tail: workgroup shape")
    lp.set_defaults(fn=loop)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
