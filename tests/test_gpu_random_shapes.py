"""Seeded sweep over small random shapes: selection sets, prefill outputs and a few decode
steps of the GPU path against the oracle, every row.  Shapes cover both head dims, every
group size 1..8, blocks 2..256, windows of 1..8 blocks, ragged lengths, both storage types.
A second sweep runs other shapes with one selection per KV head (tca_params.share).  Every case
also runs the gather-free prefill, the window and global parts merged through the log-sum-exp,
and, for bf16, the decode steps on an FP8 cache."""
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
    return tb, bufs


def _draw(rng):
    G = int(rng.integers(1, 9))
    Hkv = int(rng.integers(1, 4))
    d = int(rng.choice([64, 128]))
    b = int(2 ** rng.integers(1, 9))
    w = b * int(rng.integers(1, 9))
    L = int(rng.integers(max(b, 8), 6 * w + 3 * b + 50))
    dtype = str(rng.choice(["bf16", "f32"]))
    kind = str(rng.choice(["lowrank", "centroid"]))
    return kind, G * Hkv, Hkv, d, min(L, 1400), dtype, b, w


CASES = [(_draw(np.random.default_rng(900 + i)), 900 + i) for i in range(48)]


SHARED_CASES = [(_draw(np.random.default_rng(1900 + i)), 1900 + i) for i in range(32)]


@pytest.mark.parametrize("case,seed", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_random_shape_select_prefill_decode(mods, case, seed):
    run_case(mods, case, seed, share=False)


@pytest.mark.parametrize("case,seed", SHARED_CASES, ids=lambda v: str(v).replace(" ", ""))
def test_random_shape_shared_selection(mods, case, seed):
    run_case(mods, case, seed, share=True)


def run_case(mods, case, seed, share):
    tb, bufs = mods
    kind, Hq, Hkv, d, L, dtype, b, w = case
    print("case", case, "seed", seed, "share", share, flush=True)
    rng = np.random.default_rng(seed)
    x = wl.prefill_inputs(kind, Hq, Hkv, d, L, dtype, seed)
    Hs = Hkv if share else Hq
    GS = Hq // Hs
    fr = rng.uniform(0.03, 0.97, size=Hs)
    P_gpu = np.stack([tb.tca_config_from_budget(b, 1.0, f) for f in fr])
    P_orc = np.stack([orc.config_from_budget(b, 1.0, f) for f in fr])
    prm = H.params_for(tb, Hq, Hkv, d, b, w, dtype, share=share)
    steps = int(min(2 * b + 3, 40))
    _, rows = tb.tca_select_rows(prm, L // b, P_gpu)
    extra = np.array([tb.tca_decode_budget(b, p) for p in P_gpu]) * ((L + steps) // b - L // b + 1)
    cache = bufs.DecodeCache(prm, 1, rows + extra)
    Kd, Vd, Qd = bufs.to_device(x["K"]), bufs.to_device(x["V"]), bufs.to_device(x["Q"])
    ws = bufs.workspace(tb.tca_select_workspace_bytes(prm, L))
    tb.tca_select(prm, Qd[:, L - 1].contiguous(), Kd, Vd, L, 0, L, P_gpu, cache.offs, cache.n_rows[0],
                  cache.idx[0], cache.Kg[0], cache.Vg[0], ws)
    O = torch.full_like(Qd, float("nan"))
    wsp = bufs.workspace(tb.tca_prefill_workspace_bytes(prm, L, int(cache.offs[-1])))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, cache.idx[0], cache.Kg[0], cache.Vg[0], cache.offs, cache.n_rows[0],
                   O, None, wsp)
    tb.tca_cache_load_window(prm, cache.view, 0, Kd, Vd, L, L)
    torch.cuda.synchronize()

    Qf, Kf, Vf = wl.to_f64(x["Q"]), wl.to_f64(x["K"]), wl.to_f64(x["V"])
    Oref, sels = orc.tca_prefill(Qf, Kf, Vf, b, w, P_orc, 0.5, share=share)
    exact = True
    for n_ in range(Hs):
        o, n = int(cache.offs[n_]), int(cache.n_rows[0, n_].item())
        got = cache.idx[0, o:o + n].cpu().numpy().astype(np.int64)
        if not H.assert_selection(sels[n_], got, b, P_orc[n_], tag=f"selection head {n_}"):
            exact = False
            for h in range(n_ * GS, (n_ + 1) * GS):
                Oref[h] = orc.tca_attention(Qf[h], Kf[h // (Hq // Hkv)], Vf[h // (Hq // Hkv)], got, w)
    Og = bufs.to_host_f64(O)
    assert not np.isnan(Og).any()
    err = np.abs(Og - Oref).max()
    assert err <= H.TOL[dtype], f"prefill max abs err {err}"

    # the switches on the same shape.  Gather-free: the kept rows read through idx, bit for bit the
    # output of the call on the compacted rows.
    O2 = torch.full_like(Qd, float("nan"))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, cache.idx[0], None, None, cache.offs, cache.n_rows[0], O2, None, wsp)
    torch.cuda.synchronize()
    assert torch.equal(O2, O), "gather-free output differs"
    # Window part and global part on their own, merged through the log-sum-exp: Eq. 2 again, up to the
    # rounding of the two partial outputs to the storage type (half a unit in the last place of a
    # part each, on top of the tolerance of the one-pass kernel).
    O_w, O_g = torch.full_like(Qd, float("nan")), torch.full_like(Qd, float("nan"))
    lse2 = torch.full((2, Hq, L), float("nan"), dtype=torch.float32, device="cuda")
    tb.tca_prefill_part(prm, tb.TCA_PART_WINDOW, Qd, 0, L, Kd, Vd, L, cache.idx[0], cache.Kg[0], cache.Vg[0], cache.offs,
                        cache.n_rows[0], O_w, lse2[0], wsp)
    tb.tca_prefill_part(prm, tb.TCA_PART_GLOBAL, Qd, 0, L, Kd, Vd, L, cache.idx[0], cache.Kg[0], cache.Vg[0], cache.offs,
                        cache.n_rows[0], O_g, lse2[1], wsp)
    tb.tca_prefill_merge(prm, L, O_w, lse2[0], O_g, lse2[1], None)
    torch.cuda.synchronize()
    Om = bufs.to_host_f64(O_w)
    assert not np.isnan(Om).any()
    slack = 0.0 if dtype == "f32" else 2.0 ** -8 * max(1.0, float(np.abs(Oref).max()))
    err_m = np.abs(Om - Oref).max()
    assert err_m <= H.TOL[dtype] + slack, f"merged parts max abs err {err_m}"

    if not exact:
        return                                   # a sub-margin tie: the decode replay below needs identical sets
    ocache = orc.cache_after_prefill(Kf, Vf, sels)
    dec = wl.decode_inputs(Hq, Hkv, d, steps, dtype, seed + 2, batch=1, gains=x["gains"])
    qd, kd, vd = (bufs.to_device(dec[k]) for k in ("q", "k_new", "v_new"))
    wsd = bufs.workspace(tb.tca_decode_workspace_bytes(prm, 1, cache.max_head_rows))
    Od = torch.full((steps, 1, Hq, d), float("nan"), dtype=qd.dtype, device="cuda")
    for s in range(steps):
        tb.tca_decode(prm, cache.view, cache.offs, qd[s], kd[s], vd[s], P_gpu, Od[s], wsd)
    torch.cuda.synchronize()
    Odg = bufs.to_host_f64(Od)
    worst = 0.0
    for s in range(steps):
        ref = orc.decode_step(ocache, wl.to_f64(dec["q"][s, 0]), wl.to_f64(dec["k_new"][s, 0]),
                              wl.to_f64(dec["v_new"][s, 0]), b, w, P_orc, share=share)
        worst = max(worst, np.abs(Odg[s, 0] - ref).max())
    assert worst <= H.TOL[dtype], f"decode max abs err {worst}"
    for h in range(Hs):
        o, n = int(cache.offs[h]), int(cache.n_rows[0, h].item())
        assert np.array_equal(cache.idx[0, o:o + n].cpu().numpy(), ocache.S[h]), f"head {h} after decode"

    if dtype != "bf16":
        return
    # the same steps on an FP8 cache (codes and one scale per row), against the oracle reading the
    # rows back through the same quantisation
    gbs = bufs.GlobalBuffers(prm, rows + extra)
    tb.tca_select(prm, Qd[:, L - 1].contiguous(), Kd, Vd, L, 0, L, P_gpu, gbs.offs, gbs.n_rows, gbs.idx, gbs.Kg, gbs.Vg, ws)
    c8 = bufs.DecodeCache(prm, 1, rows + extra, kv_format=tb.TCA_KV_FP8)
    tb.tca_cache_load_global(prm, c8.view, 0, gbs.idx, gbs.Kg, gbs.Vg, gbs.offs, gbs.n_rows)
    tb.tca_cache_load_window(prm, c8.view, 0, Kd, Vd, L, L)
    o8 = orc.cache_after_prefill(Kf, Vf, sels, kv_quant="fp8")
    Od.fill_(float("nan"))
    for s in range(steps):
        tb.tca_decode(prm, c8.view, c8.offs, qd[s], kd[s], vd[s], P_gpu, Od[s], wsd)
    torch.cuda.synchronize()
    Odg = bufs.to_host_f64(Od)
    worst = 0.0
    for s in range(steps):
        ref = orc.decode_step(o8, wl.to_f64(dec["q"][s, 0]), wl.to_f64(dec["k_new"][s, 0]),
                              wl.to_f64(dec["v_new"][s, 0]), b, w, P_orc, share=share, kv_quant="fp8")
        worst = max(worst, np.abs(Odg[s, 0] - ref).max())
    assert worst <= H.TOL[dtype], f"fp8 cache decode max abs err {worst}"
    for h in range(Hs):
        o, n = int(c8.offs[h]), int(c8.n_rows[0, h].item())
        assert np.array_equal(c8.idx[0, o:o + n].cpu().numpy(), o8.S[h]), f"head {h} after decode on the fp8 cache"
