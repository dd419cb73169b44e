"""GPU parity of the layer-integration pieces around the path (extensions): the Q / K / V
projections, rotary position embedding of Q / K rows, and Alg. 1 over several layers with its
results kept in a file."""
import os

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


def _storage_round(x64, dtype):
    """fp64 -> the storage type (round to nearest even) -> fp64, by the library's conversion."""
    t = torch.from_numpy(x64)
    return (t.to(torch.bfloat16) if dtype == "bf16" else t.to(torch.float32)).to(torch.float64).numpy()


ROPE_CASES = [
    # heads, rows, d, dtype, pos0, base, pairing
    (4, 300, 128, "bf16", 0, 10000.0, "half"),
    (3, 77, 64, "f32", 131072 - 77, 10000.0, "half"),          # the last rows of a 128K sequence
    (2, 1030, 128, "f32", 5, 500000.0, "interleaved"),         # Llama-3 base, more rows than one launch row-block
    (8, 5, 64, "bf16", 100000, 10000.0, "interleaved"),
]


@pytest.mark.parametrize("case", ROPE_CASES, ids=lambda c: f"h{c[0]}-n{c[1]}-d{c[2]}-{c[3]}-pos{c[4]}-{c[6]}")
def test_rope_matches_oracle(tb, bufs, case):
    """The rotation is computed in fp64 and rounded once, so the result is the oracle's rotation
    rounded to the storage type: equal to it, or one unit in the last place away where the two
    fp64 results straddle a rounding boundary."""
    nh, n, d, dtype, pos0, base, pairing = case
    print("case", case, flush=True)
    x = wl.prefill_inputs("lowrank", nh, nh, d, n, dtype, 81)["Q"]
    prm = H.params_for(tb, nh, nh, d, 16, 16, dtype)
    Xd = bufs.to_device(x)
    tb.tca_rope(prm, Xd, nh, n, pos0, base, tb.TCA_ROPE_HALF if pairing == "half" else tb.TCA_ROPE_INTERLEAVED)
    torch.cuda.synchronize()
    got = bufs.to_host_f64(Xd)
    ref = orc.rope_rotate(wl.to_f64(x), pos0 + np.arange(n), base=base, pairing=pairing)
    ref_r = _storage_round(ref, dtype)
    ulp = np.abs(ref_r) * (2.0 ** -7 if dtype == "bf16" else 2.0 ** -23) + 1e-30
    off = np.abs(got - ref_r)
    print("rows equal to the rounded oracle:", float((off == 0).mean()), "worst, in units of the last place:", float((off / ulp).max()), flush=True)
    assert np.all(off <= ulp)
    assert (off == 0).mean() > 0.999
    # norms survive up to the storage rounding
    np.testing.assert_allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(wl.to_f64(x), axis=-1),
                               rtol=2e-2 if dtype == "bf16" else 1e-6)


def test_rope_in_front_of_the_path(tb, bufs):
    """RoPE on Q and K, then select + prefill: the oracle rotates in fp64, rounds to bf16 as the
    library's output is, and runs the method on that."""
    Hq, Hkv, d, L, b, w = 4, 2, 128, 700, 32, 128
    x = wl.prefill_inputs("lowrank", Hq, Hkv, d, L, "bf16", 83)
    prm = H.params_for(tb, Hq, Hkv, d, b, w, "bf16")
    Qd, Kd, Vd = bufs.to_device(x["Q"]), bufs.to_device(x["K"]), bufs.to_device(x["V"])
    tb.tca_rope(prm, Qd, Hq, L, 0)
    tb.tca_rope(prm, Kd, Hkv, L, 0)
    P_gpu = np.stack([tb.tca_config_from_budget(b, 1.0, f) for f in (0.1, 0.2, 0.3, 0.5)])
    P_orc = np.stack([orc.config_from_budget(b, 1.0, f) for f in (0.1, 0.2, 0.3, 0.5)])
    _, rows = tb.tca_select_rows(prm, L // b, P_gpu)
    gb = bufs.GlobalBuffers(prm, rows)
    ws = bufs.workspace(max(tb.tca_select_workspace_bytes(prm, L), tb.tca_prefill_workspace_bytes(prm, L, int(gb.offs[-1]))))
    tb.tca_select(prm, Qd[:, L - 1].contiguous(), Kd, Vd, L, 0, L, P_gpu, gb.offs, gb.n_rows, gb.idx, gb.Kg, gb.Vg, ws)
    O = torch.full_like(Qd, float("nan"))
    tb.tca_prefill(prm, Qd, 0, L, Kd, Vd, L, gb.idx, gb.Kg, gb.Vg, gb.offs, gb.n_rows, O, None, ws)
    torch.cuda.synchronize()
    # the rotated inputs as the GPU holds them are what the oracle continues from (their parity is the test above)
    Qr, Kr = bufs.to_host_f64(Qd), bufs.to_host_f64(Kd)
    assert np.abs(Qr - _storage_round(orc.rope_rotate(wl.to_f64(x["Q"]), np.arange(L)), "bf16")).max() <= 0.25
    Oref, sels = orc.tca_prefill(Qr, Kr, wl.to_f64(x["V"]), b, w, P_orc, 0.5)
    for h in range(Hq):
        H.assert_selection(sels[h], H.head_indices(gb, h), b, P_orc[h], tag=f"head {h}")
    assert np.abs(bufs.to_host_f64(O) - Oref).max() <= H.TOL["bf16"]


def test_calibrate_layers_matches_oracle_and_survives_the_file(tb, bufs, tmp_path):
    import paper_2512_09238_amd.calibration as calib
    Hq, Hkv, d, L, b, M, nl = 4, 2, 64, 512, 16, 6, 3
    prm = H.params_for(tb, Hq, Hkv, d, b, b, "bf16")
    xs = [wl.prefill_inputs("lowrank", Hq, Hkv, d, L, "bf16", 90 + l) for l in range(nl)]
    Qs, Ks = [bufs.to_device(x["Q"]) for x in xs], [bufs.to_device(x["K"]) for x in xs]
    ws = bufs.workspace(tb.tca_calibrate_workspace_bytes(prm, L, M))
    tau = 0.9
    got = tb.tca_calibrate_layers(prm, Qs, Ks, L, M, 1.0, tau, ws)
    ref = orc.calibrate_layers([wl.to_f64(x["Q"]) for x in xs], [wl.to_f64(x["K"]) for x in xs], b, M, 1.0, tau, 0.5)
    assert got["p_star"].shape == (nl, Hq, tb.tca_num_counts(b))
    for l in range(nl):
        one = tb.tca_calibrate_budgets(prm, Qs[l], Ks[l], L, M, 1.0, tau, ws)     # the per-layer call gives the same
        assert np.array_equal(one["p_star"], got["p_star"][l]) and np.array_equal(one["a"], got["a"][l])
        for h in range(Hq):
            np.testing.assert_allclose(got["a"][l, h], ref[l][h].a, rtol=1e-9, atol=1e-12)
            assert np.array_equal(got["n"][l, h], ref[l][h].n)
            if np.min(np.abs(ref[l][h].a - tau)) > 1e-9:
                assert got["cand_idx"][l, h] == ref[l][h].index and bool(got["fallback"][l, h]) == ref[l][h].fallback
                np.testing.assert_allclose(got["p_star"][l, h], ref[l][h].p, rtol=1e-12, atol=1e-15)
    path = os.path.join(tmp_path, "model.tca.json")
    calib.save_calibration(path, prm, got, M, 1.0, tau, L)
    back = calib.load_calibration(path, prm)
    assert np.array_equal(back["p_star"], got["p_star"]) and np.array_equal(back["cand_idx"], got["cand_idx"])
    assert back["n_layers"] == nl and back["tau"] == tau
    # the loaded configurations drive selection exactly as the fresh ones
    x = xs[1]
    gb1, _, _, _ = H.gpu_select(tb, bufs, prm, x, got["p_star"][1])
    gb2, _, _, _ = H.gpu_select(tb, bufs, prm, x, back["p_star"][1])
    assert torch.equal(gb1.idx, gb2.idx) and torch.equal(gb1.n_rows, gb2.n_rows)
    with pytest.raises(ValueError):
        calib.load_calibration(path, H.params_for(tb, Hq, Hkv, d, 2 * b, 2 * b, "bf16"))
    with pytest.raises(tb.TcaError):
        tb.tca_calibrate_layers(prm, Qs, [Ks[0], None, Ks[2]], L, M, 1.0, tau, ws)


# ------------------------------------------------------------ Q / K / V projections --
QKV_CASES = [
    # Hq, Hkv, d, hidden, n, dtype, bias, layout, first row written
    (4, 2, 128, 192, 300, "bf16", True, "head", 5),       # three stages, ragged token tile, rows written at an offset
    (6, 2, 64, 64, 70, "bf16", True, "token", 0),         # one stage; 640 features: the last feature tile is half empty
    (8, 8, 128, 128, 1, "bf16", False, "token", 0),       # one row (a decode step), two stages
    (32, 8, 128, 512, 2100, "bf16", False, "head", 0),    # nine token tiles: more than one per XCD; 24 feature tiles
    (4, 4, 64, 1024, 257, "bf16", True, "head", 0),       # sixteen stages, one row into the second token tile
    (4, 1, 64, 100, 50, "f32", True, "head", 3),
    (2, 2, 128, 48, 9, "f32", False, "token", 0),
]


@pytest.mark.parametrize("case", QKV_CASES, ids=lambda c: f"hq{c[0]}-hkv{c[1]}-d{c[2]}-hid{c[3]}-n{c[4]}-{c[5]}-{c[7]}")
def test_qkv_project_matches_oracle(tb, bufs, case):
    """Every element of Q, K and V against the fp64 projections.  bf16: products are exact and the
    fp32 sum of `hidden` terms carries far less error than the one rounding to bf16, so the result
    is the oracle's value rounded to bf16, or its neighbour where the two sums straddle a rounding
    boundary: within 2^-8 relative (plus the sum's own error) everywhere."""
    Hq, Hkv, d, hidden, n, dtype, with_bias, layout, row0 = case
    print("case", case, flush=True)
    x = wl.projection_inputs(Hq, Hkv, d, hidden, n, dtype, 700 + hidden + n)
    prm = H.params_for(tb, Hq, Hkv, d, 16, 16, dtype)
    Xd, Wd = bufs.to_device(x["X"]), bufs.to_device(x["W"])
    bd = bufs.to_device(x["bias"]) if with_bias else None
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    cap = n + row0 + 3                                     # rows the output buffers hold
    if layout == "head":
        Q = torch.full((Hq, cap, d), float("nan"), dtype=tdt, device="cuda")
        K = torch.full((Hkv, cap, d), float("nan"), dtype=tdt, device="cuda")
        V = torch.full((Hkv, cap, d), float("nan"), dtype=tdt, device="cuda")
        at = lambda T: T.data_ptr() + row0 * d * T.element_size()      # row `row0` of head 0
        tb.tca_qkv_project(prm, Xd, n, hidden, Wd, bd, at(Q), d, cap * d, at(K), at(V), d, cap * d)
        take = lambda T: T[:, row0:row0 + n].double().cpu().numpy()
        rest = lambda T: torch.cat([T[:, :row0], T[:, row0 + n:]], dim=1)
    else:
        Q = torch.full((cap, Hq, d), float("nan"), dtype=tdt, device="cuda")
        K = torch.full((cap, Hkv, d), float("nan"), dtype=tdt, device="cuda")
        V = torch.full((cap, Hkv, d), float("nan"), dtype=tdt, device="cuda")
        tb.tca_qkv_project(prm, Xd, n, hidden, Wd, bd, Q[row0:], Hq * d, d, K[row0:], V[row0:], Hkv * d, d)
        take = lambda T: T[row0:row0 + n].permute(1, 0, 2).double().cpu().numpy()
        rest = lambda T: torch.cat([T[:row0], T[row0 + n:]], dim=0)
    torch.cuda.synchronize()
    ref = orc.qkv_project(wl.to_f64(x["X"]), wl.to_f64(x["W"]), Hq, Hkv, d,
                          bias=wl.to_f64(x["bias"]) if with_bias else None)
    worst_rel, equal = 0.0, []
    for name, got_t, r in zip("QKV", (Q, K, V), ref):
        got = take(got_t)
        assert not np.isnan(got).any(), f"{name}: an element was never written"
        assert torch.isnan(rest(got_t)).all(), f"{name}: a row outside the call's range was written"
        err = np.abs(got - r)
        if dtype == "bf16":
            bound = 2.0 ** -8 * np.abs(r) + 1e-4
            equal.append(float((got == _storage_round(r, dtype)).mean()))
        else:
            bound = 1e-4 * np.maximum(1.0, np.abs(r))
        worst_rel = max(worst_rel, float((err / bound).max()))
        assert (err <= bound).all(), f"{name}: worst error {err.max()} at {np.unravel_index(err.argmax(), err.shape)}"
        assert err.max() <= H.TOL[dtype]
    print("worst error in units of the bound:", worst_rel, "share equal to the rounded oracle:", equal, flush=True)
    if dtype == "bf16":
        assert min(equal) > 0.99


def _draw_projection(rng):
    G, Hkv = int(rng.integers(1, 9)), int(rng.integers(1, 5))
    d = int(rng.choice([64, 128]))
    dtype = str(rng.choice(["bf16", "bf16", "f32"]))
    hidden = 64 * int(rng.integers(1, 13)) if dtype == "bf16" else int(rng.integers(3, 200))
    n = int(rng.integers(1, 1300)) if dtype == "bf16" else int(rng.integers(1, 80))
    return G * Hkv, Hkv, d, hidden, n, dtype, bool(rng.integers(0, 2)), str(rng.choice(["head", "token"])), int(rng.integers(0, 5))


@pytest.mark.parametrize("case", [_draw_projection(np.random.default_rng(4100 + i)) for i in range(16)],
                         ids=lambda c: f"hq{c[0]}-hkv{c[1]}-d{c[2]}-hid{c[3]}-n{c[4]}-{c[5]}-{c[7]}")
def test_qkv_project_random_shapes(tb, bufs, case):
    """A seeded sweep: every group size 1..8, both head dims, one to twelve stages, one to six token
    tiles with ragged ends, feature counts that leave the last feature tile a quarter to full."""
    test_qkv_project_matches_oracle(tb, bufs, case)


def test_qkv_project_refuses_what_it_cannot_do(tb, bufs):
    prm = H.params_for(tb, 4, 2, 128, 16, 16, "bf16")
    x = wl.projection_inputs(4, 2, 128, 96, 8, "bf16", 5)
    Xd, Wd = bufs.to_device(x["X"]), bufs.to_device(x["W"])
    Q = torch.zeros(4, 8, 128, dtype=torch.bfloat16, device="cuda")
    K, V = torch.zeros(2, 8, 128, dtype=torch.bfloat16, device="cuda"), torch.zeros(2, 8, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(tb.TcaError, match="multiple of 64"):
        tb.tca_qkv_project(prm, Xd, 8, 96, Wd, None, Q, 128, 8 * 128, K, V, 128, 8 * 128)
    with pytest.raises(tb.TcaError, match="stride"):
        tb.tca_qkv_project(prm, Xd, 8, 64, Wd, None, Q, 64, 8 * 128, K, V, 128, 8 * 128)
    with pytest.raises(tb.TcaError, match="multiples of 4"):
        tb.tca_qkv_project(prm, Xd, 8, 64, Wd, None, Q, 130, 8 * 130, K, V, 128, 8 * 128)
    tb.tca_qkv_project(prm, Xd, 0, 64, Wd, None, Q, 128, 8 * 128, K, V, 128, 8 * 128)      # nothing to do
    torch.cuda.synchronize()
    assert float(Q.abs().sum()) == 0.0
