"""The C-ABI library loads, exports every symbol include/*.h declares, and
its host-side routines (no GPU) agree with the oracle and reject bad input."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import tca_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in ("tca.h", "tca_diag.h"):       # the method's boundary, and the diagnostics beside it
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(tca_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_the_boundary_header_holds_no_diagnostics():
    text = open(os.path.join(ROOT, "include", "tca.h")).read()
    assert "tca_probe" not in text and "tca_diag" not in text


def test_library_exports_every_declared_symbol():
    import paper_2512_09238_amd.binding as tb
    names = _declared_symbols()
    assert "tca_select" in names and "tca_prefill" in names and "tca_decode" in names
    assert "tca_calibrate_budgets" in names
    for n in names:
        assert hasattr(tb.lib, n), n
        assert n in tb.EXPORTS, f"{n} has no ctypes signature"
    assert set(tb.EXPORTS) == set(names)


def test_host_candidates_match_oracle():
    import paper_2512_09238_amd.binding as tb
    for b, M, sigma in [(128, 14, 1.0), (32, 5, 0.7), (4, 3, 1.0), (256, 1, 2.0)]:
        got = tb.tca_make_candidates(b, M, sigma)
        np.testing.assert_allclose(got, orc.candidates(b, M, sigma), rtol=1e-13, atol=1e-300)
    for f in (0.001, 0.05, 0.1, 0.25, 0.5, 0.7, 0.77, 0.99, 1.0, 1.5):
        for b in (32, 128):
            np.testing.assert_allclose(tb.tca_config_from_budget(b, 1.0, f), orc.config_from_budget(b, 1.0, f),
                                       rtol=1e-12, atol=1e-15)


def test_host_counts_rows_and_decode_budget_match_oracle():
    import paper_2512_09238_amd.binding as tb
    rng = np.random.default_rng(0)
    b = 128
    prm = tb.make_params(4, 2, 128, b, 512, tb.TCA_BF16)
    for m in (0, 1, 7, 256, 1024, 4096):
        P = np.stack([orc.config_from_budget(b, 1.0, f) for f in rng.uniform(0.02, 0.9, 4)])
        for p in P:
            assert list(tb.tca_psi_counts(b, m, p)) == list(orc.psi_counts(m, p))
            assert tb.tca_decode_budget(b, p) == orc.decode_budget(b, p)
        total, rows = tb.tca_select_rows(prm, m, P)
        assert list(rows) == [orc.selected_rows(b, m, p) for p in P] and total == rows.sum()
    assert list(tb.tca_psi_counts(2, 8, [0.25, 0.75])) == [2, 6]
    # a shared selection has one entry per KV head, and needs room for the logits of every query head
    shared = tb.make_params(4, 2, 128, b, 512, tb.TCA_BF16, share=tb.TCA_SHARE_GROUP)
    assert tb.tca_selection_heads(prm) == 4 and tb.tca_selection_heads(shared) == 2
    total, rows = tb.tca_select_rows(shared, 256, P[:2])
    assert list(rows) == [orc.selected_rows(b, 256, p) for p in P[:2]]
    assert tb.tca_select_workspace_bytes(shared, 4096) >= 4 * 4096 * 8


def test_argument_errors_are_codes_not_crashes():
    import paper_2512_09238_amd.binding as tb
    with pytest.raises(tb.TcaError) as e:
        tb.tca_num_counts(48)
    assert e.value.code == tb.TCA_ERR_UNSUPPORTED
    with pytest.raises(tb.TcaError) as e:
        tb.tca_psi_counts(4, 8, [0.5, 0.1, 0.1])
    assert e.value.code == tb.TCA_ERR_INVALID
    bad = tb.make_params(6, 4, 128, 128, 4096, tb.TCA_BF16)
    with pytest.raises(tb.TcaError):
        tb.tca_select_rows(bad, 4, np.ones((6, 8)) / 8)
    assert tb.tca_select_workspace_bytes(bad, 1024) == 0
    for prm in (tb.make_params(4, 2, 96, 128, 4096, tb.TCA_BF16), tb.make_params(4, 2, 128, 128, 100, tb.TCA_BF16),
                tb.make_params(4, 2, 128, 128, 4096, tb.TCA_BF16, 0.5, 0.0, 2),
                tb.make_params(4, 2, 128, 128, 4096, tb.TCA_BF16, 0.5, 0.0, 0, 2),
                tb.make_params(4, 2, 128, 128, 4096, 7), tb.make_params(256, 256, 128, 128, 4096, 0)):
        with pytest.raises(tb.TcaError):
            tb.tca_select_rows(prm, 4, np.ones((prm.n_q_heads, 8)) / 8)
    # NULL device pointers are rejected before any launch
    ok = tb.make_params(4, 2, 128, 128, 4096, tb.TCA_BF16)
    p = np.ones((4, 8)) / 8
    offs = np.arange(5, dtype=np.int64) * 10
    rc = tb.lib.tca_select(ctypes.byref(ok), None, None, None, 128, 0, 128, p.ctypes.data_as(tb._dbl_p),
                           offs.ctypes.data_as(tb._i64_p), None, None, None, None, None, 0, None)
    assert rc == tb.TCA_ERR_INVALID and b"NULL" in tb.lib.tca_last_error()
    assert tb.lib.tca_strerror(-3) == b"workspace too small or misaligned"
    assert tb.tca_select_workspace_bytes(ok, 131072) > 4 * 131072


def test_probe_rejects_bad_arguments_without_a_gpu():
    import paper_2512_09238_amd.binding as tb
    assert tb.tca_probe_workspace_bytes() >= 1024 * 24
    tf, ghz = ctypes.c_double(0), ctypes.c_double(0)
    rc = tb.lib.tca_probe_mfma(1, 100, ctypes.byref(tf), ctypes.byref(ghz), None, 0, None)
    assert rc == tb.TCA_ERR_INVALID
    rc = tb.lib.tca_probe_mfma(1, 100, None, None, ctypes.c_void_p(256), 1 << 20, None)
    assert rc == tb.TCA_ERR_INVALID
    rc = tb.lib.tca_probe_mfma(1, 0, ctypes.byref(tf), ctypes.byref(ghz), ctypes.c_void_p(256), 1 << 20, None)
    assert rc == tb.TCA_ERR_INVALID
    rc = tb.lib.tca_probe_mfma(1, 100, ctypes.byref(tf), ctypes.byref(ghz), ctypes.c_void_p(256), 16, None)
    assert rc == tb.TCA_ERR_WORKSPACE


def test_prefill_work_split_over_the_xcds():
    """Host logic of the bf16 prefill launch: the ranges the eight XCDs take cover the (head, query tile)
    sequence once, in order; equal regions with few long items per CU keep whole heads per XCD (an item
    more than the CUs divide would cost a whole round); unequal regions move the cuts towards the light
    heads; and the grid is eight times the longest range."""
    import paper_2512_09238_amd.binding as tb
    Hq, Hkv, d, b, w = 32, 8, 128, 128, 4096
    prm = tb.make_params(Hq, Hkv, d, b, w, tb.TCA_BF16, 0.5, 0.0)
    L = 131072
    n_qt = L // 256                                           # long calls: 256 queries per workgroup

    def check(start, n_wg, items):
        assert start[0] == 0 and start[8] == items and (np.diff(start) >= 0).all()
        assert n_wg == 8 * int(np.diff(start).max())

    # equal regions, the whole sequence: equal work is equal counts
    offs = np.arange(Hq + 1, dtype=np.int64) * 70000
    start, n_wg = tb.tca_diag_prefill_xcd_plan(prm, offs, 0, L)
    check(start, n_wg, Hq * n_qt)
    assert np.abs(np.diff(start) - 4 * n_qt).max() <= 1 and n_wg <= 8 * (4 * n_qt + 1)
    # the last 8192-token chunk of it: 1024 long items on 256 CUs, four rounds only if every XCD takes 128
    start, n_wg = tb.tca_diag_prefill_xcd_plan(prm, offs, L - 8192, 8192)
    check(start, n_wg, Hq * 32)
    assert np.array_equal(start, np.arange(9) * 128) and n_wg == 1024
    # regions from 5 % to 50 % of the sequence, heavy heads first: the first XCDs take fewer items
    rows = np.linspace(0.5, 0.05, Hq) * L
    offs = np.concatenate([[0], np.cumsum(rows.astype(np.int64))])
    start, n_wg = tb.tca_diag_prefill_xcd_plan(prm, offs, 0, L)
    check(start, n_wg, Hq * n_qt)
    counts = np.diff(start)
    assert counts[0] < 4 * n_qt < counts[7] and (np.diff(counts) >= 0).all()
    # the work of the ranges, recomputed here from the sizes: within a few per cent of each other
    def work(g):
        h, qt = g // n_qt, n_qt - 1 - g % n_qt
        last = qt * 256 + 255
        return 64 + 4 + (rows[h] * max(0, last - w + 1) / L) / 64
    per_xcd = [sum(work(g) for g in range(start[x], start[x + 1])) for x in range(8)]
    assert max(per_xcd) / min(per_xcd) < 1.05
    # a window-only part has no regions to weigh: equal counts again
    start, n_wg = tb.tca_diag_prefill_xcd_plan(prm, offs, 0, L, part=tb.TCA_PART_WINDOW)
    check(start, n_wg, Hq * n_qt)
    assert np.abs(np.diff(start) - 4 * n_qt).max() <= 2
    # short calls use 128 queries per workgroup; head counts that are no multiple of 8 have no plan
    start, n_wg = tb.tca_diag_prefill_xcd_plan(prm, np.arange(Hq + 1, dtype=np.int64) * 1000, 0, 4096)
    check(start, n_wg, Hq * 32)
    prm12 = tb.make_params(12, 4, d, b, w, tb.TCA_BF16, 0.5, 0.0)
    with pytest.raises(ValueError):
        tb.tca_diag_prefill_xcd_plan(prm12, np.arange(13, dtype=np.int64) * 1000, 0, 4096)


def test_binding_loads_torch_before_the_library():
    """One HIP runtime per process: the binding imports torch (which ships its own copy) before it
    loads libtca.so, whatever the caller imported first."""
    import subprocess
    import sys
    code = ("import sys; import paper_2512_09238_amd.binding as tb; "
            "assert 'torch' in sys.modules; print(tb.tca_num_counts(128))")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip() == "8", r.stderr[-500:]


def test_calibration_file_round_trip(tmp_path):
    """The calibrated configurations as a file: doubles come back bit for bit, a file made for
    another layer shape is refused."""
    import paper_2512_09238_amd.binding as tb
    import paper_2512_09238_amd.calibration as calib
    prm = tb.make_params(4, 2, 128, 128, 4096, tb.TCA_BF16)
    cands = tb.tca_make_candidates(128, 14, 1.0)
    pick = np.array([[3, 7, 7, 13], [0, 5, 6, 8]])
    cal = {"p_star": cands[pick], "cand_idx": pick.astype(np.int32), "fallback": np.array([[0, 0, 0, 1], [0, 0, 0, 0]], np.int32)}
    path = os.path.join(tmp_path, "c.json")
    calib.save_calibration(path, prm, cal, 14, 1.0, 0.9, 8192)
    back = calib.load_calibration(path, prm)
    assert np.array_equal(back["p_star"], cal["p_star"]) and back["p_star"].dtype == np.float64
    assert np.array_equal(back["cand_idx"], cal["cand_idx"]) and np.array_equal(back["fallback"], cal["fallback"])
    assert (back["n_layers"], back["n_selection_heads"], back["candidates"], back["calibration_tokens"]) == (2, 4, 14, 8192)
    one = {"p_star": cands[pick[0]], "cand_idx": pick[0].astype(np.int32), "fallback": np.zeros(4, np.int32)}
    calib.save_calibration(path, prm, one, 14, 1.0, 0.9, 8192)          # a single tca_calibrate_budgets result is one layer
    assert calib.load_calibration(path)["p_star"].shape == (1, 4, 8)
    with pytest.raises(ValueError):
        calib.load_calibration(path, tb.make_params(8, 2, 128, 128, 4096, tb.TCA_BF16))
    with open(path, "w") as f:
        f.write('{"format": "something else"}')
    with pytest.raises(ValueError):
        calib.load_calibration(path)


def test_bench_refuses_more_than_one_gpu():
    """Every box has one GPU: bench.py --gpus N with N above 1 ends with a message, before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout) or "1 GPU" in (r.stderr + r.stdout) or "--gpus" in (r.stderr + r.stdout)


def test_binding_fails_loudly_without_the_library(tmp_path):
    """The product path has no fallback: with no libtca.so to load, importing the binding raises."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2512_09238_amd"
    shutil.copytree(os.path.join(ROOT, "paper_2512_09238_amd"), pkg,
                    ignore=shutil.ignore_patterns("*.so", "_build", "__pycache__", "csrc"))
    code = "import paper_2512_09238_amd.binding"
    r = subprocess.run([sys.executable, "-c", code], cwd=tmp_path, capture_output=True, text=True, timeout=300,
                       env={**os.environ, "PYTHONPATH": str(tmp_path)})
    assert r.returncode != 0 and "libtca" in r.stderr
