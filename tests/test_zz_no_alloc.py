"""tca_decode_static (the decode step on the library's own scratch array, for callers that
cannot allocate) against tca_decode on the same inputs: two calls in a row, the second on a
smaller input, then a call that does not fit."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def _filled_cache(tb, bufs, prm, B, n_rows, T0, seed):
    """A decode cache as it stands after T0 tokens: random rows at ascending random positions."""
    Hq, Hkv, d, w = prm.n_q_heads, prm.n_kv_heads, prm.head_dim, prm.window
    cache = bufs.DecodeCache(prm, B, n_rows + 8)
    g = torch.Generator(device="cuda").manual_seed(seed)
    rng = np.random.default_rng(seed)
    cache.Kg.copy_(torch.randn(cache.Kg.shape, generator=g, device="cuda", dtype=torch.float32))
    cache.Vg.copy_(torch.randn(cache.Vg.shape, generator=g, device="cuda", dtype=torch.float32))
    cache.ringK.copy_(torch.randn(cache.ringK.shape, generator=g, device="cuda", dtype=torch.float32))
    cache.ringV.copy_(torch.randn(cache.ringV.shape, generator=g, device="cuda", dtype=torch.float32))
    for s in range(B):
        for h in range(Hq):
            o = int(cache.offs[h])
            pos = np.sort(rng.choice(T0 - w, size=int(n_rows[h]), replace=False)).astype(np.int32)
            cache.idx[s, o:o + len(pos)] = torch.from_numpy(pos).cuda()
    cache.n_rows.copy_(torch.from_numpy(np.tile(n_rows.astype(np.int32), (B, 1))))
    cache.length.copy_(torch.from_numpy((T0 + rng.integers(0, prm.block, size=B)).astype(np.int64)))
    return cache


def _clone_cache(tb, bufs, prm, c):
    n = bufs.DecodeCache(prm, c.batch, np.diff(c.offs))
    for name in ("idx", "Kg", "Vg", "n_rows", "ringK", "ringV", "length"):
        getattr(n, name).copy_(getattr(c, name))
    return n


def _steps_agree(tb, bufs, prm, B, n_rows, T0, steps, seed, P):
    Hq, Hkv, d = prm.n_q_heads, prm.n_kv_heads, prm.head_dim
    ca = _filled_cache(tb, bufs, prm, B, n_rows, T0, seed)
    cb = _clone_cache(tb, bufs, prm, ca)
    dec = wl.decode_inputs(Hq, Hkv, d, steps, "bf16", seed + 1, batch=B)
    qd, kd, vd = (bufs.to_device(dec[k]) for k in ("q", "k_new", "v_new"))
    ws = bufs.workspace(tb.tca_decode_workspace_bytes(prm, B, ca.max_head_rows))
    Oa = torch.full((steps, B, Hq, d), float("nan"), dtype=qd.dtype, device="cuda")
    Ob = torch.full_like(Oa, float("nan"))
    for s in range(steps):
        tb.tca_decode(prm, ca.view, ca.offs, qd[s], kd[s], vd[s], P, Oa[s], ws)
        tb.tca_decode_static(prm, cb.view, cb.offs, qd[s], kd[s], vd[s], P, Ob[s])
    torch.cuda.synchronize()
    assert not torch.isnan(Ob.float()).any()
    # the same kernels on the same inputs: bit-identical outputs and caches
    assert torch.equal(Oa, Ob), f"outputs differ, max abs {(Oa.float() - Ob.float()).abs().max().item():.3e}"
    for name in ("idx", "Kg", "Vg", "n_rows", "ringK", "ringV", "length"):
        assert torch.equal(getattr(ca, name), getattr(cb, name)), name
    return Oa


def test_decode_static_matches_decode_twice_then_rejects_what_does_not_fit():
    import paper_2512_09238_amd.binding as tb
    import paper_2512_09238_amd.buffers as bufs
    b, w, d = 32, 128, 128
    prm = tb.make_params(8, 2, d, b, w, tb.TCA_BF16)
    fr = np.linspace(0.1, 0.6, 8)
    P = np.stack([tb.tca_config_from_budget(b, 1.0, f) for f in fr])
    # first call: batch 3, up to 2400 rows per head (several split-K slots), 40 steps: blocks complete on the way
    n_big = np.round(fr * 4000).astype(np.int64)
    print("static scratch: batch 3", flush=True)
    _steps_agree(tb, bufs, prm, 3, n_big, 6000, 40, 910, P)
    # second call, smaller: batch 1, a few hundred rows (the array still holds the first call's partials)
    n_small = np.round(fr * 500).astype(np.int64)
    print("static scratch: batch 1, smaller", flush=True)
    _steps_agree(tb, bufs, prm, 1, n_small, 900, 35, 911, P)
    # a step that needs more than the array holds is refused before anything is launched
    prm_big = tb.make_params(128, 16, d, b, w, tb.TCA_BF16)
    Pb = np.stack([tb.tca_config_from_budget(b, 1.0, 0.5)] * 128)
    rows = 40000
    assert tb.tca_decode_workspace_bytes(prm_big, 16, rows) > tb.TCA_DECODE_STATIC_BYTES
    offs = np.arange(129, dtype=np.int64) * rows
    dummy = torch.zeros(16, 128, d, dtype=torch.bfloat16, device="cuda")
    cache = tb.make_cache(16, int(offs[-1]), *([dummy] * 7))
    with pytest.raises(tb.TcaError) as e:
        tb.tca_decode_static(prm_big, cache, offs, dummy, dummy, dummy, Pb, dummy)
    assert e.value.code == tb.TCA_ERR_WORKSPACE
