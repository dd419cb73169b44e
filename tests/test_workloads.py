"""Input generators: determinism, shapes, storage rounding (checked against
torch's own bfloat16 conversion, an independent implementation)."""
import numpy as np
import torch

import workloads as wl


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.00390625, 1.01171875]            # exact ties: round to even
    bits = wl.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = wl.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())
    assert np.array_equal(wl.to_f64(bits), back.astype(np.float64))


def test_prefill_inputs_seeded_and_shaped():
    c = wl.CONFIGS[1]
    a = wl.prefill_inputs(c["kind"], c["Hq"], c["Hkv"], c["d"], c["L"], c["dtype"], wl.data_seed(1))
    b = wl.prefill_inputs(c["kind"], c["Hq"], c["Hkv"], c["d"], c["L"], c["dtype"], wl.data_seed(1))
    assert a["Q"].shape == (4, 1024, 64) and a["K"].shape == (1, 1024, 64) and a["V"].shape == (1, 1024, 64)
    assert a["Q"].dtype == np.float32
    for k in ("Q", "K", "V"):
        assert np.array_equal(a[k], b[k])
    lr = wl.prefill_inputs("lowrank", 4, 2, 32, 512, "bf16", 7)
    assert lr["K"].dtype == np.uint16 and lr["K"].shape == (2, 512, 32)
    K = wl.to_f64(lr["K"])
    assert 0.5 < K.std() < 2.0
    f = wl.budget_fractions(wl.budget_seed(2), 32)
    assert f.shape == (32,) and f.min() >= 0.05 and f.max() <= 0.5


def test_compacted_cache_inputs():
    n = np.array([5, 0, 17, 9])
    c = wl.compacted_cache_inputs(4, 2, 16, 200, 32, 8, n, "bf16", 3)
    for h in range(4):
        assert len(c["idx"][h]) == n[h] and np.all(np.diff(c["idx"][h]) > 0)
        assert c["Kg"][h].shape == (n[h], 16)
    assert c["ringK"].shape == (2, 32, 16)
