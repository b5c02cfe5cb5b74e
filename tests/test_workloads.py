"""The input generators: shapes, determinism and bf16 rounding (no method arithmetic here)."""
import numpy as np
import torch

import hbp_workloads as wl


def test_length_recipes_are_deterministic_and_fill_the_pack():
    for idx, pack_len in [(2, 8192), (3, 32768), (5, 32768)]:
        w = wl.workload(idx)
        assert w == wl.workload(idx)
        assert sum(w.lengths) >= pack_len and sum(w.lengths[:-1]) < pack_len
    assert wl.workload(3).lengths[0] == 16384
    assert wl.workload(1).lengths == (512, 256, 128, 64, 64)
    assert wl.workload(4).lengths == (98304, 32768)
    w2 = wl.workload(2)
    assert min(w2.lengths) >= 16 and max(w2.lengths) <= 4096


def test_bf16_rounding_matches_torch_rne():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.0, np.float32(1.0 + 2.0**-8)]     # a tie: rounds to even
    bits = wl.f32_to_bf16_bits(x)
    want = torch.tensor(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    back = wl.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.tensor(x).to(torch.bfloat16).float().numpy())


def test_heads_regenerate_independently():
    full = wl.tensor_bits(0, "k", 50, 4, 16)
    part = wl.tensor_bits(0, "k", 50, 4, 16, heads=[2])
    assert np.array_equal(full[:, 2], part[:, 0])
    assert not np.array_equal(full[:, 1], full[:, 2])
    assert not np.array_equal(wl.tensor_bits(0, "q", 50, 4, 16), full)
