"""The synthetic workload generator: shapes, determinism, storage rounding."""
import numpy as np
import pytest

from paper_2307_11339_amd import workloads as W


def test_bf16_rounding_matches_library_rne():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40], dtype=np.float32)])
    a = a.astype(np.float32)
    bits = W.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = W.bf16_bits_to_f32(bits)
    assert np.array_equal(W.f32_to_bf16_bits(back), bits)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.array([1.00390625], np.float32)))[0] == 1.0
    assert W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.array([1.01171875], np.float32)))[0] == 1.015625


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_named_configs_shapes_and_determinism(name):
    cfg = W.CONFIGS[name]
    if name in ("C3", "C4"):
        cfg = cfg.scaled(H=64, I=32, T=min(cfg.T, 16), len_min=4 if cfg.len_min else None)
    a = W.make_workload(cfg)
    b = W.make_workload(cfg)
    assert len(a.weights) == cfg.L * cfg.D * 4
    for l in range(cfg.L):
        for d in range(cfg.D):
            assert a.weight(l, d, 0).shape == (cfg.G * cfg.H, cfg.layer_input(l))
            assert a.weight(l, d, 1).shape == (cfg.G * cfg.H, cfg.H)
            assert a.weight(l, d, 2).shape == (cfg.G * cfg.H,)
    assert a.x.shape == (cfg.T, cfg.B, cfg.I)
    for u, v in zip(a.weights, b.weights):
        assert np.array_equal(u, v)
    assert np.array_equal(a.x, b.x)
    k = 1.0 / np.sqrt(cfg.H)
    assert max(np.abs(w).max() for w in a.weights) <= k * (1 + 2 ** -8)
    if cfg.dtype == W.BF16:
        for arr in a.weights + [a.x]:
            assert np.array_equal(W.bf16_bits_to_f32(W.f32_to_bf16_bits(arr)), arr)
    if cfg.len_min is not None:
        assert a.lengths.dtype == np.int32
        assert a.lengths.min() >= cfg.len_min and a.lengths.max() <= cfg.T
        for bb in range(cfg.B):
            assert np.all(a.x[a.lengths[bb]:, bb] == 0)
    if cfg.h0_std > 0:
        assert a.h0.shape == (cfg.L * cfg.D, cfg.B, cfg.H) and 0.05 < a.h0.std() < 0.2


def test_named_config_sizes():
    c = W.CONFIGS
    assert (c["C1"].cell, c["C1"].L, c["C1"].I, c["C1"].H, c["C1"].T, c["C1"].B, c["C1"].dtype) == (W.LSTM, 1, 64, 128, 32, 1, W.F32)
    assert (c["C2"].cell, c["C2"].L, c["C2"].I, c["C2"].H, c["C2"].T, c["C2"].B) == (W.GRU, 2, 256, 512, 100, 8)
    assert (c["C3"].L, c["C3"].I, c["C3"].H, c["C3"].T, c["C3"].B) == (4, 1024, 1024, 128, 1)
    assert (c["C4"].L, c["C4"].D, c["C4"].I, c["C4"].H, c["C4"].T, c["C4"].B, c["C4"].len_min) == (2, 2, 512, 512, 256, 64, 64)
    assert (c["C5"].L, c["C5"].I, c["C5"].H, c["C5"].T, c["C5"].B) == (8, 1024, 1024, 512, 256)
    grid = W.paper_grid()
    assert len(grid) == 13 and (grid[0].L, grid[0].B, grid[0].H, grid[0].T) == (12, 8, 64, 96)


def test_take_batch():
    cfg = W.CONFIGS["C4"].scaled(H=16, I=8, T=12, B=6, len_min=3)
    wl = W.make_workload(cfg)
    sub = wl.take_batch([4, 1])
    assert sub.cfg.B == 2 and np.array_equal(sub.x[:, 0], wl.x[:, 4]) and sub.lengths[1] == wl.lengths[1]
