"""The seeded input generator: determinism, independence of size and chunking,
distributions and the structure the workloads are meant to have. CPU only."""
import numpy as np
import torch

import tw_workloads as W


def f32(bits):
    return W.bf16_bits_to_f32(bits).astype(np.float64)


def test_same_seed_same_bits_and_prefix_property():
    a = W.normal_bf16((1000, 64), 0.5, 3, W.STREAM_RESIDUAL)
    b = W.normal_bf16((1000, 64), 0.5, 3, W.STREAM_RESIDUAL)
    assert np.array_equal(a, b)
    # counter-based: a shorter draw is a prefix of a longer one, whatever the shape
    c = W.normal_bf16((10, 64), 0.5, 3, W.STREAM_RESIDUAL)
    assert np.array_equal(a.reshape(-1)[:640], c.reshape(-1))
    big = W.normal_bf16(((1 << 21) + 4096,), 1.0, 0, 7)      # crosses the internal work-item size
    small = W.normal_bf16((5000,), 1.0, 0, 7)
    assert np.array_equal(big[:5000], small)


def test_seeds_and_streams_are_independent():
    a = f32(W.normal_bf16((4096,), 1.0, 0, 0))
    for other in (W.normal_bf16((4096,), 1.0, 1, 0), W.normal_bf16((4096,), 1.0, 0, 1)):
        o = f32(other)
        assert not np.array_equal(a, o)
        assert abs(np.corrcoef(a, o)[0, 1]) < 0.06


def test_normal_moments_and_tails():
    x = f32(W.normal_bf16((1 << 20,), 0.25, 5, W.STREAM_PARTIAL0))
    assert abs(x.mean()) < 1e-3
    assert abs(x.std() / 0.25 - 1.0) < 5e-3          # bf16 rounding adds < 1e-5 relative variance
    z = x / 0.25
    assert abs((np.abs(z) < 1).mean() - 0.6827) < 3e-3
    assert abs((np.abs(z) < 2).mean() - 0.9545) < 2e-3
    assert np.abs(z).max() < 6.5 and np.isfinite(x).all()


def test_uniform_range_and_mean():
    w = f32(W.uniform_bf16((1 << 18,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
    assert w.min() >= 0.5 and w.max() <= 1.5
    assert abs(w.mean() - 1.0) < 2e-3
    assert abs(w.var() - 1.0 / 12.0) < 1e-3


def test_outliers_have_the_stated_fraction_and_scale():
    base = f32(W.normal_bf16((1 << 20,), 1.0, 0, W.STREAM_RESIDUAL))
    out = f32(W.normal_bf16((1 << 20,), 1.0, 0, W.STREAM_RESIDUAL, outlier_frac=0.01, outlier_scale=50.0))
    changed = out != base
    assert abs(changed.mean() - 0.01) < 5e-4
    nz = changed & (base != 0)
    ratio = out[nz] / base[nz]
    assert np.all(np.abs(ratio - 50.0) < 50.0 * 2.0 ** -7)     # same draw, scaled before the one rounding
    assert np.array_equal(out[~changed], base[~changed])


def test_bf16_codec_matches_torch_and_roundtrips():
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 20000),
                        np.array([0.0, -0.0, np.inf, -np.inf, 1.0, 1.00390625, 1.01171875, 3.3895314e38],
                                 dtype=np.float32)])
    bits = W.f32_to_bf16_bits(v)
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    assert np.array_equal(W.f32_to_bf16_bits(W.bf16_bits_to_f32(bits)), bits)
    nan_bits = W.f32_to_bf16_bits(np.array([np.nan], dtype=np.float32))
    assert np.isnan(W.bf16_bits_to_f32(nan_bits))[0]


def test_configs_have_the_stated_shapes():
    want = {"c1_tiny": (64, 512, 2), "c2_8b_tp2": (2048, 4096, 2), "c3_70b_shard_tp8": (1024, 8192, 8),
            "c5_overlap_tp8": (4096, 8192, 8)}
    for name, (N, H, P) in want.items():
        c = W.CONFIGS[name]
        assert (c["N"], c["H"], c["P"]) == (N, H, P), name
    c4 = W.CONFIGS["c4_split_sweep_tp4"]
    assert (c4["H"], c4["P"]) == (8192, 4) and tuple(c4["N"]) == (256, 1024, 4096, 16384)
    assert tuple(c4["cu_budgets"]) == (16, 32, 64) and c4["split_multiple"] == 128
    g = W.CONFIGS["c5_overlap_tp8"]["gemm"]
    assert (g["M"], g["K"], g["N"], g["std"]) == (2048, 8192, 3584, 0.02)
    d = W.make_fused_inputs("c1_tiny")
    assert len(d["partials"]) == 2 and d["partials"][0].shape == (64, 512) and d["weight"].shape == (512,)
    assert d["partials"][0].dtype == np.uint16 and d["eps"] == 1e-6


def test_gemm_inputs_layouts_are_transposes_of_each_other():
    a = W.make_gemm_inputs(40, 64, 24, 0.3, seed=2, b_layout="nk")
    b = W.make_gemm_inputs(40, 64, 24, 0.3, seed=2, b_layout="kn")
    assert a["A"].shape == (40, 64) and a["B"].shape == (24, 64) and b["B"].shape == (64, 24)
    assert np.array_equal(a["A"], b["A"]) and np.array_equal(a["B"].T, b["B"])
