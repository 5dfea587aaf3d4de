"""The seeded input recipe: shapes, value distributions and routing structure of the five named workloads
(checked on the configurations themselves where that takes milliseconds, on reduced T otherwise)."""
import numpy as np
import pytest

import workloads as wl


def small(name, T):
    return wl.CONFIGS[name].with_(T=T)


@pytest.mark.parametrize("name,T", [("tiny", 16), ("decode", 128), ("prefill", 512), ("skewed", 4096), ("wide", 2048)])
def test_shapes_dtypes_and_determinism(name, T):
    cfg = small(name, T)
    a, b = wl.make(cfg), wl.make(cfg)
    assert a.X.shape == (cfg.T, cfg.H) and a.K.shape == (cfg.T, cfg.k) and a.W.shape == (cfg.T, cfg.k)
    assert a.X.dtype == (np.uint16 if cfg.dtype == wl.DTYPE_BF16 else np.float32)
    assert a.K.dtype == np.int32 and a.W.dtype == np.float32 and a.scale.shape == (cfg.E,)
    for x, y in ((a.X, b.X), (a.K, b.K), (a.W, b.W), (a.scale, b.scale)):
        assert x.tobytes() == y.tobytes()                                   # same seed, same bits
    assert wl.make(cfg, seed=1).K.tobytes() != a.K.tobytes()
    # k distinct ids per token, all in range; gate weights are a softmax over the k picks
    assert np.all((a.K >= 0) & (a.K < cfg.E))
    assert all(len(set(row)) == cfg.k for row in a.K.tolist())
    assert np.all(a.W > 0) and np.allclose(a.W.sum(1), 1.0, atol=1e-6)
    # hidden states ~ N(0,1), rounded to the storage type
    xf = wl.bf16_bits_to_f32(a.X) if cfg.dtype == wl.DTYPE_BF16 else a.X
    assert abs(xf.mean()) < 0.02 and abs(xf.std() - 1.0) < 0.02


def test_payload_bytes_match_the_targets_table():
    want = {"tiny": 49152, "decode": 33030144, "prefill": 1056964608, "skewed": 4227858432, "wide": 4831838208}
    assert {n: c.payload_bytes for n, c in wl.CONFIGS.items()} == want
    w = wl.CONFIGS["wide"]
    assert w.N * w.H * w.elem_bytes == 2 ** 31                             # the wide window is exactly 2 GiB


def test_uniform_routing_is_balanced():
    cfg = small("prefill", 4096)
    counts = np.bincount(wl.make(cfg).K.reshape(-1), minlength=cfg.E)
    mean = cfg.N / cfg.E
    assert counts.min() > 0.6 * mean and counts.max() < 1.5 * mean


def test_zipf_routing_has_hot_experts():
    cfg = small("skewed", 4096)
    counts = np.bincount(wl.make(cfg).K.reshape(-1), minlength=cfg.E)
    mean = cfg.N / cfg.E
    assert counts.max() > 10 * mean                                         # hot experts get > 10x the mean load
    assert np.count_nonzero(counts > 10 * mean) >= 3 and np.median(counts) < mean
    assert counts.max() <= cfg.T                                            # without replacement: once per token at most


def test_group_limited_routing():
    cfg = small("wide", 2048)
    K = wl.make(cfg).K
    per_group = cfg.E // cfg.n_groups
    groups = K // per_group
    assert all(len(set(g)) <= cfg.groups_per_token for g in groups.tolist())    # experts from at most 4 of 8 groups
    counts = np.bincount(K.reshape(-1), minlength=cfg.E)
    mean = cfg.N / cfg.E
    assert counts.min() > 0.6 * mean and counts.max() < 1.5 * mean


def test_tiny_uses_index_scales_and_others_uniform():
    assert wl.make(wl.CONFIGS["tiny"]).scale.tolist() == list(range(1, 9))
    s = wl.make(small("decode", 8)).scale
    assert s.min() >= 0.5 and s.max() <= 1.5


def test_bf16_storage_conversion_round_trips():
    rng = np.random.default_rng(0)
    f = rng.standard_normal(10000).astype(np.float32)
    b = wl.f32_to_bf16_bits(f)
    back = wl.bf16_bits_to_f32(b)
    assert np.all(np.abs(back - f) <= np.abs(f) * 2.0 ** -8)
    assert np.array_equal(wl.f32_to_bf16_bits(back), b)


def test_adversarial_routing_generator():
    rng = np.random.default_rng(1)
    K = wl.random_routing(rng, 200, 6, 16, p_masked=0.2, p_invalid=0.1)
    flat = K.reshape(-1)
    assert np.any(flat == -1) and np.any((flat < -1) | (flat >= 16)) and np.any((flat >= 0) & (flat < 16))
