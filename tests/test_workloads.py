"""The seeded input generators: reproducible, right shapes and laws (no GPU)."""
import numpy as np

import workloads as W


def test_splitmix64_first_values():
    """Stream 0 of the public splitmix64 generator starts 0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4."""
    v = W.splitmix64(0, np.arange(2))
    assert int(v[0]) == 0xE220A8397B1DCDAF and int(v[1]) == 0x6E789E6AA1B965F4


def test_streams_are_counter_based():
    a = W.uniform01(5, 100)
    b = W.uniform01(5, 10)
    np.testing.assert_array_equal(a[:10], b)
    assert 0 < a.min() and a.max() < 1


def test_normal_moments_and_softmax():
    z = W.normal(3, 200000, sigma=np.sqrt(2.0))
    assert abs(z.mean()) < 0.02 and abs(z.var() - 2.0) < 0.03
    p = W.softmax_rows(z[:1000].reshape(100, 10))
    assert p.dtype == np.float32 and np.allclose(p.sum(1), 1, atol=1e-6) and p.min() > 0


def test_beta22_moments():
    x = W.beta22(1, 100000)
    assert x.dtype == np.float32 and abs(x.mean() - 0.5) < 0.005 and abs(x.var() - 0.05) < 0.002


def test_config_shapes():
    w = W.config1()
    assert w["pa"].shape == (64, 10) and w["table"].shape == (10, 10) and w["table"].max() == 18
    w = W.config2(batch=32)
    assert w["p"].shape == (15, 32, 10) and 0 <= w["target"].min() and w["target"].max() <= 135
    w = W.config3(batch=16)
    assert w["table"].shape == (64, 64) and 0 <= w["table"].min() and w["table"].max() <= 255
    assert w["keep"].shape == (256,) and 96 < w["keep"].sum() < 160
    w = W.config4(batch=8)
    assert w["fact_prob"].shape == (8, 50) and list(w["fact_group"][:11]) == [0] * 10 + [1]
    np.testing.assert_array_equal(w["fact_prob"][:, 10:20], w["p"][1])
    w = W.config5(batch=2)
    assert w["p"].shape == (2, 1984) and w["tri_i"].size == 2 * 1984 + 1024
    key = w["tri_i"].astype(np.int64) * 4096 + w["tri_j"]
    assert np.all(np.diff(key) > 0)


def test_seed_changes_data_and_same_seed_repeats():
    a, b, c = W.config1(seed=0), W.config1(seed=0), W.config1(seed=1)
    np.testing.assert_array_equal(a["pa"], b["pa"])
    assert not np.array_equal(a["pa"], c["pa"])
