"""The synthetic input generators: shapes, determinism, budget arithmetic.  CPU only."""

import numpy as np

from paper_2509_15038_amd import workloads as wl


def test_config_shapes():
    c = wl.CONFIGS
    assert (c["c1"].n, c["c1"].r, c["c1"].dtype) == (1024, 32, "fp32")
    assert (c["c2"].kv_heads, c["c2"].group, c["c2"].n, c["c2"].r) == (8, 4, 8192, 64)
    assert (c["c3"].layers, c["c3"].n) == (32, 32768) and c["c3"].keep == (0.10, 0.20, 0.50)
    assert c["c4"].prefix_rows == 64 and c["c4"].prefix_scale == 10.0
    assert (c["c5"].n, c["c5"].r) == (131072, 128)


def test_uniform_budgets():
    assert wl.budgets_for(wl.CONFIGS["c1"]).tolist() == [256]
    assert set(wl.budgets_for(wl.CONFIGS["c2"]).tolist()) == {1638}
    c3 = wl.CONFIGS["c3"]
    assert [int(wl.budgets_for(c3, f)[0]) for f in c3.keep] == [3276, 6553, 16384]
    assert wl.budgets_for(c3).size == 256


def test_dirichlet_budgets():
    c5 = wl.CONFIGS["c5"]
    b = wl.budgets_for(c5).reshape(32, 8)
    assert np.all(b.sum(1) == 52428) and b.min() >= 0 and b.max() <= c5.n
    assert np.array_equal(b.reshape(-1), wl.budgets_for(c5))            # deterministic
    assert len({tuple(x) for x in b.tolist()}) == 32                     # differs per layer
    o = wl.offsets_for(b.reshape(-1))
    assert o[0] == 0 and o[-1] == 32 * 52428 and np.all(np.diff(o) == b.reshape(-1))
    # clamping keeps the sum when a share would exceed n
    tiny = wl.scaled(c5, layers=3, n=1000, dirichlet_total_frac=0.9)
    bt = wl.budgets_for(tiny).reshape(3, 8)
    assert np.all(bt.sum(1) == 7200) and bt.max() <= 1000


def test_host_generators():
    c1 = wl.CONFIGS["c1"]
    K, V = wl.host_head(c1, 0, 0)
    assert K.dtype == np.float32 and K.shape == (1024, 128)
    K2, _ = wl.host_head(c1, 0, 0)
    assert np.array_equal(K, K2) and not np.array_equal(K, V)
    ch = np.sort(np.std(K, axis=0))
    assert ch[-4] > 4 * ch[-5]                       # four outlier channels
    c2 = wl.scaled(wl.CONFIGS["c2"], n=512)
    Kb, Vb = wl.host_head(c2, 0, 3)
    assert Kb.dtype == np.uint16 and Kb.shape == (512, 128)
    c4 = wl.scaled(wl.CONFIGS["c4"], n=512, layers=1, kv_heads=1)
    K4, V4 = wl.host_head(c4, 0, 0)
    f = lambda b: (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    rn = np.sum(f(K4) ** 2, axis=1)
    assert np.median(rn[:64]) > 50 * np.median(rn[64:])
    Kc, Vc = wl.host_cache(wl.scaled(wl.CONFIGS["c2"], n=64, kv_heads=2))
    assert Kc.shape == (1, 2, 64, 128)
