"""What the selection is for: eviction loss on synthetic queries and the bound of
Lemma 1 (Section 3.1).  CPU only; uses the oracle's selection."""

import numpy as np

from oracle import curdkv_oracle as orc
from oracle import eviction_eval as ev
from paper_2509_15038_amd import workloads as wl


def _head(seed, n=1024):
    cfg = wl.scaled(wl.CONFIGS["c2"], kv_heads=1, n=n)
    K, V = wl.host_head(cfg, seed, 0)
    return orc.to_f64(K, "bf16"), orc.to_f64(V, "bf16")


def test_lemma1_bound_holds():
    rng = np.random.default_rng(1)
    for seed in range(4):
        K, V = _head(seed, 256)
        Q = rng.standard_normal((32, 128)) * 0.3
        for k in (16, 64, 200):
            S = np.sort(rng.choice(256, size=k, replace=False))
            lhs, rhs = ev.lemma1_sides(Q, K, V, S)
            assert lhs <= rhs
        lhs, rhs = ev.lemma1_sides(Q, K, V, np.arange(256))        # nothing evicted
        assert lhs < 1e-9 and rhs > 0


def test_softmax_and_full_selection():
    rng = np.random.default_rng(2)
    K, V = _head(9, 128)
    Q = rng.standard_normal((8, 128))
    P = ev.softmax_rows(Q @ K.T)
    assert np.allclose(P.sum(1), 1.0) and np.all(P >= 0)
    assert ev.eviction_loss(Q, K, V, np.arange(128)) < 1e-10


def test_value_guided_selection_shrinks_the_lemma1_term():
    # Lemma 1 bounds the loss by sqrt(n) ||V - V'||_F + ...: a value-guided selection keeps
    # that first term well below what as many random tokens would (heavy-tailed value norms)
    rng = np.random.default_rng(3)
    for seed in range(6):
        K, V = _head(100 + seed)
        n = K.shape[0]
        G = orc.sketch(5, seed, 0, 1, 128, 64, "bf16")
        S = orc.select(orc.scores(K, V, G), n // 10, 4)
        vn = np.sum(V * V, axis=1)
        kept = vn[S].sum() / vn.sum()                       # share of ||V||_F^2 retained
        assert kept > 0.3                                   # random keeps 0.1 on average
        dropped = np.sqrt(vn.sum() - vn[S].sum())           # ||V - V'||_F
        rnd = np.mean([np.sqrt(vn.sum() - vn[rng.choice(n, n // 10, replace=False)].sum())
                       for _ in range(5)])
        assert dropped < 0.9 * rnd
        # value-only scores retain at least as much value mass as the key-value product
        Sv = orc.select(orc.scores(K, V, G, source="v"), n // 10, 4)
        assert vn[Sv].sum() >= vn[S].sum() * 0.999
