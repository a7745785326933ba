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


def test_attention_output_brute_force_and_one_hot():
    import math
    rng = np.random.default_rng(4)
    m, n, d = 3, 5, 4
    Q, K, V = rng.standard_normal((m, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    want = np.zeros((m, d))
    for i in range(m):
        w = [math.exp(sum(Q[i, c] * K[j, c] for c in range(d)) / math.sqrt(d)) for j in range(n)]
        for j in range(n):
            for c in range(d):
                want[i, c] += w[j] / sum(w) * V[j, c]
    assert np.allclose(ev.attention_output(Q, K, V), want, rtol=1e-12)
    # a query that matches one key overwhelmingly returns that token's value row
    K = np.eye(4)[[0, 1, 2, 3, 0]] * 1.0
    K[4] = 0.0
    V = rng.standard_normal((5, 4)) * 3.0
    out = ev.attention_output(200.0 * np.eye(4)[[2]], K, V)
    assert np.allclose(out[0], V[2], atol=1e-9)
    # evicting a token no query attends to costs nothing; evicting the attended one does
    Qh = 200.0 * np.eye(4)[[2]]
    assert ev.eviction_loss(Qh, K, V, np.array([0, 1, 2, 3])) < 1e-9
    assert ev.eviction_loss(Qh, K, V, np.array([0, 1, 3, 4])) > 1.0


def test_policy_comparison_harness():
    # the harness itself: every policy keeps k tokens with the sinks, costs nothing at k = n,
    # and (averaged over heads) loses less the more it keeps.  No claim about which policy
    # wins on synthetic queries is made or tested.
    rng = np.random.default_rng(5)
    losses = {}
    for seed in range(4):
        K, V = _head(200 + seed, 512)
        n = K.shape[0]
        G = orc.sketch(6, seed, 0, 1, 128, 32, "bf16")
        lt = orc.scores(K, V, G)
        Q = K[rng.choice(n, 16, replace=False)] * 0.5 + rng.standard_normal((16, 128)) * 0.5   # queries near some keys
        for k in (32, 128, 384, n):
            sets = ev.selection_policies(K, V, lt, k, 4, rng)
            for name, S in sets.items():
                assert S.shape == (k,) and np.all(np.diff(S) > 0) and np.array_equal(S[:4], np.arange(4)), name
            assert np.array_equal(sets["curdkv"], orc.select(lt, k, 4))
            for name, loss in ev.compare_policies(Q, K, V, lt, k, 4, rng).items():
                losses.setdefault((name, k), []).append(loss)
                if k == n:
                    assert loss < 1e-9
    for name in ("curdkv", "key_norm", "value_norm", "random"):
        mean = [np.mean(losses[(name, k)]) for k in (32, 128, 384, 512)]
        assert mean[0] > mean[2] > mean[3], (name, mean)
