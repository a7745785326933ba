"""Pins for the oracle's sink / TopK / union / gather steps (Algorithm 1) and
for the whole-path driver, by brute force and invariants.  CPU only."""

import numpy as np
import pytest

from oracle import curdkv_oracle as orc
from paper_2509_15038_amd import workloads as wl


def _brute(lt, k, s):
    """Selection by Python's sort with the (score desc, index asc) key."""
    n = len(lt)
    if k <= s:
        return list(range(k))
    cand = sorted(range(s, n), key=lambda j: (-lt[j], j))[: k - s]
    return sorted(list(range(s)) + cand)


@pytest.mark.parametrize("n,k,s", [(16, 5, 2), (16, 16, 4), (16, 0, 4), (16, 3, 4), (16, 4, 4),
                                   (33, 10, 0), (33, 11, 7), (5, 5, 9), (5, 2, 9), (1, 1, 0)])
def test_select_brute_force_with_planted_ties(n, k, s):
    rng = np.random.default_rng([n, k, s])
    lt = rng.integers(0, 4, size=n).astype(np.float64)     # many equal scores
    S = orc.select(lt, k, s)
    assert S.tolist() == _brute(lt.tolist(), k, s)
    assert len(S) == k and len(set(S.tolist())) == k
    assert np.all(np.diff(S) > 0)


def test_select_invariants_random():
    rng = np.random.default_rng(5)
    for _ in range(50):
        n = int(rng.integers(8, 200)); s = int(rng.integers(0, 8)); k = int(rng.integers(0, n + 1))
        lt = rng.random(n)
        S = orc.select(lt, k, s)
        assert len(S) == k
        assert set(range(min(s, k))) <= set(S.tolist())            # sinks kept first
        if k > s:
            kept = np.array([j for j in S if j >= s]); drop = np.setdiff1d(np.arange(s, n), kept)
            assert len(kept) == k - s
            if drop.size:
                assert lt[kept].min() >= lt[drop].max()             # top-k property
        assert S.tolist() == _brute(lt.tolist(), k, s)


def test_sink_scores_do_not_take_topk_slots():
    # huge scores inside the sink range must not be counted among the k - s picks
    lt = np.array([100., 90., 1., 5., 4., 3., 2.])
    assert orc.select(lt, 4, 2).tolist() == [0, 1, 3, 4]
    # and small sink scores are kept anyway
    lt = np.array([0., 0., 1., 5., 4., 3., 2.])
    assert orc.select(lt, 4, 2).tolist() == [0, 1, 3, 4]
    # the +s offset: without it the picks would be [0, 1, 1, 2]
    assert orc.select(lt, 3, 2).tolist() == [0, 1, 3]


def test_select_permutation_equivariance_beyond_sinks():
    rng = np.random.default_rng(6)
    n, s, k = 60, 4, 20
    lt = rng.random(n)                                # distinct with probability one
    p = np.concatenate([np.arange(s), s + rng.permutation(n - s)])
    S = orc.select(lt, k, s)
    Sp = orc.select(lt[p], k, s)
    assert sorted(p[Sp].tolist()) == S.tolist()


def test_select_rejects_bad_budgets():
    with pytest.raises(ValueError):
        orc.select(np.ones(4), 5, 0)
    with pytest.raises(ValueError):
        orc.select(np.ones(4), -1, 0)
    with pytest.raises(ValueError):
        orc.select(np.ones(4), 2, -1)


def test_compact_is_bitwise_row_gather():
    rng = np.random.default_rng(7)
    K = rng.integers(0, 65536, size=(40, 128)).astype(np.uint16)
    V = rng.integers(0, 65536, size=(40, 128)).astype(np.uint16)
    S = np.array([0, 3, 4, 17, 39])
    Kc, Vc = orc.compact(K, V, S)
    assert np.array_equal(Kc, np.take(K, S, axis=0)) and np.array_equal(Vc, np.take(V, S, axis=0))
    assert Kc.dtype == K.dtype and Kc.shape == (5, 128)


def test_compress_whole_path_small():
    cfg = wl.scaled(wl.CONFIGS["c2"], layers=2, kv_heads=2, n=300)
    K, V = wl.host_cache(cfg)
    b = np.array([60, 0, 300, 3], dtype=np.int32)
    lt, idx, off, Kp, Vp = orc.compress(K, V, cfg.dtype, cfg.sketch_seed, cfg.r, b, cfg.n_sink)
    assert off.tolist() == [0, 60, 60, 360, 363] and Kp.shape == (363, 128)
    assert np.allclose(lt.sum(-1), 1.0)
    assert idx[1].size == 0 and idx[2].tolist() == list(range(300)) and idx[3].tolist() == [0, 1, 2]
    assert np.array_equal(Kp[60:360], K[1, 0]) and np.array_equal(Vp[60:360], V[1, 0])
    # head (0,0): gathered rows are the original rows, in ascending token order
    assert np.array_equal(Kp[:60], K[0, 0][idx[0]]) and np.array_equal(Vp[:60], V[0, 0][idx[0]])
    # output is d-dimensional rows of the original cache, not r-dimensional projections
    assert Kp.shape[1] == cfg.d and cfg.r != cfg.d
    # each group gets its own sketch: scoring head (0,1) with head (0,0)'s G changes the scores
    G00 = orc.sketch(cfg.sketch_seed, 0, 0, 2, 128, cfg.r, "bf16")
    other = orc.scores(orc.to_f64(K[0, 1], "bf16"), orc.to_f64(V[0, 1], "bf16"), G00)
    assert not np.allclose(other, lt[0, 1], rtol=1e-6)


def test_high_norm_prefix_and_value_tail_drive_selection():
    # structure the synthetic caches are built to have: a x10 prefix block is mostly
    # kept (its score is x10^4; only rows whose value norm drew near zero drop out),
    # and heavy-tailed value rows are preferred
    cfg = wl.scaled(wl.CONFIGS["c4"], layers=1, kv_heads=1, n=2048)
    K, V = wl.host_head(cfg, 0, 0)
    G = orc.sketch(cfg.sketch_seed, 0, 0, 1, 128, cfg.r, "bf16")
    lt, S, _, _ = orc.compress_group(K, V, "bf16", G, 204, 4)
    assert len(set(range(64)) & set(S.tolist())) >= 56 and set(range(4)) <= set(S.tolist())
    vn = np.sum(orc.to_f64(V, "bf16") ** 2, axis=1)
    assert np.median(vn[S]) > 2 * np.median(vn)


def test_compress_ablation_variants_small():
    cfg = wl.scaled(wl.CONFIGS["c2"], layers=1, kv_heads=2, n=200)
    K, V = wl.host_cache(cfg)
    b = np.array([40, 40], dtype=np.int32)
    base = orc.compress(K, V, "bf16", cfg.sketch_seed, cfg.r, b, 4)
    for source in ("k", "v"):
        for projection in (True, False):
            lt, idx, off, Kp, Vp = orc.compress(K, V, "bf16", cfg.sketch_seed, cfg.r, b, 4, source, projection)
            assert np.allclose(lt.sum(-1), 1.0) and Kp.shape == (80, 128)
            assert not np.allclose(lt, base[0], rtol=1e-3)
            A = orc.to_f64(K[0, 1] if source == "k" else V[0, 1], "bf16")
            if not projection:
                rn = np.sum(A * A, axis=1)
                assert np.allclose(lt[0, 1], rn / rn.sum(), rtol=1e-12)
