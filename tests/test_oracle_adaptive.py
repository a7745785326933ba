"""Pins for the oracle's AdaCurDKV budget allocation (Section 3.2, "Adaptive
budget allocation"): invariants, limiting cases and an independent construction
(boost every head's safe tokens, then one layer-wide sort).  CPU only."""

import numpy as np
import pytest

from oracle import curdkv_oracle as orc


def _boost_and_sort(lt, k, s, alpha):
    """AdaKV's description, built differently: give the sinks and each head's
    top floor(alpha*k) tokens an unbeatable score, sort the whole layer once with
    Python's sort, keep H*k, count per head."""
    H, n = len(lt), len(lt[0])
    sp = min(s, n)
    if k <= sp:
        return [k] * H
    items = []
    for h in range(H):
        safe = set(range(sp))
        rest = sorted(range(sp, n), key=lambda j: (-lt[h][j], j))
        safe |= set(rest[: max(int(np.floor(alpha * k)) - sp, 0)])
        for j in range(n):
            items.append((0 if j in safe else 1, -lt[h][j] if j not in safe else 0.0, h, j))
    items.sort()
    counts = [0] * H
    for it in items[: H * k]:
        counts[it[2]] += 1
    return counts


@pytest.mark.parametrize("H,n,k,s,alpha", [(4, 50, 10, 2, 0.2), (8, 64, 16, 4, 0.2), (3, 40, 40, 4, 0.5),
                                           (5, 30, 3, 4, 0.2), (2, 20, 7, 0, 0.0), (6, 33, 11, 4, 1.0),
                                           (4, 25, 24, 4, 0.3), (1, 30, 9, 4, 0.2)])
def test_matches_boost_and_sort(H, n, k, s, alpha):
    rng = np.random.default_rng([H, n, k, s])
    lt = rng.random((H, n)) ** 4
    lt /= lt.sum(1, keepdims=True)
    assert orc.adaptive_budgets(lt, k, s, alpha).tolist() == _boost_and_sort(lt.tolist(), k, s, alpha)
    # planted ties across heads: (head, token) order decides
    lt2 = np.round(lt * 40) / 40
    assert orc.adaptive_budgets(lt2, k, s, alpha).tolist() == _boost_and_sort(lt2.tolist(), k, s, alpha)


def test_invariants():
    rng = np.random.default_rng(3)
    for _ in range(30):
        H = int(rng.integers(1, 9)); n = int(rng.integers(10, 80)); s = int(rng.integers(0, 6))
        k = int(rng.integers(0, n + 1)); alpha = float(rng.choice([0.0, 0.2, 0.5, 1.0]))
        lt = rng.random((H, n)); lt /= lt.sum(1, keepdims=True)
        b = orc.adaptive_budgets(lt, k, s, alpha)
        assert b.sum() == H * k and b.min() >= 0 and b.max() <= n
        sp = min(s, n)
        if k > sp:
            assert b.min() >= sp + min(max(int(np.floor(alpha * k)) - sp, 0), n - sp)   # safeguard
        # the per-head selections with these budgets are the layer-wide top set: every kept
        # open token scores at least as high as every dropped one, in any head
        if 0.0 == alpha and k > sp:
            kept = [lt[h][orc.select(lt[h], int(b[h]), s)] for h in range(H)]
            kept_min = min((x[sp:].min() for x in kept if x.size > sp), default=np.inf)
            dropped_max = max((np.delete(lt[h], orc.select(lt[h], int(b[h]), s)).max()
                               for h in range(H) if b[h] < n), default=-np.inf)
            assert kept_min >= dropped_max


def test_limiting_cases():
    rng = np.random.default_rng(4)
    lt = rng.random((4, 100)); lt /= lt.sum(1, keepdims=True)
    assert orc.adaptive_budgets(lt, 20, 4, 1.0).tolist() == [20] * 4          # all safeguarded
    # identical heads share equally; the remainder goes to the lower heads (tie order)
    same = np.tile(lt[0], (4, 1))
    assert orc.adaptive_budgets(same, 20, 4, 0.2).tolist() == [20] * 4
    # one head holds every large score: it gets everything the safeguard leaves
    peaked = np.full((4, 100), 1e-6); peaked[2, 4:] = np.linspace(1, 2, 96)
    b = orc.adaptive_budgets(peaked, 20, 4, 0.2)
    g = int(np.floor(0.2 * 20)) - 4
    assert g == 0 and b.tolist() == [4, 4, 4 + 64, 4]
    b = orc.adaptive_budgets(peaked, 20, 4, 0.5)                              # g = 6 per head
    assert b.tolist() == [10, 10, 10 + 4 * 10, 10]
    # sinks are kept whatever they score, and do not compete
    lt2 = lt.copy(); lt2[:, :4] = 0.0
    assert np.array_equal(orc.adaptive_budgets(lt2, 20, 4, 0.2), orc.adaptive_budgets(lt, 20, 4, 0.2))
    # permuting heads with distinct scores permutes the budgets
    p = np.array([2, 0, 3, 1])
    assert np.array_equal(orc.adaptive_budgets(lt[p], 20, 4, 0.2), orc.adaptive_budgets(lt, 20, 4, 0.2)[p])
    # budget inside the sink block: nothing to allot
    assert orc.adaptive_budgets(lt, 3, 4, 0.2).tolist() == [3] * 4
    with pytest.raises(ValueError):
        orc.adaptive_budgets(lt, 101, 4, 0.2)
    with pytest.raises(ValueError):
        orc.adaptive_budgets(lt, 10, 4, 1.5)
