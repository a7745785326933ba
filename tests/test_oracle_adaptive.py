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


def _cut_from_one_sort(lt, k, s, alpha):
    """The score of the last token the layer-wide step lets in, read off the same single sort:
    among the H*k kept items, the non-safe one that sorts last.  None when the step admits
    nobody (budget inside the sinks, or the safeguard covers every place)."""
    H, n = len(lt), len(lt[0])
    sp = min(s, n)
    if k <= sp:
        return None
    items = []
    for h in range(H):
        rest = sorted(range(sp, n), key=lambda j: (-lt[h][j], j))
        safe = set(range(sp)) | set(rest[: max(int(np.floor(alpha * k)) - sp, 0)])
        for j in range(n):
            items.append((0 if j in safe else 1, -lt[h][j] if j not in safe else 0.0, h, j))
    items.sort()
    admitted = [it for it in items[: H * k] if it[0] == 1]
    return lt[admitted[-1][2]][admitted[-1][3]] if admitted else None


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
    # the cut score that goes with these budgets, from the same independent construction
    for a in (lt, lt2):
        assert orc.adaptive_cut_score(a, k, s, alpha) == _cut_from_one_sort(a.tolist(), k, s, alpha)


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


def test_cut_score_separates_kept_from_dropped():
    """What the cut score means, checked on the selections themselves: with the budgets fed to
    the per-head selection, no dropped token scores above the cut, and every kept token outside
    the sinks and the safeguarded ones scores at least the cut, which one of them attains."""
    rng = np.random.default_rng(11)
    seen_none = seen_value = 0
    for trial in range(60):
        H = int(rng.integers(1, 7)); n = int(rng.integers(12, 70)); s = int(rng.integers(0, 6))
        k = int(rng.integers(0, n + 1)); alpha = float(rng.choice([0.0, 0.2, 0.6, 1.0]))
        lt = rng.random((H, n)) ** 3
        if trial % 3 == 0:
            lt = np.round(lt * 12) / 12 + 1e-3                 # many equal scores
        lt /= lt.sum(1, keepdims=True)
        b = orc.adaptive_budgets(lt, k, s, alpha)
        cut = orc.adaptive_cut_score(lt, k, s, alpha)
        sp = min(s, n)
        g = min(max(int(np.floor(alpha * k)) - sp, 0), n - sp) if k > sp else 0
        if k <= sp or H * (k - sp) - H * g == 0:
            assert cut is None
            seen_none += 1
            continue
        seen_value += 1
        open_kept, dropped = [], []
        for h in range(H):
            S = orc.select(lt[h], int(b[h]), s)
            rest = sorted(range(sp, n), key=lambda j: (-lt[h][j], j))
            safe = set(range(sp)) | set(rest[:g])
            open_kept += [lt[h][j] for j in S if j not in safe]
            dropped += [lt[h][j] for j in range(n) if j not in set(S.tolist())]
        assert open_kept and min(open_kept) == cut
        assert not dropped or max(dropped) <= cut
    assert seen_none >= 5 and seen_value >= 20


def test_cut_score_hand_example():
    # two heads, no sinks, no safeguard, three places: the layer's scores in order are
    # 0.9 (h0), 0.8 (h1), 0.7 (h1), 0.6 (h0), ...: the third place goes to 0.7
    lt = np.array([[0.9, 0.6, 0.1, 0.05], [0.8, 0.7, 0.2, 0.0]])
    # (un-normalised on purpose: the allocation only compares the numbers it is given)
    assert orc.adaptive_budgets(lt, 0, 0, 0.0).tolist() == [0, 0]
    assert orc.adaptive_cut_score(lt, 0, 0, 0.0) is None
    # k is per head: k = 2 gives four places -> 0.9, 0.8, 0.7, 0.6
    assert orc.adaptive_budgets(lt, 2, 0, 0.0).tolist() == [2, 2]
    assert orc.adaptive_cut_score(lt, 2, 0, 0.0) == 0.6
    # k = 1: two places -> 0.9 and 0.8
    assert orc.adaptive_budgets(lt, 1, 0, 0.0).tolist() == [1, 1]
    assert orc.adaptive_cut_score(lt, 1, 0, 0.0) == 0.8
    # with one sink per head the sinks (0.9, 0.8) are outside the contest: k = 2 leaves two
    # places for 0.7, 0.6, 0.2, 0.1, 0.05, 0.0
    assert orc.adaptive_budgets(lt, 2, 1, 0.0).tolist() == [2, 2]
    assert orc.adaptive_cut_score(lt, 2, 1, 0.0) == 0.6
    # safeguard covering everything: alpha = 1 leaves no place to allot
    assert orc.adaptive_cut_score(lt, 2, 0, 1.0) is None
    # safeguard of one token per head (alpha*k = 1): 0.9 and 0.8 are safe, the two open places
    # go to 0.7 and 0.6
    assert orc.adaptive_cut_score(lt, 2, 0, 0.5) == 0.6
    # three tokens per head, safeguard one: open places 2*3 - 2 = 4 -> 0.7, 0.6, 0.2, 0.1
    assert orc.adaptive_budgets(lt, 3, 0, 0.34).tolist() == [3, 3]
    assert orc.adaptive_cut_score(lt, 3, 0, 0.34) == 0.1
