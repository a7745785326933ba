"""Planted mistakes for the oracle: each entry patches ONE plausible error into
`oracle.curdkv_oracle` (a dropped term, a wrong sign or index, a swapped operand,
a wrong tie rule).  `test_oracle_mutants.py` re-runs the oracle's pins with each
mistake switched on and requires that at least one pin fails, which is the
evidence that the pins would notice such a mistake in the real oracle.

CPU only; nothing here touches the HIP path."""

import numpy as np

from oracle import curdkv_oracle as orc

_orig = {name: getattr(orc, name) for name in dir(orc) if callable(getattr(orc, name))}


def _row_norm_unsquared():
    orc.row_norm_sq = lambda Y: np.sqrt(np.sum(Y * Y, axis=1))


def _row_norm_abs_sum():
    orc.row_norm_sq = lambda Y: np.sum(np.abs(Y), axis=1) ** 2


def _combine_is_sum():
    orc.combine = lambda lk, lv: lk + lv


def _combine_drops_value():
    orc.combine = lambda lk, lv: lk * lk


def _normalise_skips_sinks():
    def normalise(lkv, s=4):
        total = float(np.sum(lkv[s:]))
        return lkv / total if total > 0 else np.full(lkv.shape[0], 1.0 / lkv.shape[0])
    orc.normalise = normalise


def _normalise_by_max():
    def normalise(lkv):
        m = float(np.max(lkv))
        return lkv / m if m > 0 else np.full(lkv.shape[0], 1.0 / lkv.shape[0])
    orc.normalise = normalise


def _normalise_by_sum_of_squares():
    def normalise(lkv):
        t = float(np.sqrt(np.sum(lkv * lkv)))
        return lkv / t if t > 0 else np.full(lkv.shape[0], 1.0 / lkv.shape[0])
    orc.normalise = normalise


def _select_sinks_from_the_end():
    orig = _orig["select"]
    def select(lt, k, s):
        lt = np.asarray(lt, dtype=np.float64)
        n = lt.shape[0]
        if not (0 <= k <= n) or s < 0:
            raise ValueError("bad budget")
        if k <= s:
            return np.arange(k, dtype=np.int64)
        recent = np.arange(n - s, n, dtype=np.int64)             # the last s tokens instead of the first
        top = np.argsort(-lt[: n - s], kind="stable")[: k - s].astype(np.int64)
        return np.sort(np.concatenate([top, recent]))
    orc.select = select


def _normalise_zero_stays_zero():
    def normalise(lkv):
        total = float(np.sum(lkv))
        return lkv / total if total > 0 else np.zeros_like(lkv)
    orc.normalise = normalise


def _project_rows_reversed():
    orc.project = lambda A, G: np.asarray(A, dtype=np.float64) @ np.asarray(G, dtype=np.float64)[::-1]


def _project_accepts_transposed_sketch():
    def project(A, G):
        A = np.asarray(A, dtype=np.float64); G = np.asarray(G, dtype=np.float64)
        return A @ (G if G.shape[0] == A.shape[1] else G.T)
    orc.project = project


def _value_side_uses_another_sketch():
    def scores_unnormalised(K64, V64, G):
        lk = orc.row_norm_sq(orc.project(K64, G))
        lv = orc.row_norm_sq(orc.project(V64, np.roll(G, 1, axis=0)))
        return lk, lv, orc.combine(lk, lv)
    orc.scores_unnormalised = scores_unnormalised


def _sketch_with(**kw):
    """sketch() with one detail of the generator changed."""
    def sketch(seed, layer, head, kv_heads, d, r, dtype):
        if kw.get("ignore_head"):
            head = 0
        base = ((layer * kv_heads + head) * d) * r
        w = orc.splitmix64_outputs(seed, 2 * base + 1, 2 * d * r)
        w1, w2 = (w[1::2], w[0::2]) if kw.get("swap_words") else (w[0::2], w[1::2])
        u1 = ((w1 >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
        u2 = (w2 >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
        trig = np.sin if kw.get("sine") else np.cos
        z = np.sqrt(-2.0 * np.log(u1)) * trig(2.0 * np.pi * u2)
        if kw.get("uniform"):
            z = (u2 - 0.5) * np.sqrt(12.0)          # mean 0, variance 1, not Gaussian
        g = z / (1.0 if kw.get("unit_variance") else (float(r) if kw.get("over_r") else np.sqrt(float(r))))
        if kw.get("column_major"):
            return orc.round_to_storage(g, dtype).reshape(r, d).T.copy()
        return orc.round_to_storage(g, dtype).reshape(d, r)
    orc.sketch = sketch


def _splitmix_wrong_shift():
    def splitmix64_outputs(seed, first, count):
        with np.errstate(over="ignore"):
            i = np.arange(first, first + count, dtype=np.uint64)
            z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + i * orc._GAMMA
            z = (z ^ (z >> np.uint64(30))) * orc._M1
            z = (z ^ (z >> np.uint64(27))) * orc._M2
            return z ^ (z >> np.uint64(33))
    orc.splitmix64_outputs = splitmix64_outputs


def _splitmix_zero_based():
    orig = _orig["splitmix64_outputs"]
    orc.splitmix64_outputs = lambda seed, first, count: orig(seed, first - 1, count)


def _bf16_truncates():
    orc.f32_to_bf16_bits = lambda x: (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
                                      >> np.uint32(16)).astype(np.uint16)


def _bf16_rounds_half_up():
    def f(x):
        u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
        return ((u + np.uint32(0x8000)) >> np.uint32(16)).astype(np.uint16)
    orc.f32_to_bf16_bits = f


def _leverage_unsquared():
    orig = _orig["leverage_exact"]
    orc.leverage_exact = lambda A, rcond=1e-12: np.sqrt(orig(A, rcond))


def _leverage_keeps_null_directions():
    def leverage_exact(A, rcond=1e-12):
        U, _, _ = np.linalg.svd(np.asarray(A, dtype=np.float64), full_matrices=False)
        return np.sum(U * U, axis=1)
    orc.leverage_exact = leverage_exact


def _select_with(**kw):
    def select(lt, k, s):
        lt = np.asarray(lt, dtype=np.float64)
        n = lt.shape[0]
        if not (0 <= k <= n):
            raise ValueError("budget k must satisfy 0 <= k <= n")
        if s < 0:
            raise ValueError("num_sink must be >= 0")
        if k <= s:
            return np.arange(k, dtype=np.int64)
        sink = np.arange(s, dtype=np.int64)
        if kw.get("sinks_compete"):                      # top-k over all rows, then the union
            top = np.argsort(-lt, kind="stable")[: k - s].astype(np.int64)
            return np.unique(np.concatenate([sink, top]))
        cand = lt[s:]
        if kw.get("ties_high_index"):
            order = (cand.shape[0] - 1 - np.argsort(-cand[::-1], kind="stable"))
        elif kw.get("smallest"):
            order = np.argsort(cand, kind="stable")
        else:
            order = np.argsort(-cand, kind="stable")
        take = k - s - 1 if kw.get("one_short") else k - s
        top = order[:take].astype(np.int64) + (0 if kw.get("no_offset") else s)
        out = np.concatenate([sink, top])
        return out if kw.get("unsorted") else np.sort(out)
    orc.select = select


def _select_small_budget_keeps_sinks():
    orig = _orig["select"]
    def select(lt, k, s):
        if 0 < k <= s:
            return np.arange(s, dtype=np.int64)          # all sinks although the budget is smaller
        return orig(lt, k, s)
    orc.select = select


def _compact_swaps_outputs():
    orc.compact = lambda K, V, S: (V[S], K[S])


def _compact_sorted_by_score_not_index():
    orc.compact = lambda K, V, S: (K[S[::-1]], V[S[::-1]])


def _fold_is_sum():
    orc.fold_gqa = lambda q: np.sum(np.asarray(q, dtype=np.float64), axis=0)


def _fold_is_max():
    orc.fold_gqa = lambda q: np.max(np.asarray(q, dtype=np.float64), axis=0)


def _adaptive_with(**kw):
    def adaptive_budgets(lt, k, s, alpha):
        lt = np.asarray(lt, dtype=np.float64)
        H, n = lt.shape
        if not (0 <= k <= n) or s < 0 or not (0.0 <= alpha <= 1.0):
            raise ValueError("need 0 <= k <= n, s >= 0, 0 <= alpha <= 1")
        sp = min(s, n)
        if k <= sp:
            return np.full(H, k, dtype=np.int64)
        floor = int(np.floor(alpha * k))
        if kw.get("no_safeguard"):
            g = 0
        elif kw.get("sinks_outside_safeguard"):
            g = min(floor, n - sp)
        else:
            g = min(max(floor - sp, 0), n - sp)
        R = H * (k - sp) - (0 if kw.get("open_budget_ignores_safeguard") else H * g)
        cand = lt[:, sp:]
        order = np.argsort(-cand, axis=1, kind="stable")
        rank = np.empty_like(order)
        rows = np.arange(H)[:, None]
        rank[rows, order] = np.arange(n - sp)[None, :]
        open_ = rank >= (0 if kw.get("safe_tokens_compete_again") else g)
        head_of = np.broadcast_to(rows, cand.shape)[open_]
        vals = cand[open_]
        if kw.get("ties_last_head_first"):
            picked = (vals.shape[0] - 1 - np.argsort(-vals[::-1], kind="stable"))[:max(R, 0)]
        else:
            picked = np.argsort(-vals, kind="stable")[:max(R, 0)]
        extra = np.bincount(head_of[picked], minlength=H)
        return ((0 if kw.get("sinks_not_counted") else sp) + g + extra).astype(np.int64)
    orc.adaptive_budgets = adaptive_budgets


def _cut_with(**kw):
    """adaptive_cut_score with one mistake in how the cut is read off the layer-wide ranking."""
    def adaptive_cut_score(lt, k, s, alpha):
        lt = np.asarray(lt, dtype=np.float64)
        H, n = lt.shape
        sp = min(s, n)
        if k <= sp:
            return None
        g = min(max(int(np.floor(alpha * k)) - sp, 0), n - sp)
        R = H * (k - sp) - H * g
        if R <= 0:
            return None
        cand = lt[:, sp:]
        order = np.argsort(-cand, axis=1, kind="stable")
        rank = np.empty_like(order)
        rows = np.arange(H)[:, None]
        rank[rows, order] = np.arange(n - sp)[None, :]
        open_ = rank >= g
        if kw.get("before_safeguard_mask"):            # safe tokens take part in the ranking
            vals = cand.reshape(-1)
        else:
            vals = cand[open_]
        ranked = np.sort(vals)[::-1]
        if kw.get("largest_admitted"):
            return float(ranked[0])
        if kw.get("first_left_out"):
            return float(ranked[min(R, ranked.size - 1)])
        return float(ranked[R - 1])
    orc.adaptive_cut_score = adaptive_cut_score


def _adaptive_uniform():
    orc.adaptive_budgets = lambda lt, k, s, alpha: np.full(np.asarray(lt).shape[0], k, dtype=np.int64)


def _scores_ignore_source():
    orig = _orig["scores"]
    def scores(K64, V64, G, source="kv", projection=True):
        if source not in ("kv", "k", "v"):
            raise ValueError("unknown score source")
        return orig(K64, V64, G, "kv", projection)
    orc.scores = scores


def _scores_project_even_when_told_not_to():
    orig = _orig["scores"]
    def scores(K64, V64, G, source="kv", projection=True):
        return orig(K64, V64, G if G is not None else np.eye(np.asarray(K64).shape[1])[:, ::2] , source, True)
    orc.scores = scores


def _eviction(which):
    from oracle import eviction_eval as ev
    if which == "no_scaling_loss":
        ev.attention_output = lambda Q, K, V: ev.softmax_rows(Q @ K.T) @ V[::-1]
    elif which == "softmax_columns":
        def softmax_rows(X):
            E = np.exp(X - X.max())
            return E / E.sum(axis=0, keepdims=True)
        ev.softmax_rows = softmax_rows
    elif which == "lemma_drops_second_term":
        orig = ev.lemma1_sides
        def lemma1_sides(Q, K, V, S):
            lhs, _ = orig(Q, K, V, S)
            n = K.shape[0]
            keep = np.zeros(n, dtype=bool); keep[S] = True
            return lhs, float(np.sqrt(n) * np.linalg.norm(V - V * keep[:, None]))
        ev.lemma1_sides = lemma1_sides


MUTANTS = {
    "row_norm_unsquared": _row_norm_unsquared,
    "row_norm_abs_sum": _row_norm_abs_sum,
    "combine_is_sum": _combine_is_sum,
    "combine_drops_value": _combine_drops_value,
    "normalise_skips_sinks": _normalise_skips_sinks,
    "normalise_by_max": _normalise_by_max,
    "normalise_zero_stays_zero": _normalise_zero_stays_zero,
    "project_rows_reversed": _project_rows_reversed,
    "project_accepts_transposed_sketch": _project_accepts_transposed_sketch,
    "value_side_uses_another_sketch": _value_side_uses_another_sketch,
    "sketch_unit_variance": lambda: _sketch_with(unit_variance=True),
    "sketch_variance_one_over_r_squared": lambda: _sketch_with(over_r=True),
    "sketch_sine": lambda: _sketch_with(sine=True),
    "sketch_words_swapped": lambda: _sketch_with(swap_words=True),
    "sketch_same_for_every_head": lambda: _sketch_with(ignore_head=True),
    "sketch_column_major_counter": lambda: _sketch_with(column_major=True),
    "sketch_uniform_not_gaussian": lambda: _sketch_with(uniform=True),
    "splitmix_wrong_shift": _splitmix_wrong_shift,
    "splitmix_zero_based": _splitmix_zero_based,
    "bf16_truncates": _bf16_truncates,
    "bf16_rounds_half_up": _bf16_rounds_half_up,
    "leverage_unsquared": _leverage_unsquared,
    "leverage_keeps_null_directions": _leverage_keeps_null_directions,
    "select_ties_high_index": lambda: _select_with(ties_high_index=True),
    "select_smallest": lambda: _select_with(smallest=True),
    "select_no_offset": lambda: _select_with(no_offset=True),
    "select_sinks_compete": lambda: _select_with(sinks_compete=True),
    "select_one_short": lambda: _select_with(one_short=True),
    "select_unsorted": lambda: _select_with(unsorted=True),
    "select_small_budget_keeps_sinks": _select_small_budget_keeps_sinks,
    "compact_swaps_outputs": _compact_swaps_outputs,
    "compact_reversed_rows": _compact_sorted_by_score_not_index,
    "fold_is_sum": _fold_is_sum,
    "fold_is_max": _fold_is_max,
    "adaptive_no_safeguard": lambda: _adaptive_with(no_safeguard=True),
    "adaptive_sinks_outside_safeguard": lambda: _adaptive_with(sinks_outside_safeguard=True),
    "adaptive_ties_last_head_first": lambda: _adaptive_with(ties_last_head_first=True),
    "adaptive_uniform": _adaptive_uniform,
    "adaptive_open_budget_ignores_safeguard": lambda: _adaptive_with(open_budget_ignores_safeguard=True),
    "adaptive_safe_tokens_compete_again": lambda: _adaptive_with(safe_tokens_compete_again=True),
    "adaptive_sinks_not_counted": lambda: _adaptive_with(sinks_not_counted=True),
    "cut_score_is_largest_admitted": lambda: _cut_with(largest_admitted=True),
    "cut_score_is_first_left_out": lambda: _cut_with(first_left_out=True),
    "cut_score_ranked_before_safeguard_mask": lambda: _cut_with(before_safeguard_mask=True),
    "normalise_by_sum_of_squares": _normalise_by_sum_of_squares,
    "select_sinks_from_the_end": _select_sinks_from_the_end,
    "scores_ignore_source": _scores_ignore_source,
    "scores_project_without_sketch": _scores_project_even_when_told_not_to,
    "eviction_rows_misaligned": lambda: _eviction("no_scaling_loss"),
    "softmax_over_columns": lambda: _eviction("softmax_columns"),
    "lemma_drops_second_term": lambda: _eviction("lemma_drops_second_term"),
}
