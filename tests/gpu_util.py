"""Helpers for the GPU parity tests: run the HIP path through the C ABI on a
host-generated cache and compare with the oracle.  Not collected by pytest."""

from __future__ import annotations

import numpy as np

from oracle import curdkv_oracle as orc
from paper_2509_15038_amd import binding as B
from paper_2509_15038_amd import workloads as wl

RTOL = 1e-3     # relative tolerance on scores: fp32 accumulation of exact bf16 products


def to_device(a: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t, dtype: str) -> np.ndarray:
    import torch
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class Guarded:
    """A device buffer with canary elements before and after it: a kernel that writes outside
    the buffer it was given (an overrun past the last group, an offset gone negative) changes
    them, which poisoning the payload alone would not show."""

    GUARD = 1024          # elements on each side; keeps 16-byte alignment for every dtype used here
    _PATTERN = {4: 0x5A5A5A5A, 2: 0x5A5A, 8: 0x5A5A5A5A5A5A5A5A}

    def __init__(self, shape, dtype, fill):
        import torch
        count = int(np.prod(shape))
        row = int(np.prod(shape[1:])) if len(shape) > 1 else 1
        self._g = -(-self.GUARD // row) * row       # whole rows
        self._back = torch.empty((count + 2 * self._g,), dtype=dtype, device="cuda")
        self._ibits = {4: torch.int32, 2: torch.int16, 8: torch.int64}[self._back.element_size()]
        self._pat = self._PATTERN[self._back.element_size()]
        raw = self._back.view(self._ibits)
        raw[: self._g] = self._pat
        raw[self._g + count:] = self._pat
        self.t = self._back[self._g: self._g + count].view(*shape)
        self.t.fill_(fill)

    def check(self, what=""):
        raw = self._back.view(self._ibits)
        n = self.t.numel()
        assert bool((raw[: self._g] == self._pat).all()), f"{what}: written before the start of the buffer"
        assert bool((raw[self._g + n:] == self._pat).all()), f"{what}: written past the end of the buffer"


def run_path(ctx: B.Context, Kd, Vd, n: int, budgets: np.ndarray, n_sink: int, dtype: str,
             one_call: bool = False):
    """scores -> select -> compact through the C ABI (or the one-call entry point,
    which picks the fused kernel when it applies).  Returns device tensors.  Every output
    buffer sits between canaries, checked after the calls."""
    import torch
    heads = ctx.heads
    offsets = wl.offsets_for(budgets)
    total = int(offsets[-1])
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g_sc = Guarded((heads, n), torch.float32, float("nan"))
    g_ix = Guarded((max(total, 1),), torch.int32, -7)
    # (filled with NaN bit patterns: a row that is left out cannot hide behind stale memory)
    g_ko = Guarded((max(total, 1), 128), tdt, float("nan"))
    g_vo = Guarded((max(total, 1), 128), tdt, float("nan"))
    scores, indices, Ko, Vo = g_sc.t, g_ix.t, g_ko.t, g_vo.t
    if one_call:
        ctx.compress(Kd, Vd, n, budgets, n_sink, offsets, scores, indices, Ko, Vo)
    else:
        ctx.scores(Kd, Vd, n, scores)
        ctx.select(scores, n, budgets, n_sink, offsets, indices)
        ctx.compact(Kd, Vd, n, indices, offsets, Ko, Vo)
    torch.cuda.synchronize()
    for g, what in ((g_sc, "scores"), (g_ix, "indices"), (g_ko, "K_out"), (g_vo, "V_out")):
        g.check(what)
    if total == 0:                                  # nothing may have been written at all
        assert int(indices[0]) == -7 and bool(torch.isnan(Ko.float()).all()) and bool(torch.isnan(Vo.float()).all())
    return scores, indices[:total], Ko[:total], Vo[:total], offsets


def check_scores(got: np.ndarray, want: np.ndarray, where=""):
    err = np.abs(got.astype(np.float64) - want)
    bad = err > RTOL * np.abs(want) + 1e-37
    assert not bad.any(), f"{where}: {int(bad.sum())} scores off, worst rel {np.max(err / np.maximum(np.abs(want), 1e-300)):.3e}"
    return float(np.max(err / np.maximum(np.abs(want), 1e-300)))


def check_selection(got: np.ndarray, lt: np.ndarray, k: int, s: int, where=""):
    """Index set: identical to the oracle's except for tokens whose oracle score
    is within RTOL (relative) of the oracle's score at the cut."""
    want = orc.select(lt, k, s)
    assert got.shape == want.shape, f"{where}: size {got.shape} vs {want.shape}"
    assert np.all(np.diff(got) > 0), f"{where}: indices not strictly ascending"
    if k:
        assert got[0] >= 0 and got[-1] < lt.size, where
    if np.array_equal(got, want):
        return 0
    assert k > s, where
    diff = np.setxor1d(got, want)
    assert np.all(diff >= s), f"{where}: sink tokens differ"
    cut = np.min(lt[want[want >= s]])          # the (k-s)-th largest candidate score
    assert np.all(np.abs(lt[diff] - cut) <= RTOL * cut), \
        f"{where}: {diff.size} tokens differ beyond the near-cut band"
    return int(diff.size)


def check_head(cfg, ctxargs, K, V, G, scores_g, idx_g, Ko_g, Vo_g, k, s, where="",
               source="kv", projection=True, lt=None):
    """All three comparisons for one (layer, head) given host copies.  lt: the oracle's scores
    of this group when the caller has them already (they do not depend on the budget)."""
    if lt is None:
        lt = orc.scores(orc.to_f64(K, cfg.dtype), orc.to_f64(V, cfg.dtype), G, source, projection)
    rel = check_scores(scores_g, lt, where)
    ndiff = check_selection(idx_g.astype(np.int64), lt, k, s, where)
    Kc, Vc = orc.compact(K, V, idx_g.astype(np.int64))
    assert np.array_equal(Ko_g, Kc), f"{where}: gathered K differs"
    assert np.array_equal(Vo_g, Vc), f"{where}: gathered V differs"
    return rel, ndiff


def check_adaptive_budgets(got: np.ndarray, lt: np.ndarray, k: int, s: int, alpha: float, where=""):
    """Head-wise budgets of one layer against the oracle's, which are computed from the
    oracle's own float64 scores lt [H, n].  The GPU decides on its fp32 scores, so the two may
    disagree about tokens whose oracle score is within RTOL (relative) of the oracle's cut
    score: a head's budget may differ by at most the number of its tokens in that band, the
    layer's total and the safeguard must hold exactly."""
    H, n = lt.shape
    want = orc.adaptive_budgets(lt, k, s, alpha)
    assert got.shape == want.shape and int(got.sum()) == int(want.sum()), f"{where}: layer total"
    sp = min(s, n)
    if k > sp:
        g = min(max(int(np.floor(alpha * k)) - sp, 0), n - sp)
        assert got.min() >= sp + g, f"{where}: safeguard"
    if np.array_equal(got, want):
        return 0
    cut = orc.adaptive_cut_score(lt, k, s, alpha)
    assert cut is not None, f"{where}: budgets differ although nothing is allotted layer-wide"
    band = np.sum(np.abs(lt[:, sp:] - cut) <= RTOL * cut, axis=1)
    assert np.all(np.abs(got.astype(np.int64) - want) <= band), \
        f"{where}: budgets {got.tolist()} vs {want.tolist()}, near-cut tokens per head {band.tolist()}"
    return int(np.abs(got.astype(np.int64) - want).sum())


def run_and_check(cfg: wl.Config, budgets: np.ndarray, n_sink=None, K=None, V=None,
                  one_call: bool = False, source: str = "kv", projection: bool = True, fused=None):
    """Whole path on a host cache, every head compared with the oracle.  fused = True / False
    additionally asserts which kernels the library says it launches for this shape."""
    s = cfg.n_sink if n_sink is None else n_sink
    if K is None:
        K, V = wl.host_cache(cfg)
    L, H, n = cfg.layers, cfg.kv_heads, cfg.n
    Kd, Vd = to_device(K, cfg.dtype), to_device(V, cfg.dtype)
    worst, ndiff = 0.0, 0
    with B.Context(L, H, cfg.group, cfg.d, cfg.r, cfg.dtype, n, cfg.sketch_seed, source, projection) as ctx:
        if fused is not None:
            assert ctx.uses_fused_kernel(n) == fused, f"{cfg.name}: expected fused={fused} for {L * H} heads, n={n}"
        sc, idx, Ko, Vo, off = run_path(ctx, Kd, Vd, n, budgets, s, cfg.dtype, one_call)
        sc_h, idx_h = sc.cpu().numpy(), idx.cpu().numpy()
        Ko_h, Vo_h = to_host(Ko, cfg.dtype), to_host(Vo, cfg.dtype)
        for l in range(L):
            for h in range(H):
                i = l * H + h
                G = orc.sketch(cfg.sketch_seed, l, h, H, cfg.d, cfg.r, cfg.dtype)
                a, b = int(off[i]), int(off[i + 1])
                rel, nd = check_head(cfg, None, K[l, h], V[l, h], G, sc_h[i], idx_h[a:b],
                                     Ko_h[a:b], Vo_h[a:b], int(budgets[i]), s,
                                     where=f"{cfg.name} l{l} h{h} n{n} {source} proj={projection}",
                                     source=source, projection=projection)
                worst = max(worst, rel)
                ndiff += nd
    return worst, ndiff
