"""CurDKV post-prefill KV selection: the slow, plain CPU oracle (float64, numpy).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the HIP
kernels can be checked against something written straight from the paper.
Only tests, the smoke check and the benchmark's cpu-baseline leg may import
it; the product path (the C-ABI library and its Python binding) never does,
and it shares no code, table or helper with that path.

What is computed (Algorithm 1 of the paper, the CUR-based compression with GQA
support), per layer and per KV group i, in this order:

  1. a Gaussian sketch G with d rows, r columns and entry variance 1/r is drawn;
  2. the keys and the values of the group are both multiplied by it from the right;
  3. every projected row is scored by its squared Euclidean norm, which gives one
     key score and one value score per token;
  4. the two are multiplied into one score per token;
  5. the scores are divided by their sum over all n tokens;
  6. the first s tokens are set aside as sinks, the k - s best of the remaining
     tokens are added to them;
  7. the rows of the ORIGINAL keys and values at those positions are the output.

Each step is a function of its own below (`sketch`, `project`, `row_norm_sq`,
`combine`, `normalise`, `select`, `compact`), and `compress_group` chains them.

The method is an approximation followed by a heuristic selection, so the
oracle follows the algorithm's steps in the paper's order; it is not a
different route to an exactly defined quantity.  The exact leverage scores of
Section 3.1 (row norms of the left singular vectors) are provided separately
and are used only to pin this file in the tests.

Readings taken where the paper is silent or inconsistent:
  * Algorithm 1 overwrites K_i by K_i G and then gathers rows of K_i; the
    output shape g x k x d fixes that the gather is from the ORIGINAL K_i, V_i.
  * Section 3.1 defines the leverage score un-squared while the introduction
    and Algorithm 1 use squared norms: squared everywhere here.
  * Section 3.1 states that the squared row leverage scores sum to n; for a
    semi-unitary U with rank(A) columns they sum to rank(A).  The tests use
    the latter.
  * One G per (layer, group), shared by K and V (it is sampled once inside
    the group loop and used for both projections).
  * The paper gives no seed: G comes from the counter-based generator below,
    and is rounded to the storage type of K and V, so both sides of a parity
    test multiply by identical numbers.
  * sum_j lKV_j == 0: lt_j := 1/n (keeps the sum at one).
  * TopK ties: larger score first, then smaller token index.
  * S_i is reported in ascending token order.
  * k <= s keeps tokens 0..k-1; k == 0 keeps nothing; k == n keeps all.

parity unpinned: the paper prints no score, index set or sketch value, so no
function here is pinned to a number from the paper.  Each is pinned instead by
closed forms, invariants, textbook special cases and brute force (tests/).
"""

from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# storage types: exact up-casts and round-to-nearest-even down-casts
# --------------------------------------------------------------------------


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Stored K/V (dtype 'bf16': uint16 bit patterns, 'fp32': float32) -> float64."""
    if dtype == "bf16":
        return bf16_bits_to_f64(a)
    if dtype == "fp32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def round_to_storage(x64: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the K/V storage type and return them as float64."""
    x32 = np.asarray(x64, dtype=np.float64).astype(np.float32)  # RNE
    if dtype == "fp32":
        return x32.astype(np.float64)
    if dtype == "bf16":
        # float64 -> float32 -> bfloat16 is a double rounding; it differs from a
        # direct rounding only when the float32 result lands exactly on a bf16
        # tie, which needs the float64 value within 2^-29 relative of it.
        return bf16_bits_to_f64(f32_to_bf16_bits(x32))
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# the sketch G (Algorithm 1, sampling step; Section 3.2,
# "Approximate leverage scores and Gaussian projections")
# --------------------------------------------------------------------------

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64_outputs(seed: int, first: int, count: int) -> np.ndarray:
    """Outputs number first .. first+count-1 (1-based) of the SplitMix64
    generator (Steele, Lea, Flood 2014) started from state `seed`.

    Output number i is mix(seed + i*gamma): the generator is a counter passed
    through a fixed 64-bit finaliser, so any output can be had directly.
    """
    with np.errstate(over="ignore"):
        i = np.arange(first, first + count, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + i * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def sketch(seed: int, layer: int, head: int, kv_heads: int, d: int, r: int,
           dtype: str) -> np.ndarray:
    """G in R^{d x r} with entries N(0, 1/r) for group (layer, head).

    Element (i, j) has counter c = ((layer*kv_heads + head)*d + i)*r + j and
    uses SplitMix64 outputs 2c+1 and 2c+2 of the stream seeded by `seed`:
        u1 = ((w1 >> 11) + 1) * 2^-53   in (0, 1]
        u2 =  (w2 >> 11)      * 2^-53   in [0, 1)
        z  = sqrt(-2 ln u1) * cos(2 pi u2)        (Box-Muller)
        G_ij = z / sqrt(r), rounded to the storage type of K and V.
    Returned as float64 holding the rounded values.
    """
    base = ((layer * kv_heads + head) * d) * r
    w = splitmix64_outputs(seed, 2 * base + 1, 2 * d * r)
    w1 = w[0::2]
    w2 = w[1::2]
    two53 = 2.0 ** -53
    u1 = ((w1 >> np.uint64(11)).astype(np.float64) + 1.0) * two53
    u2 = (w2 >> np.uint64(11)).astype(np.float64) * two53
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    g = z / np.sqrt(float(r))
    return round_to_storage(g, dtype).reshape(d, r)


# --------------------------------------------------------------------------
# exact leverage scores (Section 3.1, row leverage score equation) -- used
# only to pin the sketched scores in the tests
# --------------------------------------------------------------------------


def leverage_exact(A: np.ndarray, rcond: float = 1e-12) -> np.ndarray:
    """Squared row leverage scores ||U(j,:)||_2^2 of A = U Sigma V^*, where U
    keeps the rank(A) left singular vectors with non-negligible singular value."""
    A = np.asarray(A, dtype=np.float64)
    U, sv, _ = np.linalg.svd(A, full_matrices=False)
    rank = int(np.sum(sv > rcond * sv.max())) if sv.size and sv.max() > 0 else 0
    U = U[:, :rank]
    return np.sum(U * U, axis=1)


# --------------------------------------------------------------------------
# Algorithm 1, step by step
# --------------------------------------------------------------------------


def project(A: np.ndarray, G: np.ndarray) -> np.ndarray:
    """Projection step of Algorithm 1: A G with A in R^{n x d}, G in R^{d x r}."""
    return np.asarray(A, dtype=np.float64) @ np.asarray(G, dtype=np.float64)


def row_norm_sq(Y: np.ndarray) -> np.ndarray:
    """Scoring step of Algorithm 1: l_j = ||Y[j]||_2^2, the squared norm of projected row j."""
    return np.sum(Y * Y, axis=1)


def combine(lk: np.ndarray, lv: np.ndarray) -> np.ndarray:
    """Combination step of Algorithm 1: key score times value score, token by token
    (the ablation section describes it as an elementwise product as well)."""
    return lk * lv


def normalise(lkv: np.ndarray) -> np.ndarray:
    """Normalisation step of Algorithm 1: divide by the sum over all n rows (sinks
    included, since the sink step comes later).  All-zero input gives 1/n everywhere."""
    total = float(np.sum(lkv))
    n = lkv.shape[0]
    if not total > 0.0:
        return np.full(n, 1.0 / n, dtype=np.float64)
    return lkv / total


def scores(K64: np.ndarray, V64: np.ndarray, G, source: str = "kv",
           projection: bool = True) -> np.ndarray:
    """Normalised scores lt in R^n of one group.

    K64, V64: float64 [n, d] (exact up-casts of the stored cache).
    G: float64 [d, r] holding the storage-rounded sketch (unused without projection).

    The two ablations of the appendix ("Ablation Study"):
      source = "k" / "v": leverage scores from the keys or the values alone instead
        of their elementwise product (the combination step is dropped);
      projection = False: the sampling and projection steps are dropped and the row
        norms are taken on the original matrices."""
    if source not in ("kv", "k", "v"):
        raise ValueError(f"unknown score source {source!r}")
    lk = row_norm_sq(project(K64, G) if projection else np.asarray(K64, dtype=np.float64))
    lv = row_norm_sq(project(V64, G) if projection else np.asarray(V64, dtype=np.float64))
    if source == "kv":
        return normalise(combine(lk, lv))
    return normalise(lk if source == "k" else lv)


def scores_unnormalised(K64: np.ndarray, V64: np.ndarray, G: np.ndarray):
    """(lK, lV, lKV) before normalisation, for tests that look inside."""
    lk = row_norm_sq(project(K64, G))
    lv = row_norm_sq(project(V64, G))
    return lk, lv, combine(lk, lv)


def fold_gqa(scores_q: np.ndarray) -> np.ndarray:
    """Fold per-query-head scores [group, n] of one KV group into one score per
    token by the mean over the group (the GQA-compatible aggregation the
    related-work section attributes to AdaKV).  CurDKV's own scores are a
    function of K_i and V_i, which the group shares, so every row is the same
    and the fold returns it unchanged."""
    return np.mean(np.asarray(scores_q, dtype=np.float64), axis=0)


def select(lt: np.ndarray, k: int, s: int) -> np.ndarray:
    """Sink, top-k and union steps of Algorithm 1.  Returns S_i ascending, |S_i| = k."""
    lt = np.asarray(lt, dtype=np.float64)
    n = lt.shape[0]
    if not (0 <= k <= n):
        raise ValueError("budget k must satisfy 0 <= k <= n")
    if s < 0:
        raise ValueError("num_sink must be >= 0")
    if k <= s:
        return np.arange(k, dtype=np.int64)
    sink = np.arange(s, dtype=np.int64)
    order = np.argsort(-lt[s:], kind="stable")  # larger first, ties: lower index
    top = order[: k - s].astype(np.int64) + s
    return np.sort(np.concatenate([sink, top]))


def adaptive_budgets(lt: np.ndarray, k: int, s: int, alpha: float) -> np.ndarray:
    """AdaCurDKV's head-wise budgets for one layer (Section 3.2, "Adaptive budget
    allocation"): the layer keeps H*k tokens in all, chosen as the top scores
    ACROSS the heads of the layer, except that every head is guaranteed a minimum
    fraction alpha of the group budget (the safeguard of AdaKV, alpha = 0.20 in the
    paper).  Returns int64 [H]: tokens to keep per head, sinks included; feeding
    them to `select` head by head gives the layer-wide selection.

    lt: float64 [H, n], the normalised scores of the layer's heads.

    Reading (the paper gives one sentence and points to AdaKV): the first
    s' = min(s, n) tokens of every head are sinks, always kept and part of the
    head's count.  Each head's own best floor(alpha*k) tokens, sinks first, are
    safe: that is g = max(floor(alpha*k) - s', 0) non-sink tokens per head (at
    most n - s').  The remaining R = H*(k - s') - H*g places go to the largest
    scores among all non-sink, non-safe tokens of the layer; equal scores are
    taken in (head, token) order.  k <= s' leaves nothing to allot: k per head."""
    budgets, _ = _adaptive_allot(lt, k, s, alpha)
    return budgets


def adaptive_cut_score(lt: np.ndarray, k: int, s: int, alpha: float):
    """The smallest score that `adaptive_budgets` admits in its layer-wide step (the score of
    the last of the R places), or None when that step has nothing to allot.  Tests use it to
    tell which tokens sit so close to the cut that fp32 scores may order them differently."""
    _, cut = _adaptive_allot(lt, k, s, alpha)
    return cut


def _adaptive_allot(lt: np.ndarray, k: int, s: int, alpha: float):
    lt = np.asarray(lt, dtype=np.float64)
    H, n = lt.shape
    if not (0 <= k <= n) or s < 0 or not (0.0 <= alpha <= 1.0):
        raise ValueError("need 0 <= k <= n, s >= 0, 0 <= alpha <= 1")
    sp = min(s, n)
    if k <= sp:
        return np.full(H, k, dtype=np.int64), None
    g = min(max(int(np.floor(alpha * k)) - sp, 0), n - sp)
    R = H * (k - sp) - H * g
    cand = lt[:, sp:]
    # rank of every non-sink token inside its head: larger score first, then lower index
    order = np.argsort(-cand, axis=1, kind="stable")
    rank = np.empty_like(order)
    rows = np.arange(H)[:, None]
    rank[rows, order] = np.arange(n - sp)[None, :]
    open_ = rank >= g                               # not covered by the safeguard
    head_of = np.broadcast_to(rows, cand.shape)[open_]        # (head, token) order
    picked = np.argsort(-cand[open_], kind="stable")[:R]
    extra = np.bincount(head_of[picked], minlength=H)
    cut = float(cand[open_][picked[-1]]) if R > 0 else None
    return (sp + g + extra).astype(np.int64), cut


def compact(K: np.ndarray, V: np.ndarray, S: np.ndarray):
    """Gather step of Algorithm 1: K'_i = K_i[S_i], V'_i = V_i[S_i], rows of the
    stored (original-type) arrays, bit for bit."""
    return K[S], V[S]


def compress_group(K: np.ndarray, V: np.ndarray, dtype: str, G,
                   k: int, s: int, source: str = "kv", projection: bool = True):
    """Whole of Algorithm 1 for one group.  K, V in storage form [n, d].
    Returns (lt, S, K', V')."""
    lt = scores(to_f64(K, dtype), to_f64(V, dtype), G, source, projection)
    S = select(lt, k, s)
    Kc, Vc = compact(K, V, S)
    return lt, S, Kc, Vc


def compress(K: np.ndarray, V: np.ndarray, dtype: str, seed: int, r: int,
             budgets: np.ndarray, s: int, source: str = "kv", projection: bool = True):
    """Algorithm 1 over a cache [layers, kv_heads, n, d] with one budget per
    (layer, head).  Returns (scores [L,H,n] float64, list of index arrays,
    offsets [L*H+1], packed K' [sum k, d], packed V' [sum k, d])."""
    L, H, n, d = K.shape
    budgets = np.asarray(budgets, dtype=np.int64).reshape(L * H)
    offsets = np.zeros(L * H + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(budgets)
    lt_all = np.empty((L, H, n), dtype=np.float64)
    idx = []
    Kp = np.empty((int(offsets[-1]), d), dtype=K.dtype)
    Vp = np.empty((int(offsets[-1]), d), dtype=V.dtype)
    for l in range(L):
        for h in range(H):
            G = sketch(seed, l, h, H, d, r, dtype) if projection else None
            lt, S, Kc, Vc = compress_group(K[l, h], V[l, h], dtype, G,
                                           int(budgets[l * H + h]), s, source, projection)
            lt_all[l, h] = lt
            idx.append(S)
            o = int(offsets[l * H + h])
            Kp[o:o + S.size] = Kc
            Vp[o:o + S.size] = Vc
    return lt_all, idx, offsets, Kp, Vp
