"""Pins for the oracle's scoring steps (Algorithm 1: project, row-norm squared,
combine, normalise) against closed forms, textbook special cases, exact
leverage scores (Section 3.1) and brute force.  CPU only."""

import math

import numpy as np
import pytest

from oracle import curdkv_oracle as orc


def _rng(*k):
    return np.random.default_rng([7, *k])


# ---- exact leverage scores (Section 3.1) --------------------------------

@pytest.mark.parametrize("n,d", [(8, 3), (64, 8), (40, 5)])
def test_exact_leverage_svd_equals_qr_and_invariants(n, d):
    A = _rng(n, d).standard_normal((n, d))
    lev = orc.leverage_exact(A)
    Q, _ = np.linalg.qr(A)                       # hat matrix diag via QR
    assert np.allclose(lev, np.sum(Q * Q, axis=1), atol=1e-12)
    assert np.all(lev >= -1e-15) and np.all(lev <= 1 + 1e-12)
    # sums to rank(A) = d  (the paper's "= n" cannot hold: U has rank(A) columns)
    assert abs(lev.sum() - d) < 1e-10
    # hat-matrix definition, written out
    Hm = A @ np.linalg.inv(A.T @ A) @ A.T
    assert np.allclose(lev, np.diag(Hm), atol=1e-10)


def test_exact_leverage_rank_deficient():
    rng = _rng(1)
    B = rng.standard_normal((30, 3))
    A = np.concatenate([B, B @ rng.standard_normal((3, 4))], axis=1)   # 30 x 7, rank 3
    lev = orc.leverage_exact(A)
    assert abs(lev.sum() - 3.0) < 1e-9
    assert np.all(lev <= 1 + 1e-12)
    # a row that alone spans a direction has leverage one
    C = np.zeros((5, 2)); C[0, 0] = 3.0; C[1:, 1] = [1, 1, 1, 1]
    assert np.allclose(orc.leverage_exact(C), [1, .25, .25, .25, .25])


# ---- projection and row-norm squared ------------------------------------

def test_identity_sketch_is_plain_row_norm_squared():
    # the no-projection ablation (appendix, ablation study): scores on the raw rows
    A = _rng(2).standard_normal((50, 16))
    got = orc.row_norm_sq(orc.project(A, np.eye(16)))
    assert np.allclose(got, np.linalg.norm(A, axis=1) ** 2, rtol=1e-13)


def test_projection_brute_force_loops():
    rng = _rng(3)
    n, d, r = 5, 4, 3
    A, G = rng.standard_normal((n, d)), rng.standard_normal((d, r))
    want = np.zeros(n)
    for j in range(n):
        for c in range(r):
            y = 0.0
            for i in range(d):
                y += A[j, i] * G[i, c]          # (A G)[j, c]
            want[j] += y * y
    assert np.allclose(orc.row_norm_sq(orc.project(A, G)), want, rtol=1e-13)
    # G^T in place of G has the wrong shape and must not be silently accepted
    with pytest.raises(ValueError):
        orc.project(A, G.T)


@pytest.mark.parametrize("r", [8, 32, 64])
def test_sketched_score_is_chi_square(r):
    # G_ij ~ N(0, 1/r)  =>  ||a G||^2 / ||a||^2 ~ chi^2_r / r : mean 1, variance 2/r
    d, T = 128, 2400
    a = _rng(4, r).standard_normal((3, d)) * np.array([[1.0], [7.0], [0.01]])
    na = np.sum(a * a, axis=1)
    ratios = np.empty((T, 3))
    for t in range(T):
        G = orc.sketch(1000 + t, 0, 0, 1, d, r, "fp32")
        ratios[t] = orc.row_norm_sq(orc.project(a, G)) / na
    se_mean = math.sqrt(2.0 / r / T)
    assert np.all(np.abs(ratios.mean(0) - 1.0) < 5 * se_mean)
    var = ratios.var(0, ddof=1)
    # var of sample variance of chi2_r/r: (2/r)^2 * (2/(T-1) + 12/(r T))
    se_var = (2.0 / r) * math.sqrt(2.0 / (T - 1) + 12.0 / (r * T))
    assert np.all(np.abs(var - 2.0 / r) < 5 * se_var)


def test_converges_to_exact_leverage_on_orthonormal_columns():
    # A^T A = I  =>  ||A[j]||^2 is the exact leverage score; sketched score -> it as r grows
    n, d = 256, 16
    A, _ = np.linalg.qr(_rng(5).standard_normal((n, d)))
    lev = orc.leverage_exact(A)
    assert np.allclose(lev, np.sum(A * A, axis=1), atol=1e-12)
    rs = [8, 32, 128, 512, 2048]
    err = []
    for r in rs:
        e = []
        for t in range(8):
            G = orc.sketch(77 + t, 0, 0, 1, d, r, "fp32")
            s = orc.row_norm_sq(orc.project(A, G))
            e.append(np.sqrt(np.mean((s / lev - 1.0) ** 2)))
        err.append(np.mean(e))
    err = np.array(err)
    assert np.allclose(err, np.sqrt(2.0 / np.array(rs)), rtol=0.15)
    slope = np.polyfit(np.log(rs), np.log(err), 1)[0]
    assert abs(slope + 0.5) < 0.05


def test_general_matrix_limit_is_row_norm_not_leverage():
    # without whitening the large-r limit is ||A[j]||^2; it differs from the exact
    # leverage score unless the columns are orthonormal
    n, d, r = 64, 8, 4096
    A = _rng(6).standard_normal((n, d)) * np.linspace(1, 6, d)
    G = orc.sketch(3, 0, 0, 1, d, r, "fp32")
    s = orc.row_norm_sq(orc.project(A, G))
    rn = np.sum(A * A, axis=1)
    assert np.sqrt(np.mean((s / rn - 1) ** 2)) < 3 * math.sqrt(2.0 / r)
    lev = orc.leverage_exact(A)
    assert np.max(np.abs(s / s.sum() - lev / lev.sum())) > 1e-3


# ---- combine + normalise -------------------------------------------------

def test_combine_is_a_product_hand_example():
    K = np.array([[1., 0.], [0., 2.], [3., 0.], [0., 0.]])
    V = np.array([[2., 0.], [0., 1.], [0., 0.], [1., 2.]])
    lk, lv, lkv = orc.scores_unnormalised(K, V, np.eye(2))
    assert np.array_equal(lk, [1, 4, 9, 0]) and np.array_equal(lv, [4, 1, 0, 5])
    assert np.array_equal(lkv, [4, 4, 0, 0])
    assert np.array_equal(orc.scores(K, V, np.eye(2)), [0.5, 0.5, 0, 0])


def test_normalise_invariants_and_scale_invariance():
    rng = _rng(8)
    K, V = rng.standard_normal((200, 128)), rng.standard_normal((200, 128))
    G = orc.sketch(9, 0, 0, 1, 128, 32, "bf16")
    lt = orc.scores(K, V, G)
    assert abs(lt.sum() - 1.0) < 1e-12 and np.all(lt >= 0)
    assert np.allclose(orc.scores(-3.5 * K, 0.02 * V, G), lt, rtol=1e-12)
    z = orc.scores(np.zeros((7, 128)), V[:7], G)
    assert np.allclose(z, 1.0 / 7)
    # the sum runs over all rows, the first s included
    lk, lv, lkv = orc.scores_unnormalised(K, V, G)
    assert np.allclose(lt, lkv / lkv.sum(), rtol=1e-13)
    assert np.allclose(lt[4:].sum(), 1.0 - lt[:4].sum())


def test_same_sketch_for_keys_and_values():
    # K == V  =>  lKV = lK^2, which needs the same G on both sides
    rng = _rng(9)
    K = rng.standard_normal((100, 128))
    G = orc.sketch(10, 0, 0, 1, 128, 32, "fp32")
    lk, lv, lkv = orc.scores_unnormalised(K, K, G)
    assert np.array_equal(lk, lv) and np.allclose(lkv, lk ** 2)
    assert np.array_equal(np.argsort(-orc.scores(K, K, G), kind="stable"),
                          np.argsort(-lk, kind="stable"))


def test_constant_value_rows_reduce_to_key_only_ranking():
    rng = _rng(10)
    K = rng.standard_normal((100, 128))
    V = np.ones((100, 128))
    G = orc.sketch(11, 0, 0, 1, 128, 32, "fp32")
    lk, lv, _ = orc.scores_unnormalised(K, V, G)
    assert np.allclose(lv, lv[0])
    assert np.allclose(orc.scores(K, V, G), lk / lk.sum(), rtol=1e-12)


def test_scores_permutation_equivariant():
    rng = _rng(11)
    K, V = rng.standard_normal((64, 128)), rng.standard_normal((64, 128))
    G = orc.sketch(12, 0, 0, 1, 128, 64, "bf16")
    p = rng.permutation(64)
    assert np.allclose(orc.scores(K[p], V[p], G), orc.scores(K, V, G)[p], rtol=1e-12)


def test_bf16_inputs_are_upcast_exactly():
    x = _rng(12).standard_normal((16, 128)).astype(np.float32)
    bits = orc.f32_to_bf16_bits(x)
    up = orc.to_f64(bits, "bf16")
    assert np.array_equal(orc.f32_to_bf16_bits(up.astype(np.float32)), bits)
    assert np.max(np.abs(up - x) / np.abs(x)) <= 2.0 ** -8


def test_fold_gqa():
    a = _rng(13).random(50)
    assert np.array_equal(orc.fold_gqa(np.stack([a, a, a, a])), a)     # CurDKV: identity
    assert np.array_equal(orc.fold_gqa(np.array([[1., 2.], [3., 6.]])), [2., 4.])


# ---- ablation variants (appendix, "Ablation Study") ------------------------------

def test_single_source_scores():
    rng = _rng(14)
    K, V = rng.standard_normal((80, 128)), rng.standard_normal((80, 128)) * 3.0
    G = orc.sketch(13, 0, 0, 1, 128, 32, "fp32")
    lk, lv, lkv = orc.scores_unnormalised(K, V, G)
    assert np.allclose(orc.scores(K, V, G, source="k"), lk / lk.sum(), rtol=1e-13)
    assert np.allclose(orc.scores(K, V, G, source="v"), lv / lv.sum(), rtol=1e-13)
    assert np.allclose(orc.scores(K, V, G, source="kv"), lkv / lkv.sum(), rtol=1e-13)
    # key-only scores ignore V altogether, value-only ignore K
    assert np.array_equal(orc.scores(K, 7 * V + 1, G, source="k"), orc.scores(K, V, G, source="k"))
    assert np.array_equal(orc.scores(K - 2, V, G, source="v"), orc.scores(K, V, G, source="v"))
    # the product is not either factor
    assert not np.allclose(orc.scores(K, V, G), orc.scores(K, V, G, source="k"), rtol=1e-3)
    with pytest.raises(ValueError):
        orc.scores(K, V, G, source="q")


def test_no_projection_is_raw_row_norm():
    rng = _rng(15)
    K, V = rng.standard_normal((60, 128)), rng.standard_normal((60, 128))
    nk, nv = np.linalg.norm(K, axis=1) ** 2, np.linalg.norm(V, axis=1) ** 2
    assert np.allclose(orc.scores(K, V, None, "k", projection=False), nk / nk.sum(), rtol=1e-13)
    assert np.allclose(orc.scores(K, V, None, "v", projection=False), nv / nv.sum(), rtol=1e-13)
    assert np.allclose(orc.scores(K, V, None, "kv", projection=False), nk * nv / np.sum(nk * nv), rtol=1e-13)
    # same as projecting through the identity
    assert np.allclose(orc.scores(K, V, None, projection=False), orc.scores(K, V, np.eye(128)), rtol=1e-13)
    # and the sketched scores scatter around it with the chi-square spread sqrt(2/r) per factor
    G = orc.sketch(14, 0, 0, 1, 128, 64, "fp32")
    lk, _, _ = orc.scores_unnormalised(K, V, G)
    assert abs(np.sqrt(np.mean((lk / nk - 1) ** 2)) - math.sqrt(2 / 64)) < 0.06
