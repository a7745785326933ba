"""Eviction loss of a KV selection, on synthetic queries (CPU, float64).

Test infrastructure, like the rest of this package: a small evaluator of what the
selection is FOR.  The paper motivates CurDKV by the change in the attention
output softmax(Q K^T) V when tokens are evicted (Figures 1 and 2, Lemma 1 of
Section 3.1); real queries need model weights, so the tests draw synthetic ones.
"""

from __future__ import annotations

import numpy as np


def softmax_rows(X: np.ndarray) -> np.ndarray:
    X = X - X.max(axis=1, keepdims=True)
    E = np.exp(X)
    return E / E.sum(axis=1, keepdims=True)


def attention_output(Q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """softmax(Q K^T / sqrt(d)) V for Q [m, d], K, V [n, d]."""
    d = Q.shape[1]
    return softmax_rows(Q @ K.T / np.sqrt(d)) @ V


def eviction_loss(Q: np.ndarray, K: np.ndarray, V: np.ndarray, S: np.ndarray) -> float:
    """|| attn(Q, K, V) - attn(Q, K[S], V[S]) ||_F : the kept tokens S are all the
    model attends to after compression."""
    return float(np.linalg.norm(attention_output(Q, K, V) - attention_output(Q, K[S], V[S])))


def lemma1_sides(Q: np.ndarray, K: np.ndarray, V: np.ndarray, S: np.ndarray):
    """Both sides of Lemma 1 (Section 3.1) as stated: K', V' are K, V with the rows
    outside S zeroed out (same shape), no 1/sqrt(d) scaling:
        || sm(Q K^T) V - sm(Q K'^T) V' ||_F  <=  sqrt(n) ||V - V'||_F + 2 sqrt(n) ||V'||_F ."""
    n = K.shape[0]
    keep = np.zeros(n, dtype=bool)
    keep[S] = True
    Kp, Vp = K * keep[:, None], V * keep[:, None]
    lhs = np.linalg.norm(softmax_rows(Q @ K.T) @ V - softmax_rows(Q @ Kp.T) @ Vp)
    rhs = np.sqrt(n) * np.linalg.norm(V - Vp) + 2.0 * np.sqrt(n) * np.linalg.norm(Vp)
    return float(lhs), float(rhs)


def selection_policies(K: np.ndarray, V: np.ndarray, scores_kv: np.ndarray, k: int, s: int,
                       rng: np.random.Generator) -> dict:
    """Index sets of k tokens (the first s always kept) under the selection the paper proposes
    and under the simple policies it is compared with in spirit: `curdkv` takes the given
    CurDKV scores, `key_norm` / `value_norm` the squared row norms of K / V alone, `random` a
    uniform draw.  Ascending indices.  (The paper's baselines proper -- SnapKV, ChunkKV, Knorm,
    StreamingLLM -- need attention weights or their own code and are out of scope.)"""
    n = K.shape[0]
    s = min(s, k, n)

    def top(score):
        order = np.argsort(-score[s:], kind="stable")[: k - s] + s
        return np.sort(np.concatenate([np.arange(s), order]))

    return {
        "curdkv": top(np.asarray(scores_kv, dtype=np.float64)),
        "key_norm": top(np.sum(K * K, axis=1)),
        "value_norm": top(np.sum(V * V, axis=1)),
        "random": np.sort(np.concatenate([np.arange(s), rng.choice(np.arange(s, n), size=k - s, replace=False)])),
    }


def compare_policies(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scores_kv: np.ndarray, k: int, s: int,
                     rng: np.random.Generator) -> dict:
    """Eviction loss || attn(Q,K,V) - attn(Q,K[S],V[S]) ||_F of each policy's index set."""
    return {name: eviction_loss(Q, K, V, S) for name, S in selection_policies(K, V, scores_kv, k, s, rng).items()}
