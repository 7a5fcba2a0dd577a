"""Offline identification (Sec. 4.1): the dense preference score of a layer
(Eq. 6-8) and the layer classification (Eq. 9), in float64.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings where the paper is silent:
  * Eq. 6 is taken as printed: every one of the n_q most recent query vectors
    attends to all n keys of the prompt (no causal mask is written there).
  * Grouped-query heads: query head j uses the keys of KV head j // (Hq // Hkv),
    as in Eq. 3; one score per query head.
  * "Top_k" of a row with fewer than k entries takes all of them (the score of
    that row is then 0).
  * Eq. 9 compares "the" score of a layer with tau.  With tau = 0.2 (Sec. 5.1) and
    Eq. 8 growing with n_q, the comparison is read per query row and averaged:
    P_l = mean over heads of P_head / n_q, the average attention mass that lies
    outside the top-k keys.
"""
from __future__ import annotations

import numpy as np


def dense_preference(q_last: np.ndarray, k: np.ndarray, top_k: int, sm_scale: float) -> np.ndarray:
    """Eq. 6-8 per query head.  q_last [n_q, Hq, D], k [Hkv, n, D] (any real
    dtype)  ->  float64 [Hq]:  P = n_q - sum over rows of the k largest entries
    of softmax(q K^T * sm_scale)."""
    q = np.asarray(q_last, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    n_q, hq, _ = q.shape
    hkv, n, _ = kk.shape
    g = hq // hkv
    out = np.zeros(hq, dtype=np.float64)
    for j in range(hq):
        logits = (q[:, j] @ kk[j // g].T) * float(sm_scale)          # [n_q, n]
        logits -= logits.max(axis=1, keepdims=True)
        a = np.exp(logits)
        a /= a.sum(axis=1, keepdims=True)                             # Eq. 6
        kk_eff = min(int(top_k), n)
        top = np.sort(a, axis=1)[:, n - kk_eff:]                      # Eq. 7: the k largest of every row
        out[j] = n_q - top.sum()                                      # Eq. 8
    return out


def layer_score(p_heads: np.ndarray, n_q: int) -> float:
    """The score Eq. 9 compares with tau: mean over heads of P / n_q."""
    return float(np.mean(np.asarray(p_heads, dtype=np.float64)) / n_q)


def classify(p_heads: np.ndarray, n_q: int, tau: float) -> str:
    """Eq. 9."""
    return "quantization-friendly" if layer_score(p_heads, n_q) > tau else "sparsity-friendly"
