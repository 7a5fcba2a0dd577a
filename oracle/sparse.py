"""Sparsity-friendly layer: Stage 2 of the dynamic retrieval of Sec. 4.2
(approximate scores from the critical query channels and the critical key
cache, Top-K selection) and the exact attention over n_local + n_topk tokens
(Sec. 5.1, implementation paragraph).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings where the paper is silent:
  * The channel list is an input of Stage 2 (int32 [Hkv, d_s], ascending).  The
    paper re-selects it every step from |q_hat_i| * max|K_i| (Eq. 10, Stage 1):
    ``critical_channels`` is Eq. 10 for one query vector, ``select_channels``
    its grouped-query form in the pinned float32 order that the library takes.
  * Grouped-query heads in Stage 1: one channel list per KV head; the
    contribution of channel i is summed over the group's query heads,
        s_i = (((|q_0,i| + |q_1,i|) + ...) * max_t |K[t, i]|,
    each operation one float32 operation, ties to the lower channel.
  * Grouped-query heads: one Top-K index set per KV head; the group's score is
    the sum of its query heads' approximate scores.
  * Tokens resident on the GPU (the first n_sink and the last n_window) are not
    candidates, so sinks, Top-K and window are disjoint.
  * Top-K order: score descending, ties to the lower token index; the selected
    indices are returned ascending, padded with -1 to k.
  * The approximate score decides integers (the index set), so it is computed
    in the pinned float32 order below on both sides:
        a_j = (((p_0 + p_1) + p_2) + ... + p_{d_s-1}),  p_i = q_j[c_i] * K[t, c_i]
    (each product of two fp16 values is exact in float32), query heads j of the
    group ascending, S(t) = ((a_0 + a_1) + a_2) + ..., then S(t) + 0.0 so that
    -0 becomes +0.  No 1/sqrt(d) factor (it does not change the order).
"""
from __future__ import annotations

import numpy as np

from . import attention


def key_summary(k: np.ndarray, channels: np.ndarray) -> np.ndarray:
    """Critical key cache: the listed channels of every key.  k fp16 [Hkv, N, D],
    channels int [Hkv, d_s]  ->  fp16 [Hkv, N, d_s]."""
    return np.stack([k[h][:, channels[h]] for h in range(k.shape[0])])


def approx_scores(q: np.ndarray, summary: np.ndarray, channels: np.ndarray) -> np.ndarray:
    """float32 [Hkv, N]: pinned-order approximate scores (module docstring)."""
    assert q.dtype == np.float16 and summary.dtype == np.float16
    hq = q.shape[0]
    hkv, n, ds = summary.shape
    g = hq // hkv
    out = np.zeros((hkv, n), dtype=np.float32)
    for h in range(hkv):
        s32 = summary[h].astype(np.float32)                    # [N, d_s]
        total = None
        for j in range(h * g, (h + 1) * g):
            qc = q[j][channels[h]].astype(np.float32)          # [d_s]
            a = s32[:, 0] * qc[0]                               # exact product
            for i in range(1, ds):
                p = s32[:, i] * qc[i]                           # exact product
                a = a + p                                       # one RN32 add
            total = a if total is None else total + a           # one RN32 add
        out[h] = total + np.float32(0.0)
    return out


def topk_indices(scores: np.ndarray, k: int, lo: int, hi: int) -> tuple[np.ndarray, int]:
    """Exact Top-K of one head's scores over candidates t in [lo, hi).

    Order: score descending, then index ascending.  Returns (int32 [k] with the
    selected indices ascending then -1 padding, count)."""
    out = np.full(k, -1, dtype=np.int32)
    if hi <= lo or k <= 0:
        return out, 0
    cand = np.arange(lo, hi)
    order = np.argsort(-scores[lo:hi].astype(np.float64), kind="stable")
    k_eff = min(k, hi - lo)
    sel = np.sort(cand[order[:k_eff]])
    out[:k_eff] = sel
    return out, k_eff


def estimate_topk(q, summary, channels, n_tokens: int, *, top_k: int, n_sink: int, n_window: int):
    """Stage 2 of Sec. 4.2 for one sequence: (int32 [Hkv, top_k], int32 [Hkv])."""
    hkv = summary.shape[0]
    n = int(n_tokens)
    s = approx_scores(q, summary[:, :n], channels)
    lo, hi = min(n_sink, n), max(n - n_window, min(n_sink, n))
    idx = np.full((hkv, top_k), -1, dtype=np.int32)
    cnt = np.zeros(hkv, dtype=np.int32)
    for h in range(hkv):
        idx[h], cnt[h] = topk_indices(s[h], top_k, lo, hi)
    return idx, cnt


def attended_set(n_tokens: int, selected: np.ndarray, n_sink: int, n_window: int) -> np.ndarray:
    """Sinks [0, n_sink) U selected U window [N - n_window, N), deduplicated, ascending."""
    n = int(n_tokens)
    sinks = np.arange(0, min(n_sink, n))
    window = np.arange(max(n - n_window, min(n_sink, n)), n)
    sel = np.asarray(selected)
    sel = sel[sel >= 0]
    return np.unique(np.concatenate([sinks, sel, window])).astype(np.int64)


def sparse_attention(q, k, v, topk_idx, topk_count, n_tokens: int, sm_scale: float,
                     *, n_sink: int, n_window: int) -> np.ndarray:
    """Exact attention (Eq. 3) of every query head over its KV head's attended
    set, with the true fp16 K, V rows.  float64 [Hq, D]."""
    hq, d = q.shape
    hkv = k.shape[0]
    g = hq // hkv
    out = np.zeros((hq, d), dtype=np.float64)
    for h in range(hkv):
        rows = attended_set(n_tokens, topk_idx[h][: int(topk_count[h])], n_sink, n_window)
        o = attention.decode_attention(q[h * g:(h + 1) * g], k[h:h + 1, rows], v[h:h + 1, rows], sm_scale)
        out[h * g:(h + 1) * g] = o
    return out


def critical_channels(q_hat: np.ndarray, k: np.ndarray, n_channels: int) -> np.ndarray:
    """Stage 1 of Sec. 4.2, Eq. 10: s_i = |q_hat_i| * max_t |K[t, i]| per channel;
    the n_channels largest (ties to the lower channel), ascending.
    q_hat [D], k [N, D]  ->  int32 [n_channels]."""
    s = np.abs(np.asarray(q_hat, np.float64)) * np.abs(np.asarray(k, np.float64)).max(axis=0)
    order = np.argsort(-s, kind="stable")[:n_channels]
    return np.sort(order).astype(np.int32)


def channel_absmax(k: np.ndarray) -> np.ndarray:
    """max_t |K[t, i]| of Eq. 10 per KV head and channel (exact: a maximum of
    fp16 magnitudes).  k fp16 [Hkv, N, D] -> float32 [Hkv, D]; zeros for N = 0."""
    hkv, n, d = k.shape
    if n == 0:
        return np.zeros((hkv, d), np.float32)
    return np.abs(k.astype(np.float32)).max(axis=1)


def select_channels(q_hat: np.ndarray, k_absmax: np.ndarray, n_channels: int) -> np.ndarray:
    """Stage 1 of Sec. 4.2 (Eq. 10) for grouped-query heads, pinned float32 order
    (module docstring).  q_hat fp16 [Hq, D], k_absmax float32 [Hkv, D]
    ->  int32 [Hkv, n_channels], ascending."""
    assert q_hat.dtype == np.float16 and k_absmax.dtype == np.float32
    hq, d = q_hat.shape
    hkv = k_absmax.shape[0]
    g = hq // hkv
    out = np.zeros((hkv, n_channels), np.int32)
    for h in range(hkv):
        a = np.abs(q_hat[h * g].astype(np.float32))
        for j in range(h * g + 1, (h + 1) * g):
            a = a + np.abs(q_hat[j].astype(np.float32))          # one RN32 add
        s = a * k_absmax[h]                                       # one RN32 multiply
        order = np.argsort(-s.astype(np.float64), kind="stable")[:n_channels]
        out[h] = np.sort(order)
    return out
