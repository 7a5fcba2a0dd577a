"""Decode attention (Sec. 2.1, Eq. 3) in float64, over a dequantized cache
(Sec. 4.3) and with the split-K softmax merge used to check chunked kernels.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).
"""
from __future__ import annotations

import numpy as np

from . import quant


def decode_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, sm_scale: float) -> np.ndarray:
    """Eq. 3 for one decode step with grouped-query heads.

    q [Hq, D]; k, v [Hkv, N, D] (any real dtype); query head i reads KV head
    i // (Hq // Hkv).  a = softmax(q K^T * sm_scale), o = a V.  float64 [Hq, D].
    An empty cache (N == 0) gives zeros.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    hq, d = q.shape
    hkv, n, _ = k.shape
    g = hq // hkv
    out = np.zeros((hq, d), dtype=np.float64)
    if n == 0:
        return out
    for i in range(hq):
        h = i // g
        logits = (k[h] @ q[i]) * float(sm_scale)
        logits -= logits.max()
        w = np.exp(logits)
        out[i] = (w @ v[h]) / w.sum()
    return out


def quant_attention(q: np.ndarray, cache: quant.QuantizedKV, sm_scale: float) -> np.ndarray:
    """Attention of a quantization-friendly layer: Eq. 3 over the dequantized
    codes (code*s+z, Eq. 4 inverted) followed by the fp16 tail, one softmax
    over all N tokens."""
    k = np.concatenate([quant.dequantize_k(cache), cache.k_resid.astype(np.float64)], axis=1)
    v = np.concatenate([quant.dequantize_v(cache), cache.v_resid.astype(np.float64)], axis=1)
    return decode_attention(q, k, v, sm_scale)


def partial_attention(q_i: np.ndarray, k: np.ndarray, v: np.ndarray, sm_scale: float):
    """(m, l, o) of one chunk for one query head: m = max logit,
    l = sum exp(logit - m), o = sum exp(logit - m) * v.  Empty chunk: (-inf, 0, 0)."""
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if k.shape[0] == 0:
        return -np.inf, 0.0, np.zeros(v.shape[-1])
    logits = (k @ np.asarray(q_i, dtype=np.float64)) * float(sm_scale)
    m = logits.max()
    w = np.exp(logits - m)
    return m, w.sum(), w @ v


def merge_partials(parts) -> np.ndarray:
    """Log-sum-exp merge of per-chunk (m, l, o): m* = max m_i,
    l* = sum l_i e^{m_i - m*}, o* = sum o_i e^{m_i - m*}; result o*/l*."""
    ms = np.array([p[0] for p in parts], dtype=np.float64)
    m_star = ms.max()
    if not np.isfinite(m_star):
        return np.zeros_like(parts[0][2])
    l_star = 0.0
    o_star = np.zeros_like(parts[0][2], dtype=np.float64)
    for m, l, o in parts:
        if l == 0.0:
            continue
        w = np.exp(m - m_star)
        l_star += l * w
        o_star += o * w
    return o_star / l_star


def max_rel_err(out: np.ndarray, ref: np.ndarray) -> float:
    """Error metric of the attention outputs: per query-head vector,
    max_c |out - ref| / max_c |ref|; the maximum over heads is returned."""
    out = np.asarray(out, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(out - ref).max(axis=-1)
    den = np.abs(ref).max(axis=-1)
    den = np.where(den == 0, 1.0, den)
    return float((num / den).max())


def elementwise_rel_err(out: np.ndarray, ref: np.ndarray, floor: float = 2e-3) -> float:
    """Reported beside max_rel_err (never asserted): per query-head vector,
    max_c |out - ref| / max(|ref_c|, floor * rms_c(ref)); the maximum over heads is
    returned.  The floor keeps channels whose reference value is nearly zero from
    dominating; a head whose reference is all zero uses a denominator of 1."""
    out = np.asarray(out, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt((ref * ref).mean(axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref), float(floor) * rms)
    den = np.where(den == 0, 1.0, den)
    return float((np.abs(out - ref) / den).max())
