"""Synthetic decode-time KV workloads shaped like Llama-3.1-8B attention.

The paper evaluates on long-context suites with trained weights; neither is
available offline, so every test and benchmark uses tensors drawn here.  The
value structure follows what the paper reports about real caches (Fig. 2 of
Sec. 3 and the outlier appendix): a few key/query channels carry outliers, the
value cache has none, and a handful of tokens dominate the attention of
sparsity-friendly layers.

Recipe (all draws from numpy's PCG64 seeded with [config, layer, seq, tensor]):
  * q [Hq, D], k [Hkv, N, D], v [Hkv, N, D] ~ N(0, 1), drawn in float32 and
    rounded once to float16;
  * per KV head, 4 channels chosen without replacement; those key channels are
    multiplied by 10 for every token;
  * per KV head, 8 "dominant" token positions chosen without replacement from
    the candidate range [n_sink, N - n_window); their key rows are replaced by
    0.8 * q_dir + 0.2 * noise with q_dir = sqrt(D) * m / |m|, m the mean of the
    head group's query vectors (times ``dominance_gain``), noise ~ N(0,1)^D.

No arithmetic of the method itself lives here.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class HeadShape:
    n_q_heads: int = 32
    n_kv_heads: int = 8
    head_dim: int = 128

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


#: Attention shape of Llama-3.1-8B (32 query heads, 8 KV heads; Table of model
#: configurations in the paper's appendix) with head_dim 128.
LLAMA31_8B = HeadShape(32, 8, 128)

_T_Q, _T_K, _T_V, _T_OUTLIER, _T_DOMINANT, _T_NOISE, _T_LEN = range(7)


@dataclass
class LayerInputs:
    """One layer's decode-step inputs for one sequence."""

    q: np.ndarray  # float16 [Hq, D]
    k: np.ndarray  # float16 [Hkv, N, D]
    v: np.ndarray  # float16 [Hkv, N, D]
    outlier_channels: np.ndarray  # int64 [Hkv, 4]
    dominant_tokens: np.ndarray  # int64 [Hkv, n_dominant] (may be empty)
    meta: dict = field(default_factory=dict)


def _rng(config: int, layer: int, seq: int, tensor: int) -> np.random.Generator:
    return np.random.default_rng([config, layer, seq, tensor])


def make_layer(
    n_tokens: int,
    *,
    shape: HeadShape = LLAMA31_8B,
    config: int = 0,
    layer: int = 0,
    seq: int = 0,
    n_outlier: int = 4,
    outlier_gain: float = 10.0,
    n_dominant: int = 8,
    dominance_gain: float = 1.0,
    n_sink: int = 4,
    n_window: int = 64,
) -> LayerInputs:
    """Draw q, k, v for one layer of one sequence (see module docstring)."""
    hq, hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    g = shape.group
    n = int(n_tokens)

    q32 = _rng(config, layer, seq, _T_Q).standard_normal((hq, d), dtype=np.float32)
    k32 = _rng(config, layer, seq, _T_K).standard_normal((hkv, n, d), dtype=np.float32)
    v32 = _rng(config, layer, seq, _T_V).standard_normal((hkv, n, d), dtype=np.float32)

    r_out = _rng(config, layer, seq, _T_OUTLIER)
    outliers = np.stack(
        [np.sort(r_out.choice(d, size=n_outlier, replace=False)) for _ in range(hkv)]
    ) if n_outlier > 0 else np.zeros((hkv, 0), dtype=np.int64)
    for h in range(hkv):
        k32[h][:, outliers[h]] *= np.float32(outlier_gain)

    lo, hi = n_sink, n - n_window
    n_dom = n_dominant if hi - lo >= n_dominant else 0
    dominant = np.zeros((hkv, n_dom), dtype=np.int64)
    if n_dom > 0:
        r_dom = _rng(config, layer, seq, _T_DOMINANT)
        r_noise = _rng(config, layer, seq, _T_NOISE)
        for h in range(hkv):
            pos = np.sort(r_dom.choice(hi - lo, size=n_dom, replace=False) + lo)
            dominant[h] = pos
            m = q32[h * g:(h + 1) * g].astype(np.float64).mean(axis=0)
            q_dir = np.sqrt(d) * m / np.linalg.norm(m) * dominance_gain
            noise = r_noise.standard_normal((n_dom, d))
            k32[h][pos] = (0.8 * q_dir[None, :] + 0.2 * noise).astype(np.float32)

    return LayerInputs(
        q=q32.astype(np.float16),
        k=k32.astype(np.float16),
        v=v32.astype(np.float16),
        outlier_channels=outliers.astype(np.int64),
        dominant_tokens=dominant,
        meta=dict(n_tokens=n, config=config, layer=layer, seq=seq,
                  n_sink=n_sink, n_window=n_window),
    )


def static_channels(k: np.ndarray, n_channels: int) -> np.ndarray:
    """Channel list used as the key summary: per KV head the ``n_channels``
    channels with the largest mean |k| over all tokens (float64 mean, ties to the
    lower channel), returned ascending as int32 [Hkv, n_channels].

    This is input preparation (which columns of K are kept on the GPU), not part
    of the scored arithmetic: the list is handed to both implementations.
    """
    mean_abs = np.abs(k.astype(np.float64)).mean(axis=1)  # [Hkv, D]
    order = np.argsort(-mean_abs, axis=1, kind="stable")[:, :n_channels]
    return np.sort(order, axis=1).astype(np.int32)


def ragged_lengths(batch: int, lo: int, hi: int, *, config: int = 4) -> np.ndarray:
    """Sequence lengths for the batched configuration: uniform in [lo, hi]."""
    r = _rng(config, 0, 0, _T_LEN)
    return r.integers(lo, hi + 1, size=batch).astype(np.int32)
