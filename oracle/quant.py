"""Uniform asymmetric quantizer of the KV cache (Sec. 2.2, Eq. 4) with the static
policy of Sec. 4.3: keys per channel, values per token, fp16 zero-point and
scaler (Sec. 4.4).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings where the paper is silent:
  * The newest tokens stay fp16 (a per-channel key group needs ``g`` complete
    tokens): with residual ``W`` the first Nq = g*floor((N-W)/g) tokens are
    quantized (0 if N < W), the last N-Nq in [W, W+g-1] are not.
  * z = min X is stored as is (it is an fp16 value).  The scaler is computed
    in float32, s32 = (f32(max) - f32(min)) / f32(2^b - 1), and stored rounded
    to nearest-even fp16.  Codes use the *stored* s and z so that
    dequantization is self-consistent:
        code = clamp(rint((f32(x) - f32(z)) / f32(s)), 0, 2^b - 1),
    each operation a single float32 operation, rint = round half to even.
  * A group whose stored scaler is 0 gets code 0 everywhere (dequant = z).
  * bits == 16 is a passthrough used by tests: "codes" are the fp16 bit
    patterns and dequantization returns the input.

The float32 steps are the ones that decide an integer (the code) or a stored
fp16 value (the scaler): both implementations must take them in the same
precision for a bit-exact comparison to be meaningful.  Everything downstream
(dequantization, attention) is float64.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def partition(n_tokens: int, residual: int, group: int) -> tuple[int, int]:
    """(Nq, R): number of quantized tokens and of fp16 tail tokens."""
    n, w, g = int(n_tokens), int(residual), int(group)
    nq = g * ((n - w) // g) if n >= w else 0
    return nq, n - nq


def _scale_zero(mn: np.ndarray, mx: np.ndarray, bits: int) -> tuple[np.ndarray, np.ndarray]:
    """Eq. 4's z = min X and s = (max X - min X) / (2^b - 1), in the pinned
    float32 order, returned as fp16."""
    assert mn.dtype == np.float16 and mx.dtype == np.float16
    rng32 = mx.astype(np.float32) - mn.astype(np.float32)          # one RN32 op
    s32 = rng32 / np.float32((1 << bits) - 1)                      # one RN32 op
    with np.errstate(over="ignore"):
        s16 = s32.astype(np.float16)                               # RNE to fp16
    return s16, mn.copy()


def quantize_lastaxis(x: np.ndarray, bits: int) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Quantize fp16 ``x`` with one (scale, zero) per slice along the last axis.

    Returns (codes uint8 same shape as x, scale fp16 x.shape[:-1], zero fp16
    x.shape[:-1]).  Eq. 4 applied to each group X = x[..., :].
    """
    assert x.dtype == np.float16
    assert 1 <= bits <= 8
    qmax = (1 << bits) - 1
    mn = x.min(axis=-1)
    mx = x.max(axis=-1)
    s16, z16 = _scale_zero(mn, mx, bits)
    s32 = s16.astype(np.float32)[..., None]
    z32 = z16.astype(np.float32)[..., None]
    diff = x.astype(np.float32) - z32                               # one RN32 op
    with np.errstate(divide="ignore", invalid="ignore"):
        t = diff / s32                                              # one RN32 op
    code = np.clip(np.rint(t), 0, qmax)
    code = np.where(s32 == 0, 0, code)
    return code.astype(np.uint8), s16, z16


@dataclass
class QuantizedKV:
    """Logical (layout-free) quantized cache of one sequence of one layer."""

    bits: int
    group: int
    n_quant: int                 # Nq
    k_codes: np.ndarray          # uint8 [Hkv, Nq, D]   (uint16 bit patterns if bits == 16)
    k_scale: np.ndarray          # fp16  [Hkv, Nq/g, D] per token-group, per channel
    k_zero: np.ndarray           # fp16  [Hkv, Nq/g, D]
    v_codes: np.ndarray          # uint8 [Hkv, Nq, D]
    v_scale: np.ndarray          # fp16  [Hkv, Nq, D/g] per token, per channel-group
    v_zero: np.ndarray           # fp16  [Hkv, Nq, D/g]
    k_resid: np.ndarray          # fp16  [Hkv, R, D] newest tokens, oldest first
    v_resid: np.ndarray          # fp16  [Hkv, R, D]


def quantize_kv(k: np.ndarray, v: np.ndarray, *, bits: int, group: int, residual: int) -> QuantizedKV:
    """Static policy of Sec. 4.3: K per channel over ``group`` tokens, V per token
    over ``group`` channels, both with Eq. 4; tail kept fp16."""
    assert k.dtype == np.float16 and v.dtype == np.float16 and k.shape == v.shape
    hkv, n, d = k.shape
    g = int(group)
    assert d % g == 0
    nq, _ = partition(n, residual, g)
    kq, vq = k[:, :nq], v[:, :nq]
    if bits == 16:
        return QuantizedKV(16, g, nq, kq.view(np.uint16).copy(),
                           np.zeros((hkv, nq // g, d), np.float16), np.zeros((hkv, nq // g, d), np.float16),
                           vq.view(np.uint16).copy(),
                           np.zeros((hkv, nq, d // g), np.float16), np.zeros((hkv, nq, d // g), np.float16),
                           k[:, nq:].copy(), v[:, nq:].copy())
    # K: group over tokens -> bring the token-in-group axis last.
    kg = kq.reshape(hkv, nq // g, g, d).transpose(0, 1, 3, 2)        # [Hkv, J, D, g]
    kc, ks, kz = quantize_lastaxis(np.ascontiguousarray(kg), bits)
    k_codes = kc.transpose(0, 1, 3, 2).reshape(hkv, nq, d)
    # V: group over channels.
    vg = vq.reshape(hkv, nq, d // g, g)
    vc, vs, vz = quantize_lastaxis(np.ascontiguousarray(vg), bits)
    v_codes = vc.reshape(hkv, nq, d)
    return QuantizedKV(bits, g, nq, np.ascontiguousarray(k_codes), ks, kz,
                       np.ascontiguousarray(v_codes), vs, vz,
                       k[:, nq:].copy(), v[:, nq:].copy())


def dequantize_k(c: QuantizedKV) -> np.ndarray:
    """float64 [Hkv, Nq, D]: code * s + z with the stored fp16 s, z (exact in float64)."""
    if c.bits == 16:
        return c.k_codes.view(np.float16).astype(np.float64)
    s = np.repeat(c.k_scale.astype(np.float64), c.group, axis=1)
    z = np.repeat(c.k_zero.astype(np.float64), c.group, axis=1)
    return c.k_codes.astype(np.float64) * s + z


def dequantize_v(c: QuantizedKV) -> np.ndarray:
    """float64 [Hkv, Nq, D]."""
    if c.bits == 16:
        return c.v_codes.view(np.float16).astype(np.float64)
    s = np.repeat(c.v_scale.astype(np.float64), c.group, axis=2)
    z = np.repeat(c.v_zero.astype(np.float64), c.group, axis=2)
    return c.v_codes.astype(np.float64) * s + z


def table2_quant_elements(n_tokens: int, n_heads: int, head_dim: int, n_layers: int,
                          bits: int, group: int) -> float:
    """Sec. 4.4, Table 2, row for quantization-friendly layers, generalised from
    1 bit to b bits: fp16-element count 2 * l_q * n * h * d_h * (b/16 + 2/g)
    (codes at b/16 of an fp16 element, plus one zero-point and one scaler per
    group of g elements).  The table's own entry is the b = 1 case."""
    return 2.0 * n_layers * n_tokens * n_heads * head_dim * (bits / 16.0 + 2.0 / group)


def table2_sparse_elements(n_tokens: int, n_heads: int, n_channels: int) -> float:
    """Sec. 4.4, Table 2, row for sparsity-friendly layers: 2 * n * h * d_s
    fp16 elements (two buffers of the critical key cache of one layer)."""
    return 2.0 * n_tokens * n_heads * n_channels
