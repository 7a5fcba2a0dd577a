"""Physical layout of the packed quantized cache, written from the layout
description in include/tkv.h (an interface, not arithmetic of the method) so
that tests can turn the library's packed words back into logical codes and
compare them bit for bit with oracle/quant.py.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

All arrays are per KV head and per token group j = t // 32 (g = 32 tokens,
D = 128 channels).  ``t`` below is the token index inside its group, ``c`` the
channel.  A code occupies ``bits`` consecutive bits, least significant first,
at field F of a little-endian 32-bit word.

K codes, 2 bit:  word = 4*lane + 2*tau + wd, field F = f + 8*e
    r = 4*(t//8) + t%4, tau = (t%8)//4, lane = r + 16*((c%32)//8)
    wd = c//64, f = (c%8)//2 + 4*((c//32)%2), e = c%2
K codes, 4 bit:  word = 256*tau + 4*lane + c//32, field F = (c%8)//2 + 4*(c%2)
V codes, 2 bit:  word = 4*lane + wd, field F = f + 8*e
    lane = c%16 + 16*(t//8), wd = c//32, f = (t%8)//2 + 4*((c//16)%2), e = t%2
V codes, 4 bit:  word = 256*(c//64) + 4*lane + (c//16)%4, field F = (t%8)//2 + 4*(t%2)
K scale / zero:  fp16 [group][c]
V scale / zero:  fp16 [group][u][t]   (u = channel group c // 32)
"""
from __future__ import annotations

import numpy as np

G = 32
D = 128


def _k_pos(bits: int):
    t = np.arange(G)[:, None]
    c = np.arange(D)[None, :]
    r = 4 * (t // 8) + t % 4
    tau = (t % 8) // 4
    lane = r + 16 * ((c % 32) // 8)
    if bits == 2:
        word = 4 * lane + 2 * tau + c // 64
        field = (c % 8) // 2 + 4 * ((c // 32) % 2) + 8 * (c % 2)
    elif bits == 4:
        word = 256 * tau + 4 * lane + c // 32
        field = (c % 8) // 2 + 4 * (c % 2)
    else:
        raise ValueError(bits)
    return np.broadcast_to(word, (G, D)).copy(), np.broadcast_to(field, (G, D)).copy()


def _v_pos(bits: int):
    t = np.arange(G)[:, None]
    c = np.arange(D)[None, :]
    lane = c % 16 + 16 * (t // 8)
    if bits == 2:
        word = 4 * lane + c // 32
        field = (t % 8) // 2 + 4 * ((c // 16) % 2) + 8 * (t % 2)
    elif bits == 4:
        word = 256 * (c // 64) + 4 * lane + (c // 16) % 4
        field = (t % 8) // 2 + 4 * (t % 2)
    else:
        raise ValueError(bits)
    return np.broadcast_to(word, (G, D)).copy(), np.broadcast_to(field, (G, D)).copy()


def words_per_group(bits: int) -> int:
    return G * D * bits // 32


def _pack(codes: np.ndarray, bits: int, pos) -> np.ndarray:
    """codes uint8 [..., Nq, D] -> uint32 [..., Nq/32, words_per_group]."""
    word, field = pos
    lead = codes.shape[:-2]
    nq = codes.shape[-2]
    assert nq % G == 0 and codes.shape[-1] == D
    blocks = codes.reshape(*lead, nq // G, G * D).astype(np.uint32)
    out = np.zeros((*lead, nq // G, words_per_group(bits)), dtype=np.uint32)
    w, f = word.ravel(), field.ravel()
    for fld in range(32 // bits):
        sel = np.nonzero(f == fld)[0]
        # every word receives exactly one element per field
        assert np.array_equal(np.sort(w[sel]), np.arange(words_per_group(bits)))
        out[..., w[sel]] |= blocks[..., sel] << np.uint32(bits * fld)
    return out


def _unpack(words: np.ndarray, bits: int, pos) -> np.ndarray:
    """uint32 [..., J, words_per_group] -> uint8 [..., J*32, D]."""
    word, field = pos
    lead = words.shape[:-2]
    j = words.shape[-2]
    w, f = word.ravel(), field.ravel()
    vals = (words[..., w] >> (f.astype(np.uint32) * np.uint32(bits))) & np.uint32((1 << bits) - 1)
    return vals.astype(np.uint8).reshape(*lead, j * G, D)


def pack_k(codes, bits):
    return _pack(codes, bits, _k_pos(bits))


def unpack_k(words, bits):
    return _unpack(words, bits, _k_pos(bits))


def pack_v(codes, bits):
    return _pack(codes, bits, _v_pos(bits))


def unpack_v(words, bits):
    return _unpack(words, bits, _v_pos(bits))


def v_meta_to_physical(meta: np.ndarray) -> np.ndarray:
    """Logical fp16 [..., Nq, D/32] -> physical [..., Nq/32, D/32, 32]."""
    lead = meta.shape[:-2]
    nq, u = meta.shape[-2:]
    x = meta.reshape(*lead, nq // G, G, u)
    return np.ascontiguousarray(np.swapaxes(x, -1, -2))


def v_meta_to_logical(meta: np.ndarray) -> np.ndarray:
    """Physical [..., J, D/32, 32] -> logical [..., J*32, D/32]."""
    lead = meta.shape[:-3]
    j, u, g = meta.shape[-3:]
    return np.ascontiguousarray(np.swapaxes(meta, -1, -2)).reshape(*lead, j * g, u)
