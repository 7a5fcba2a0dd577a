"""Physical layout of the packed quantized cache, written from the layout
description in include/tkv.h (an interface, not arithmetic of the method) so
that tests can turn the library's packed words back into logical codes and
compare them bit for bit with oracle/quant.py.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Codes are stored per KV head in blocks of 32 tokens x D = 128 channels, whatever
the quantization group g (32 or 64).  ``t`` below is the token index inside its
block, ``c`` the channel.  A code occupies ``bits`` consecutive bits, least
significant first, at field F of a little-endian 32-bit word.

K codes, 1 bit:  word = 64*tau + lane, field F = (c%8)//2 + 4*((c//32)%2) + 8*(c//64) + 16*(c%2)
    (r, tau, lane as for 2 bit)
V codes, 1 bit:  word = 64*(c//64) + lane, field F = (t%8)//2 + 4*((c//16)%2) + 8*((c//32)%2) + 16*(t%2)
    (lane as for 2 bit)

K codes, 2 bit:  word = 4*lane + 2*tau + wd, field F = f + 8*e
    r = 4*(t//8) + t%4, tau = (t%8)//4, lane = r + 16*((c%32)//8)
    wd = c//64, f = (c%8)//2 + 4*((c//32)%2), e = c%2
K codes, 4 bit:  word = 256*tau + 4*lane + c//32, field F = (c%8)//2 + 4*(c%2)
V codes, 2 bit:  word = 4*lane + wd, field F = f + 8*e
    lane = c%16 + 16*(t//8), wd = c//32, f = (t%8)//2 + 4*((c//16)%2), e = t%2
V codes, 4 bit:  word = 256*(c//64) + 4*lane + (c//16)%4, field F = (t%8)//2 + 4*(t%2)
K scale / zero:  fp16 [token group of g][c]
V scale / zero:  fp16 [block of 32 tokens][u][t]   (u = channel group c // g)
"""
from __future__ import annotations

import numpy as np

BLK = 32   # tokens per code block
D = 128


def _k_pos(bits: int):
    t = np.arange(BLK)[:, None]
    c = np.arange(D)[None, :]
    r = 4 * (t // 8) + t % 4
    tau = (t % 8) // 4
    lane = r + 16 * ((c % 32) // 8)
    if bits == 1:
        word = 64 * tau + lane
        field = (c % 8) // 2 + 4 * ((c // 32) % 2) + 8 * (c // 64) + 16 * (c % 2)
    elif bits == 2:
        word = 4 * lane + 2 * tau + c // 64
        field = (c % 8) // 2 + 4 * ((c // 32) % 2) + 8 * (c % 2)
    elif bits == 4:
        word = 256 * tau + 4 * lane + c // 32
        field = (c % 8) // 2 + 4 * (c % 2)
    else:
        raise ValueError(bits)
    return np.broadcast_to(word, (BLK, D)).copy(), np.broadcast_to(field, (BLK, D)).copy()


def _v_pos(bits: int):
    t = np.arange(BLK)[:, None]
    c = np.arange(D)[None, :]
    lane = c % 16 + 16 * (t // 8)
    if bits == 1:
        word = 64 * (c // 64) + lane
        field = (t % 8) // 2 + 4 * ((c // 16) % 2) + 8 * ((c // 32) % 2) + 16 * (t % 2)
    elif bits == 2:
        word = 4 * lane + c // 32
        field = (t % 8) // 2 + 4 * ((c // 16) % 2) + 8 * (t % 2)
    elif bits == 4:
        word = 256 * (c // 64) + 4 * lane + (c // 16) % 4
        field = (t % 8) // 2 + 4 * (t % 2)
    else:
        raise ValueError(bits)
    return np.broadcast_to(word, (BLK, D)).copy(), np.broadcast_to(field, (BLK, D)).copy()


def words_per_block(bits: int) -> int:
    return BLK * D * bits // 32


def _pack(codes: np.ndarray, bits: int, pos) -> np.ndarray:
    """codes uint8 [..., Nq, D] -> uint32 [..., Nq/32, words_per_block]."""
    word, field = pos
    lead = codes.shape[:-2]
    nq = codes.shape[-2]
    assert nq % BLK == 0 and codes.shape[-1] == D
    blocks = codes.reshape(*lead, nq // BLK, BLK * D).astype(np.uint32)
    out = np.zeros((*lead, nq // BLK, words_per_block(bits)), dtype=np.uint32)
    w, f = word.ravel(), field.ravel()
    for fld in range(32 // bits):
        sel = np.nonzero(f == fld)[0]
        # every word receives exactly one element per field
        assert np.array_equal(np.sort(w[sel]), np.arange(words_per_block(bits)))
        out[..., w[sel]] |= blocks[..., sel] << np.uint32(bits * fld)
    return out


def _unpack(words: np.ndarray, bits: int, pos) -> np.ndarray:
    """uint32 [..., J, words_per_block] -> uint8 [..., J*32, D]."""
    word, field = pos
    lead = words.shape[:-2]
    j = words.shape[-2]
    w, f = word.ravel(), field.ravel()
    vals = (words[..., w] >> (f.astype(np.uint32) * np.uint32(bits))) & np.uint32((1 << bits) - 1)
    return vals.astype(np.uint8).reshape(*lead, j * BLK, D)


def pack_k(codes, bits):
    return _pack(codes, bits, _k_pos(bits))


def unpack_k(words, bits):
    return _unpack(words, bits, _k_pos(bits))


def pack_v(codes, bits):
    return _pack(codes, bits, _v_pos(bits))


def unpack_v(words, bits):
    return _unpack(words, bits, _v_pos(bits))


def v_meta_to_physical(meta: np.ndarray) -> np.ndarray:
    """Logical fp16 [..., Nq, D/g] -> physical [..., Nq/32, D/g, 32]."""
    lead = meta.shape[:-2]
    nq, u = meta.shape[-2:]
    x = meta.reshape(*lead, nq // BLK, BLK, u)
    return np.ascontiguousarray(np.swapaxes(x, -1, -2))


def v_meta_to_logical(meta: np.ndarray) -> np.ndarray:
    """Physical [..., J, D/g, 32] -> logical [..., J*32, D/g]."""
    lead = meta.shape[:-3]
    j, u, g = meta.shape[-3:]
    return np.ascontiguousarray(np.swapaxes(meta, -1, -2)).reshape(*lead, j * g, u)
