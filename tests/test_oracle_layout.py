"""The packed layout is a bijection and has the documented endianness."""
import numpy as np
import pytest

from oracle import layout


@pytest.mark.parametrize("bits", [1, 2, 4])
@pytest.mark.parametrize("which", ["k", "v"])
def test_pack_unpack_round_trip(bits, which):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 1 << bits, size=(2, 3, 96, 128)).astype(np.uint8)
    pack = layout.pack_k if which == "k" else layout.pack_v
    unpack = layout.unpack_k if which == "k" else layout.unpack_v
    words = pack(codes, bits)
    assert words.shape == (2, 3, 3, 128 * bits) and words.dtype == np.uint32
    assert np.array_equal(unpack(words, bits), codes)


@pytest.mark.parametrize("bits", [1, 2, 4])
def test_one_hot_positions(bits):
    """Spot positions computed by hand from the formulas in include/tkv.h."""
    qmax = (1 << bits) - 1
    def where(pack, t, c):
        codes = np.zeros((32, 128), np.uint8)
        codes[t, c] = qmax
        w = pack(codes, bits)[0]
        (idx,) = np.nonzero(w)
        assert len(idx) == 1
        val = int(w[idx[0]])
        shift = (val & -val).bit_length() - 1
        assert val == qmax << shift
        return int(idx[0]), shift // bits
    if bits == 1:
        assert where(layout.pack_k, 0, 0) == (0, 0)
        assert where(layout.pack_k, 0, 1) == (0, 16)          # odd channel -> upper half-word
        assert where(layout.pack_k, 0, 6) == (0, 3)
        assert where(layout.pack_k, 0, 8) == (16, 0)          # next 8-channel block -> lane 16
        assert where(layout.pack_k, 0, 32) == (0, 4)          # 32-channel blocks 1, 2, 3 -> bits 4.., 8.., 12..
        assert where(layout.pack_k, 0, 64) == (0, 8)
        assert where(layout.pack_k, 0, 96) == (0, 12)
        assert where(layout.pack_k, 4, 0) == (64, 0)          # tau = 1 -> second half of the block
        assert where(layout.pack_k, 8, 0) == (4, 0)           # r = 4
        assert where(layout.pack_k, 31, 127) == (64 + 63, 31)
        assert where(layout.pack_v, 0, 0) == (0, 0)
        assert where(layout.pack_v, 1, 0) == (0, 16)          # odd token -> upper half-word
        assert where(layout.pack_v, 6, 0) == (0, 3)
        assert where(layout.pack_v, 0, 16) == (0, 4)          # 16-channel blocks 1, 2, 3 -> bits 4.., 8.., 12..
        assert where(layout.pack_v, 0, 32) == (0, 8)
        assert where(layout.pack_v, 0, 48) == (0, 12)
        assert where(layout.pack_v, 0, 64) == (64, 0)
        assert where(layout.pack_v, 8, 5) == (5 + 16, 0)
        assert where(layout.pack_v, 31, 127) == (64 + 63, 31)
    elif bits == 2:
        assert where(layout.pack_k, 0, 0) == (0, 0)
        assert where(layout.pack_k, 0, 1) == (0, 8)          # e = 1 -> upper half-word
        assert where(layout.pack_k, 0, 2) == (0, 1)
        assert where(layout.pack_k, 0, 8) == (4 * 16, 0)      # next 8-channel block -> lane 16
        assert where(layout.pack_k, 0, 32) == (0, 4)          # second 32-channel block -> fields 4..7
        assert where(layout.pack_k, 0, 64) == (1, 0)          # wd = 1
        assert where(layout.pack_k, 4, 0) == (2, 0)           # tau = 1
        assert where(layout.pack_k, 8, 0) == (4 * 4, 0)       # r = 4
        assert where(layout.pack_k, 31, 127) == (4 * (15 + 48) + 3, 15)
        assert where(layout.pack_v, 0, 0) == (0, 0)
        assert where(layout.pack_v, 1, 0) == (0, 8)
        assert where(layout.pack_v, 2, 0) == (0, 1)
        assert where(layout.pack_v, 0, 16) == (0, 4)
        assert where(layout.pack_v, 0, 32) == (1, 0)
        assert where(layout.pack_v, 8, 5) == (4 * (5 + 16), 0)
        assert where(layout.pack_v, 31, 127) == (4 * 63 + 3, 15)
    else:
        assert where(layout.pack_k, 0, 0) == (0, 0)
        assert where(layout.pack_k, 0, 1) == (0, 4)
        assert where(layout.pack_k, 0, 6) == (0, 3)
        assert where(layout.pack_k, 0, 32) == (1, 0)
        assert where(layout.pack_k, 4, 0) == (256, 0)
        assert where(layout.pack_k, 31, 127) == (256 + 4 * 63 + 3, 7)
        assert where(layout.pack_v, 0, 0) == (0, 0)
        assert where(layout.pack_v, 1, 0) == (0, 4)
        assert where(layout.pack_v, 0, 16) == (1, 0)
        assert where(layout.pack_v, 0, 64) == (256, 0)
        assert where(layout.pack_v, 31, 127) == (256 + 4 * 63 + 3, 7)


def test_v_meta_layout():
    m = np.arange(2 * 64 * 4, dtype=np.float16).reshape(2, 64, 4)
    p = layout.v_meta_to_physical(m)
    assert p.shape == (2, 2, 4, 32)
    assert p[1, 1, 3, 5] == m[1, 32 + 5, 3]
    assert np.array_equal(layout.v_meta_to_logical(p), m)


def test_v_meta_layout_two_channel_groups():
    """g = 64: two channel groups per token, still blocks of 32 tokens."""
    m = np.arange(64 * 2, dtype=np.float16).reshape(64, 2)
    p = layout.v_meta_to_physical(m)
    assert p.shape == (2, 2, 32)
    assert p[1, 1, 5] == m[32 + 5, 1]
    assert np.array_equal(layout.v_meta_to_logical(p), m)
