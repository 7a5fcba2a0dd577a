"""Pins of the oracle's quantizer (Sec. 2.2 Eq. 4, Sec. 4.3 policy, Sec. 4.4 Table 2)
against things other than itself: hand-worked groups, closed forms, invariants."""
import os

import numpy as np
import pytest

from oracle import layout, quant
from synth import make_layer


def _parse_floats(s):
    return np.array([float(x) for x in s.split()], dtype=np.float64)


def test_eq4_hand_worked_groups(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "eq4_worked.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        bits, vals, s, z, codes, deq = [f.strip() for f in line.split("|")]
        x = _parse_floats(vals).astype(np.float16)
        c, s16, z16 = quant.quantize_lastaxis(x[None, :], int(bits))
        assert float(s16[0]) == float(s), line
        assert float(z16[0]) == float(z), line
        assert c[0].tolist() == [int(v) for v in codes.split()], line
        xhat = c[0].astype(np.float64) * float(s16[0]) + float(z16[0])
        assert np.array_equal(xhat, _parse_floats(deq)), line
        n += 1
    assert n >= 7


def test_table2_closed_form(golden_dir):
    for line in open(os.path.join(golden_dir, "table2_memory.txt")):
        if line.startswith("#") or not line.strip():
            continue
        kind, bits, g, n, h, d, lq, expect = line.split()
        if kind == "Q":
            got = quant.table2_quant_elements(int(n), int(h), int(d), int(lq), int(bits), int(g))
        else:
            got = quant.table2_sparse_elements(int(n), int(h), int(d))
        assert got == float(expect), line


@pytest.mark.parametrize("bits,g", [(2, 32), (4, 32), (1, 64), (2, 64)])
def test_table2_matches_actual_buffer_bytes(bits, g):
    """Bytes of the arrays the quantizer really produces equal the Table 2 count
    (the table's own setting is 1 bit with groups of 64)."""
    inp = make_layer(64 * 5, seq=3)
    c = quant.quantize_kv(inp.k, inp.v, bits=bits, group=g, residual=0)
    hkv, nq, d = c.k_codes.shape
    assert c.k_scale.shape == (hkv, nq // g, d) and c.v_scale.shape == (hkv, nq, d // g)
    code_bytes = 2 * hkv * nq * d * bits // 8
    meta_bytes = 2 * (c.k_scale.nbytes + c.v_scale.nbytes)
    elems = quant.table2_quant_elements(nq, hkv, d, 1, bits, g)
    assert code_bytes + meta_bytes == int(elems * 2)
    assert (code_bytes + meta_bytes) // (hkv * nq) == {(2, 32): 96, (4, 32): 160, (1, 64): 48, (2, 64): 80}[bits, g]
    # packed words have exactly the code bytes
    assert layout.pack_k(c.k_codes, bits).nbytes + layout.pack_v(c.v_codes, bits).nbytes == code_bytes


def test_partition():
    assert quant.partition(4096, 128, 32) == (3968, 128)
    assert quant.partition(32768, 128, 32) == (32640, 128)
    assert quant.partition(131072, 128, 32) == (130944, 128)
    assert quant.partition(100, 128, 32) == (0, 100)
    assert quant.partition(128, 128, 32) == (0, 128)
    assert quant.partition(159, 128, 32) == (0, 159)
    assert quant.partition(160, 128, 32) == (32, 128)
    for n in range(0, 700):
        nq, r = quant.partition(n, 128, 32)
        assert nq % 32 == 0 and nq + r == n
        assert (n < 128 and nq == 0) or 128 <= r <= 159


def test_sixteen_bit_is_identity():
    inp = make_layer(300, seq=1)
    c = quant.quantize_kv(inp.k, inp.v, bits=16, group=32, residual=128)
    k = np.concatenate([quant.dequantize_k(c), c.k_resid.astype(np.float64)], axis=1)
    v = np.concatenate([quant.dequantize_v(c), c.v_resid.astype(np.float64)], axis=1)
    assert np.array_equal(k.astype(np.float16).view(np.uint16), inp.k.view(np.uint16))
    assert np.array_equal(v.astype(np.float16).view(np.uint16), inp.v.view(np.uint16))


@pytest.mark.parametrize("bits,g", [(1, 32), (2, 32), (4, 32), (8, 32), (1, 64), (2, 64)])
def test_error_bound_and_endpoints(bits, g):
    inp = make_layer(32 * 40, seq=2)
    c = quant.quantize_kv(inp.k, inp.v, bits=bits, group=g, residual=0)
    qmax = (1 << bits) - 1
    for x, xhat, s, axis in (
        (inp.k, quant.dequantize_k(c), np.repeat(c.k_scale, g, axis=1), 1),
        (inp.v, quant.dequantize_v(c), np.repeat(c.v_scale, g, axis=2), 2),
    ):
        x = x.astype(np.float64)
        s = s.astype(np.float64)
        normal = s >= 2.0 ** -14
        assert normal.all()  # N(0,1) data never produces subnormal scalers
        err = np.abs(x - xhat)
        assert (err <= s / 2 * (1 + 2.0 ** -10)).all()
        # at least one group is close to the bound (a dropped rounding would halve/double it)
        assert (err / s).max() > 0.45
    # code(min) == 0 and code(max) == qmax in every group
    kg_codes = c.k_codes.reshape(8, -1, g, 128)
    kg = inp.k.reshape(8, -1, g, 128)
    amin = kg.argmin(axis=2)
    amax = kg.argmax(axis=2)
    assert (np.take_along_axis(kg_codes, amin[:, :, None, :], axis=2) == 0).all()
    assert (np.take_along_axis(kg_codes, amax[:, :, None, :], axis=2) == qmax).all()
    vg_codes = c.v_codes.reshape(8, -1, 128 // g, g)
    vg = inp.v.reshape(8, -1, 128 // g, g)
    assert (np.take_along_axis(vg_codes, vg.argmin(axis=3)[..., None], axis=3) == 0).all()
    assert (np.take_along_axis(vg_codes, vg.argmax(axis=3)[..., None], axis=3) == qmax).all()
    # dequantized values stay inside [min, max + s/2]
    kh = quant.dequantize_k(c).reshape(8, -1, g, 128)
    assert (kh >= kg.min(axis=2, keepdims=True)).all()
    assert (kh <= kg.max(axis=2, keepdims=True).astype(np.float64)
            + c.k_scale.astype(np.float64)[:, :, None, :] / 2 + 1e-12).all()


@pytest.mark.parametrize("bits", [2, 4])
def test_lattice_inputs_reproduce_exactly(bits):
    qmax = (1 << bits) - 1
    rng = np.random.default_rng(7)
    for s in (2.0 ** -3, 1.0, 4.0):
        for z in (-3.0, 0.0, 0.625):
            codes = rng.integers(0, qmax + 1, size=(5, 32))
            codes[:, 0], codes[:, 1] = 0, qmax          # range spans the full lattice
            x = (z + codes * s).astype(np.float16)
            c, s16, z16 = quant.quantize_lastaxis(x, bits)
            assert np.array_equal(c, codes)
            assert (s16 == np.float16(s)).all() and (z16 == np.float16(z)).all()
            assert np.array_equal(c * float(s) + z, x.astype(np.float64))
    # two-valued group -> codes in {0, qmax}, exact
    x = np.where(rng.random((4, 32)) < 0.5, -1.5, 2.25).astype(np.float16)
    x[:, 0], x[:, 1] = -1.5, 2.25
    c, s16, z16 = quant.quantize_lastaxis(x, bits)
    assert set(np.unique(c)) == {0, qmax}
    xhat = c.astype(np.float64) * s16.astype(np.float64)[:, None] + z16.astype(np.float64)[:, None]
    # s = 3.75/qmax is exact in fp16 for qmax = 3 (1.25) and 15 (0.25)
    assert np.array_equal(xhat, x.astype(np.float64))


def test_flat_and_tiny_range_groups():
    x = np.full((3, 32), -0.37, dtype=np.float16)
    c, s, z = quant.quantize_lastaxis(x, 2)
    assert (c == 0).all() and (s == 0).all() and (z == x[:, 0]).all()
    # range so small that the scaler is a subnormal fp16 or rounds to zero:
    # behaviour is defined (no NaN, codes in range, dequant finite), not bounded by s/2.
    tiny = np.float16(2.0 ** -24)
    x = np.zeros((1, 32), dtype=np.float16)
    x[0, 1] = tiny
    for bits in (2, 4):
        c, s, z = quant.quantize_lastaxis(x, bits)
        assert c.max() <= (1 << bits) - 1 and np.isfinite(s.astype(np.float64)).all()
        if s[0] == 0:
            assert (c == 0).all()


@pytest.mark.parametrize("bits,g", [(2, 32), (1, 64)])
def test_k_and_v_policies_are_the_same_scalar_quantizer(bits, g):
    """Per-channel K quantization of a g x g block equals per-token V
    quantization of its transpose (Sec. 4.3: same Eq. 4, different grouping)."""
    rng = np.random.default_rng(11)
    blk = rng.standard_normal((g, g)).astype(np.float16)
    k = np.zeros((1, g, 128), np.float16)
    v = np.zeros((1, g, 128), np.float16)
    k[0, :, :g] = blk          # tokens x channels
    v[0, :, :g] = blk.T        # tokens x channels, transposed block
    c = quant.quantize_kv(k, v, bits=bits, group=g, residual=0)
    assert np.array_equal(c.k_codes[0, :, :g], c.v_codes[0, :, :g].T)
    assert np.array_equal(c.k_scale[0, 0, :g], c.v_scale[0, :, 0])
    assert np.array_equal(c.k_zero[0, 0, :g], c.v_zero[0, :, 0])


def test_scale_is_float32_division_rounded_to_fp16():
    """s must be RN16(RN32(max-min)/RN32(qmax)); check against exact rationals."""
    from fractions import Fraction
    rng = np.random.default_rng(5)
    x = rng.standard_normal((200, 32)).astype(np.float16)
    for bits in (2, 4):
        _, s16, _ = quant.quantize_lastaxis(x, bits)
        qmax = (1 << bits) - 1
        for i in range(x.shape[0]):
            exact = (Fraction(float(x[i].max())) - Fraction(float(x[i].min()))) / qmax
            s32 = np.float32(float(exact))       # range is exact in f32, so one rounding
            assert np.float16(s32) == s16[i]
            assert abs(Fraction(float(s16[i])) - exact) <= exact * Fraction(1, 2 ** 11) * Fraction(1001, 1000)
