"""Pins of the oracle's attention (Sec. 2.1 Eq. 3) and split-K merge."""
import numpy as np
import pytest
import torch

from oracle import attention, quant
from synth import HeadShape, make_layer

SMALL = HeadShape(8, 2, 128)


def _torch_reference(q, k, v, sm_scale):
    """Library routine for Eq. 3 (not the oracle's own code path)."""
    q = torch.from_numpy(np.asarray(q, np.float64))
    k = torch.from_numpy(np.asarray(k, np.float64))
    v = torch.from_numpy(np.asarray(v, np.float64))
    g = q.shape[0] // k.shape[0]
    k = k.repeat_interleave(g, dim=0)
    v = v.repeat_interleave(g, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(
        q[:, None, :], k, v, scale=float(sm_scale))
    return o[:, 0, :].numpy()


def test_dense_attention_matches_library_sdpa():
    inp = make_layer(777, shape=SMALL, seq=4)
    sm = 1 / np.sqrt(128)
    ref = _torch_reference(inp.q, inp.k, inp.v, sm)
    got = attention.decode_attention(inp.q, inp.k, inp.v, sm)
    assert np.abs(got - ref).max() < 1e-12


def test_gqa_head_mapping():
    """Query head i must read KV head i // G: make KV heads distinguishable."""
    rng = np.random.default_rng(0)
    q = rng.standard_normal((8, 128)).astype(np.float16)
    k = rng.standard_normal((2, 50, 128)).astype(np.float16)
    v = np.zeros((2, 50, 128), np.float16)
    v[0] += 1.0
    v[1] += 2.0
    o = attention.decode_attention(q, k, v, 0.1)
    assert np.allclose(o[:4], 1.0) and np.allclose(o[4:], 2.0)


def test_special_cases():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((4, 128)).astype(np.float16)
    v = rng.standard_normal((1, 33, 128)).astype(np.float16)
    # all-equal keys -> uniform weights -> mean of V
    k = np.tile(rng.standard_normal((1, 1, 128)).astype(np.float16), (1, 33, 1))
    o = attention.decode_attention(q, k, v, 0.3)
    assert np.allclose(o, v.astype(np.float64).mean(axis=1), atol=1e-12)
    # one key with a far larger logit -> that V row
    k = np.zeros((1, 33, 128), np.float16)
    k[0, 17] = (q[2].astype(np.float32) * 40).astype(np.float16)
    o = attention.decode_attention(q[2:3], k, v, 1.0)
    assert np.allclose(o[0], v[0, 17].astype(np.float64), atol=1e-9)
    # permutation invariance
    k = rng.standard_normal((1, 33, 128)).astype(np.float16)
    perm = rng.permutation(33)
    a = attention.decode_attention(q, k, v, 0.09)
    b = attention.decode_attention(q, k[:, perm], v[:, perm], 0.09)
    assert np.abs(a - b).max() < 1e-13
    # softmax weights sum to one: V of all ones -> output of all ones
    o = attention.decode_attention(q, k, np.ones_like(v), 0.09)
    assert np.allclose(o, 1.0, atol=1e-13)
    # sm_scale really multiplies the logits: scale 0 -> mean of V
    o = attention.decode_attention(q, k, v, 0.0)
    assert np.allclose(o, v.astype(np.float64).mean(axis=1), atol=1e-13)


@pytest.mark.parametrize("chunks", [[0, 1000], [0, 1, 2, 999, 1000], [0, 0, 256, 256, 700, 1000, 1000],
                                    list(range(0, 1001, 40))])
def test_split_k_merge_equals_single_pass(chunks):
    inp = make_layer(1000, shape=SMALL, seq=5)
    sm = 1 / np.sqrt(128)
    ref = attention.decode_attention(inp.q, inp.k, inp.v, sm)
    for i in range(8):
        h = i // 4
        parts = [attention.partial_attention(inp.q[i], inp.k[h, a:b], inp.v[h, a:b], sm)
                 for a, b in zip(chunks[:-1], chunks[1:])]
        got = attention.merge_partials(parts)
        assert np.abs(got - ref[i]).max() < 1e-12


@pytest.mark.parametrize("bits", [2, 4])
def test_quant_attention_is_dense_attention_on_dequantized_cache(bits):
    inp = make_layer(500, shape=SMALL, seq=6)
    c = quant.quantize_kv(inp.k, inp.v, bits=bits, group=32, residual=128)
    assert c.n_quant == 352 and c.k_resid.shape[1] == 148
    sm = 1 / np.sqrt(128)
    khat = np.concatenate([quant.dequantize_k(c), inp.k[:, 352:].astype(np.float64)], axis=1)
    vhat = np.concatenate([quant.dequantize_v(c), inp.v[:, 352:].astype(np.float64)], axis=1)
    ref = _torch_reference(inp.q, khat, vhat, sm)
    got = attention.quant_attention(inp.q, c, sm)
    assert np.abs(got - ref).max() < 1e-12
    # and the quantized result is near, but not equal to, the unquantized one
    dense = attention.decode_attention(inp.q, inp.k, inp.v, sm)
    err = attention.max_rel_err(got, dense)
    finer = quant.quantize_kv(inp.k, inp.v, bits=8, group=32, residual=128)
    err8 = attention.max_rel_err(attention.quant_attention(inp.q, finer, sm), dense)
    assert err > 1e-4 and err8 < 0.05 and err8 < err


def test_sixteen_bit_quant_attention_equals_dense():
    inp = make_layer(400, shape=SMALL, seq=7)
    c = quant.quantize_kv(inp.k, inp.v, bits=16, group=32, residual=128)
    sm = 1 / np.sqrt(128)
    a = attention.quant_attention(inp.q, c, sm)
    b = attention.decode_attention(inp.q, inp.k, inp.v, sm)
    assert np.array_equal(a, b)


def test_dequant_group_mapping_is_not_transposed():
    """K scalers are per channel within a token group, V scalers per token within
    a channel group: perturb one scaler and see exactly its group change."""
    inp = make_layer(32 * 4, shape=SMALL, seq=8)
    c = quant.quantize_kv(inp.k, inp.v, bits=2, group=32, residual=0)
    base_k, base_v = quant.dequantize_k(c), quant.dequantize_v(c)
    c.k_scale[1, 2, 77] *= np.float16(2)
    c.v_scale[0, 45, 3] *= np.float16(2)
    dk = quant.dequantize_k(c) != base_k
    dv = quant.dequantize_v(c) != base_v
    tk, ck = np.nonzero(dk[1])
    assert set(ck) == {77} and tk.min() >= 64 and tk.max() < 96
    tv, cv = np.nonzero(dv[0])
    assert set(tv) == {45} and cv.min() >= 96 and cv.max() < 128
    assert not dk[0].any() and not dv[1].any()


def test_error_metric_hand_worked():
    """Pins the metric behind every attention parity assertion: per query-head vector,
    max_c |out - ref| / max_c |ref|, then the maximum over heads.  All values are binary
    fractions, so the expected numbers are exact.

    head 0: ref (8, 1, -2, 0), errors (1/64, 0, 0, 1/16): the largest error sits on the
            channel whose reference is 0, the largest |ref| on another -> (1/16) / 8 = 2^-7
    head 1: ref (1/2, -1/4, 1/8, 1/4), errors (0, 1/64, 0, 0) -> (1/64) / (1/2) = 2^-5
    The worst head (1) is not the head with the largest reference or the largest absolute
    error (0).  Variants that must NOT come out: whole-tensor denominator 2^-7, minimum over
    heads 2^-7, mean over heads 5 * 2^-8, error and reference taken on the same channel (inf)."""
    ref = np.array([[8.0, 1.0, -2.0, 0.0], [0.5, -0.25, 0.125, 0.25]])
    out = ref + np.array([[1 / 64, 0.0, 0.0, 1 / 16], [0.0, -1 / 64, 0.0, 0.0]])
    assert attention.max_rel_err(out, ref) == 2.0 ** -5
    # each head on its own, and symmetric in the sign of the error
    assert attention.max_rel_err(out[0], ref[0]) == 2.0 ** -7
    assert attention.max_rel_err(out[1], ref[1]) == 2.0 ** -5
    assert attention.max_rel_err(2 * ref - out, ref) == 2.0 ** -5
    # heads swapped: the same value (maximum over heads, not the first or the last head)
    assert attention.max_rel_err(out[::-1], ref[::-1]) == 2.0 ** -5
    # a leading batch axis is just more heads
    assert attention.max_rel_err(out[None], ref[None]) == 2.0 ** -5
    # all-zero reference head: denominator 1, the error itself is reported
    z = np.zeros((1, 4))
    assert attention.max_rel_err(z + np.array([0.0, 2.0 ** -9, 0.0, 0.0]), z) == 2.0 ** -9
    assert attention.max_rel_err(ref, ref) == 0.0
    # scaling both by a constant leaves the metric unchanged (it is relative)
    assert attention.max_rel_err(4 * out, 4 * ref) == 2.0 ** -5


def test_elementwise_error_hand_worked():
    """The reported-only companion: max_c |out - ref| / max(|ref_c|, floor * rms(ref)) per head.
    Same example.  head 0: rms = sqrt((64 + 1 + 4 + 0) / 4) = sqrt(17.25); channel 3 has
    ref 0, so its denominator is the floor 2e-3 * sqrt(17.25) -> (1/16) / that; channel 0
    gives (1/64) / 8.  head 1: floor = 2e-3 * sqrt(0.390625 / 4) is below every |ref_c| ->
    (1/64) / (1/4) = 1/16."""
    ref = np.array([[8.0, 1.0, -2.0, 0.0], [0.5, -0.25, 0.125, 0.25]])
    out = ref + np.array([[1 / 64, 0.0, 0.0, 1 / 16], [0.0, -1 / 64, 0.0, 0.0]])
    h0 = (1 / 16) / (2e-3 * np.sqrt(17.25))
    assert attention.elementwise_rel_err(out[0], ref[0]) == pytest.approx(h0, rel=1e-12)
    assert attention.elementwise_rel_err(out[1], ref[1]) == 1 / 16
    assert attention.elementwise_rel_err(out, ref) == pytest.approx(h0, rel=1e-12)
    # a larger floor takes over the denominators of small channels
    assert attention.elementwise_rel_err(out[1], ref[1], floor=1.0) == pytest.approx(
        (1 / 64) / np.sqrt(0.390625 / 4), rel=1e-12)
    # all-zero reference: denominator 1
    z = np.zeros((2, 4))
    assert attention.elementwise_rel_err(z + 0.25, z) == 0.25
    assert attention.elementwise_rel_err(ref, ref) == 0.0
