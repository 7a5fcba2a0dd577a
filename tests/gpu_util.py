"""Helpers for the GPU parity tests: move synthetic inputs to the device, read the
library's buffers back, compare with the oracle."""
import numpy as np
import torch

import paper_2505_19586_amd as tkv
from oracle import attention, layout, quant


def to_new(x: np.ndarray) -> torch.Tensor:
    """[Hkv, n, D] numpy fp16 -> device [1, n, Hkv, D]."""
    return torch.from_numpy(np.ascontiguousarray(x.transpose(1, 0, 2))[None]).cuda()


def to_new_batch(xs, n_max) -> torch.Tensor:
    """list of [Hkv, n_b, D] -> device [B, n_max, Hkv, D] zero padded."""
    hkv, _, d = xs[0].shape
    out = np.zeros((len(xs), n_max, hkv, d), np.float16)
    for b, x in enumerate(xs):
        out[b, : x.shape[1]] = x.transpose(1, 0, 2)
    return torch.from_numpy(out).cuda()


def check_quant_cache(layer: "tkv.QuantLayer", b: int, k: np.ndarray, v: np.ndarray):
    """Bit-exact comparison of sequence b of the library's cache with the oracle's."""
    d = layer.desc
    n = k.shape[1]
    assert int(layer.seq_len[b]) == n
    g = d.group_size
    ref = quant.quantize_kv(k, v, bits=d.bits, group=g, residual=d.residual)
    jq = ref.n_quant // 32   # code blocks
    torch.cuda.synchronize()
    kc = layer.view("k_codes")[b, :, :jq].cpu().numpy().view(np.uint32)
    vc = layer.view("v_codes")[b, :, :jq].cpu().numpy().view(np.uint32)
    assert np.array_equal(layout.unpack_k(kc, d.bits), ref.k_codes), "k codes"
    assert np.array_equal(layout.unpack_v(vc, d.bits), ref.v_codes), "v codes"
    assert np.array_equal(kc, layout.pack_k(ref.k_codes, d.bits)), "k words"
    assert np.array_equal(vc, layout.pack_v(ref.v_codes, d.bits)), "v words"
    for name, want in (("k_scale", ref.k_scale), ("k_zero", ref.k_zero)):
        got = layer.view(name)[b, :, :ref.n_quant // g].cpu().numpy()
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), name
    for name, want in (("v_scale", ref.v_scale), ("v_zero", ref.v_zero)):
        got = layout.v_meta_to_logical(layer.view(name)[b, :, :jq].cpu().numpy())
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), name
    ring = d.residual + g
    slots = np.arange(ref.n_quant, n) % ring
    for name, want in (("k_resid", ref.k_resid), ("v_resid", ref.v_resid)):
        got = layer.view(name)[b].cpu().numpy()[:, slots]
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), name
    return ref


def attn_err(out: torch.Tensor, ref: np.ndarray) -> float:
    return attention.max_rel_err(out.float().cpu().numpy().astype(np.float64), ref)


def attn_err_elementwise(out: torch.Tensor, ref: np.ndarray) -> float:
    """Reported beside attn_err, never asserted: element-wise relative error with a floor of
    2e-3 * rms(ref) under every denominator."""
    return attention.elementwise_rel_err(out.float().cpu().numpy().astype(np.float64), ref)
