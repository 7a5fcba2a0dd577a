"""tkv_quant_attn_decode_static (fixed scratch array inside the library, nothing allocated)
against tkv_quant_attn_decode (caller's workspace), called through the C ABI: two calls in a
row on the same GPU, the second with a smaller input, then the limits."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from paper_2505_19586_amd.tkv import QuantCache, QuantDesc
from oracle import attention, quant
from synth import make_layer

from gpu_util import attn_err, to_new, to_new_batch

pytestmark = pytest.mark.gpu
SM = 1.0 / np.sqrt(128.0)


def _layer(n, seq, bits=2, batch=1, lens=None):
    if batch == 1:
        inp = make_layer(n, config=1, layer=5, seq=seq)
        layer = tkv.QuantLayer(bits=bits, capacity=(n + 63) // 32 * 32)
        layer.append(to_new(inp.k), to_new(inp.v))
        return layer, torch.from_numpy(inp.q)[None].cuda(), [inp]
    inps = [make_layer(m, config=4, layer=5, seq=seq + b) for b, m in enumerate(lens)]
    layer = tkv.QuantLayer(bits=bits, capacity=n, batch=batch)
    layer.append(to_new_batch([i.k for i in inps], n), to_new_batch([i.v for i in inps], n), n_valid=lens)
    return layer, torch.from_numpy(np.stack([i.q for i in inps])).cuda(), inps


def _both(layer, q):
    """Outputs of the workspace call and of the static call (raw ctypes calls, caller-owned outputs)."""
    L = tkv.lib()
    d, c = layer.desc, layer.cache
    want = torch.full_like(q, float("nan"))
    got = torch.full_like(q, float("nan"))
    torch.cuda.synchronize()
    s = torch.cuda.current_stream().cuda_stream
    assert L.tkv_quant_attn_decode(C.byref(d), C.byref(c), q.data_ptr(), want.data_ptr(), C.c_float(SM),
                                   layer.workspace.data_ptr(), layer.workspace_bytes, s) == 0
    before = torch.cuda.memory_allocated()
    assert L.tkv_quant_attn_decode_static(C.byref(d), C.byref(c), q.data_ptr(), got.data_ptr(), C.c_float(SM), s) == 0
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    print("case static: n=20000 then n=3000 (same scratch array, second call smaller)", flush=True)
    big, q_big, inp_big = _layer(20000, seq=1)
    small, q_small, inp_small = _layer(3000, seq=2)
    for layer, q, inps in ((big, q_big, inp_big), (small, q_small, inp_small), (big, q_big, inp_big)):
        want, got = _both(layer, q)
        # same kernels, same launch shape: the two calls agree bit for bit
        assert torch.equal(want.view(torch.int16), got.view(torch.int16))
        ref = quant.quantize_kv(inps[0].k, inps[0].v, bits=2, group=32, residual=128)
        assert attn_err(got[0], attention.quant_attention(inps[0].q, ref, SM)) <= 2e-3


def test_static_scratch_batched_and_four_bit():
    print("case static: batch 8 ragged, then 4 bit", flush=True)
    lens = [700, 2048, 33, 1999, 1024, 128, 0, 1500]
    layer, q, inps = _layer(2048, seq=10, batch=8, lens=lens)
    want, got = _both(layer, q)
    assert torch.equal(want.view(torch.int16), got.view(torch.int16))
    assert (got[6] == 0).all()
    l4, q4, inp4 = _layer(5000, seq=3, bits=4)
    want, got = _both(l4, q4)
    assert torch.equal(want.view(torch.int16), got.view(torch.int16))
    ref = quant.quantize_kv(inp4[0].k, inp4[0].v, bits=4, group=32, residual=128)
    assert attn_err(got[0], attention.quant_attention(inp4[0].q, ref, SM)) <= 2e-3


def test_static_scratch_limits_are_errors():
    """Beyond the fixed array: a clear error, nothing enqueued (argument checks need no data)."""
    L = tkv.lib()
    layer, q, _ = _layer(1024, seq=4)
    out = torch.zeros_like(q)
    # 64 sequences x 128 KV heads = 8192 (sequence, head) pairs > TKV_STATIC_MAX_HEADS
    d = QuantDesc(C.sizeof(QuantDesc), 128, 128, 128, 2, 32, 128, 1024, 64)
    lens = (C.c_int32 * 64)(*([0] * 64))
    c = QuantCache(*([layer.cache.k_codes] * 8), lens)
    assert L.tkv_quant_attn_decode_static(C.byref(d), C.byref(c), q.data_ptr(), out.data_ptr(), C.c_float(SM), None) == -4
    assert L.tkv_quant_attn_decode_static(C.byref(layer.desc), None, q.data_ptr(), out.data_ptr(), C.c_float(SM), None) == -1
    assert L.tkv_quant_attn_decode_static(None, None, None, None, C.c_float(SM), None) == -1
