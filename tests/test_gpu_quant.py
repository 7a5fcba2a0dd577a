"""GPU parity of tkv_quantize_append and tkv_quant_attn_decode against the oracle
(through the C ABI).  Codes, scalers, zero-points: bit-exact.  Attention: max
relative error <= 2e-3 per query head (fp16 I/O, fp32 accumulate)."""
import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from oracle import attention, quant
from synth import HeadShape, make_layer

from gpu_util import attn_err, check_quant_cache, to_new, to_new_batch

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(autouse=True, params=["mfma", "reference"])
def kernel_choice(request):
    """Every case runs with the matrix-core kernel and with the reference kernel."""
    tkv.debug_quant_attn_config(0 if request.param == "mfma" else 1)
    yield request.param
    tkv.debug_quant_attn_config(0)

SM = 1.0 / np.sqrt(128.0)
# (bits, quantization group): the benchmark's settings, the paper's (Sec. 5.1: 1 and 2 bits,
# groups of 64), and two that only the reference kernel is built for
SETTINGS = [(2, 32), (4, 32), (1, 64), (2, 64), (1, 32), (4, 64)]
MAIN_SETTINGS = SETTINGS[:4]


@pytest.mark.parametrize("bits,g", SETTINGS)
@pytest.mark.parametrize("n", [4096, 1, 127, 128, 159, 160, 161, 191, 192, 193, 1000])
def test_bulk_append_and_attention(bits, g, n):
    print(f"case bulk bits={bits} g={g} n={n}", flush=True)
    inp = make_layer(n, config=0, layer=0, seq=n % 97)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=4096 + 64)
    layer.append(to_new(inp.k), to_new(inp.v))
    ref = check_quant_cache(layer, 0, inp.k, inp.v)
    out = layer.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    want = attention.quant_attention(inp.q, ref, SM)
    err = attn_err(out[0], want)
    print(f"   err {err:.3e}", flush=True)
    assert err <= TOL


@pytest.mark.parametrize("bits,g", MAIN_SETTINGS)
def test_incremental_append_equals_bulk(bits, g):
    """Decode loop: 8 single-token steps that cross no group boundary, then 40 that
    cross one, then uneven multi-token appends; after each phase the cache must be
    the oracle's cache of the whole prefix."""
    print(f"case incremental bits={bits} g={g}", flush=True)
    n0, total = 4096, 4096 + 8 + 40 + 7 + 90 + 300
    inp = make_layer(total, config=0, layer=0, seq=5)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=8192)
    kd, vd = to_new(inp.k), to_new(inp.v)
    layer.append(kd[:, :n0].contiguous(), vd[:, :n0].contiguous())
    pos = n0
    q = torch.from_numpy(inp.q)[None].cuda()
    for step_sizes in ([1] * 8, [1] * 40, [7], [90], [300]):
        for s in step_sizes:
            layer.append(kd[:, pos:pos + s].contiguous(), vd[:, pos:pos + s].contiguous())
            pos += s
        ref = check_quant_cache(layer, 0, inp.k[:, :pos], inp.v[:, :pos])
        out = layer.attn_decode(q, SM)
        assert attn_err(out[0], attention.quant_attention(inp.q, ref, SM)) <= TOL
    assert pos == total


@pytest.mark.parametrize("bits,g", MAIN_SETTINGS + [(1, 32)])
def test_decode_step_in_one_call(bits, g):
    """tkv_quant_decode over 70 single-token steps (which cross group boundaries: those steps take
    the separate append) and a few multi-token ones: after every step the attention output is
    within the bound of the oracle's over the grown prefix; the cache is the oracle's cache bit
    for bit at checkpoints.  (1, 32) is served by the reference kernel only: always two calls.)"""
    print(f"case decode step bits={bits} g={g}", flush=True)
    n0 = 3000
    steps = [1] * 70 + [3, 1, 1, 40, 1, 1]
    total = n0 + sum(steps)
    inp = make_layer(total, config=0, layer=0, seq=11)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=4096)
    kd, vd = to_new(inp.k), to_new(inp.v)
    layer.append(kd[:, :n0].contiguous(), vd[:, :n0].contiguous())
    q = torch.from_numpy(inp.q)[None].cuda()
    pos = n0
    for i, s in enumerate(steps):
        out = layer.decode(q, SM, kd[:, pos:pos + s].contiguous(), vd[:, pos:pos + s].contiguous())
        pos += s
        assert int(layer.seq_len[0]) == pos
        if i % 9 == 0 or i >= 68:
            ref = check_quant_cache(layer, 0, inp.k[:, :pos], inp.v[:, :pos])
            err = attn_err(out[0], attention.quant_attention(inp.q, ref, SM))
            print(f"   step {i} n={pos} err {err:.3e}", flush=True)
            assert err <= TOL
    assert pos == total


@pytest.mark.parametrize("bits,g", [(2, 32), (1, 64)])
def test_decode_steps_from_an_empty_cache(bits, g):
    """tkv_quant_decode from the first token on: no quantized group yet, then the first ones."""
    total = 300
    inp = make_layer(total, seq=9)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=512)
    kd, vd = to_new(inp.k), to_new(inp.v)
    q = torch.from_numpy(inp.q)[None].cuda()
    for pos in range(total):
        out = layer.decode(q, SM, kd[:, pos:pos + 1].contiguous(), vd[:, pos:pos + 1].contiguous())
        if pos in (0, 1, 31, 127, 128, 159, 160, 191, 192, 255, 299):
            ref = check_quant_cache(layer, 0, inp.k[:, :pos + 1], inp.v[:, :pos + 1])
            assert attn_err(out[0], attention.quant_attention(inp.q, ref, SM)) <= TOL, pos


def test_decode_step_ragged_batch_and_groups_of_eight():
    """tkv_quant_decode on a padded batch (one sequence gets no token, one completes a group in
    some steps) with 8 query heads per KV head (two workgroups per KV head read the new rows,
    one writes them)."""
    shape = HeadShape(16, 2, 128)
    lens = [700, 129, 2040, 333]
    adds = [[1, 0, 1, 1]] * 12 + [[2, 1, 0, 3]] * 3
    grow = [sum(a[b] for a in adds) for b in range(4)]
    inps = [make_layer(n + grow[b], shape=shape, seq=40 + b) for b, n in enumerate(lens)]
    layer = tkv.QuantLayer(n_q_heads=16, n_kv_heads=2, bits=2, capacity=2560, batch=4)
    layer.append(to_new_batch([i.k[:, :n] for i, n in zip(inps, lens)], 2048),
                 to_new_batch([i.v[:, :n] for i, n in zip(inps, lens)], 2048), n_valid=lens)
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    pos = list(lens)
    for a in adds:
        w = max(a)
        kn = to_new_batch([i.k[:, p:p + x] for i, p, x in zip(inps, pos, a)], w)
        vn = to_new_batch([i.v[:, p:p + x] for i, p, x in zip(inps, pos, a)], w)
        out = layer.decode(q, SM, kn, vn, n_valid=a)
        pos = [p + x for p, x in zip(pos, a)]
    for b, inp in enumerate(inps):
        ref = check_quant_cache(layer, b, inp.k[:, :pos[b]], inp.v[:, :pos[b]])
        assert attn_err(out[b], attention.quant_attention(inp.q, ref, SM)) <= TOL


@pytest.mark.parametrize("bits,g", [(2, 32), (1, 64)])
def test_append_from_empty_in_small_steps(bits, g):
    inp = make_layer(400, seq=6)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=512)
    kd, vd = to_new(inp.k), to_new(inp.v)
    pos = 0
    for s in [1, 1, 30, 96, 31, 1, 1, 200, 39]:
        layer.append(kd[:, pos:pos + s].contiguous(), vd[:, pos:pos + s].contiguous())
        pos += s
        check_quant_cache(layer, 0, inp.k[:, :pos], inp.v[:, :pos])


@pytest.mark.parametrize("bits,g", MAIN_SETTINGS)
def test_ragged_batch(bits, g):
    print(f"case ragged bits={bits} g={g}", flush=True)
    lens = [700, 1, 2048, 333, 160]
    inps = [make_layer(n, config=4, layer=0, seq=b) for b, n in enumerate(lens)]
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=2048, batch=len(lens))
    layer.append(to_new_batch([i.k for i in inps], 2048), to_new_batch([i.v for i in inps], 2048), n_valid=lens)
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    out = layer.attn_decode(q, SM)
    for b, inp in enumerate(inps):
        ref = check_quant_cache(layer, b, inp.k, inp.v)
        assert attn_err(out[b], attention.quant_attention(inp.q, ref, SM)) <= TOL


def test_empty_sequence_gives_zeros():
    layer = tkv.QuantLayer(bits=2, capacity=256)
    q = torch.randn(1, 32, 128, dtype=torch.float16, device="cuda")
    out = layer.attn_decode(q, SM)
    torch.cuda.synchronize()
    assert (out == 0).all()


@pytest.mark.parametrize("bits,g", [(2, 32), (4, 32), (1, 64)])
@pytest.mark.parametrize("shape", [HeadShape(64, 8, 128), HeadShape(56, 8, 128), HeadShape(10, 2, 128),
                                   HeadShape(6, 1, 128), HeadShape(3, 1, 128)])
def test_groups_of_up_to_eight_query_heads(shape, bits, g):
    """Groups of 5 to 8 query heads per KV head are served 4 heads at a time (two workgroups per
    KV head and chunk); groups of 3 leave a column of the kernel's four unused."""
    print(f"case quant attention Hq={shape.n_q_heads} Hkv={shape.n_kv_heads} bits={bits} g={g}", flush=True)
    n = 2500
    inp = make_layer(n, shape=shape, seq=3)
    layer = tkv.QuantLayer(n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, bits=bits, group_size=g,
                           capacity=2560)
    layer.append(to_new(inp.k), to_new(inp.v))
    ref = check_quant_cache(layer, 0, inp.k, inp.v)
    want = attention.quant_attention(inp.q, ref, SM)
    q = torch.from_numpy(inp.q)[None].cuda()
    out = layer.attn_decode(q, SM)
    assert attn_err(out[0], want) <= TOL
    out2 = layer.attn_decode(q, SM)              # the arrival counters were left clean
    assert attn_err(out2[0], want) <= TOL
    assert attn_err(layer.attn_decode_static(q, SM, torch.empty_like(q))[0], want) <= TOL


def test_group_of_eight_ragged_batch_long_context():
    shape = HeadShape(16, 2, 128)
    lens = [40000, 9000, 131]
    layer = tkv.QuantLayer(n_q_heads=16, n_kv_heads=2, bits=2, capacity=40000 + 32, batch=3)
    inps = [make_layer(n, shape=shape, seq=20 + i) for i, n in enumerate(lens)]
    k, v = to_new_batch([i.k for i in inps], max(lens)), to_new_batch([i.v for i in inps], max(lens))
    layer.append(k, v, n_valid=lens)
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    out = layer.attn_decode(q, SM)
    for b, inp in enumerate(inps):
        ref = check_quant_cache(layer, b, inp.k, inp.v)
        err = attn_err(out[b], attention.quant_attention(inp.q, ref, SM))
        print(f"   n={lens[b]} err {err:.3e}", flush=True)
        assert err <= TOL


@pytest.mark.parametrize("shape", [HeadShape(8, 8, 128), HeadShape(16, 8, 128), HeadShape(4, 1, 128)])
def test_other_head_groupings(shape):
    inp = make_layer(777, shape=shape, seq=8)
    layer = tkv.QuantLayer(n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, bits=2, capacity=1024)
    layer.append(to_new(inp.k), to_new(inp.v))
    ref = check_quant_cache(layer, 0, inp.k, inp.v)
    out = layer.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    assert attn_err(out[0], attention.quant_attention(inp.q, ref, SM)) <= TOL


def test_peaked_attention_and_extreme_values():
    """A dominant token (large logit) and large-magnitude keys: softmax must not overflow."""
    inp = make_layer(2048, seq=9, dominance_gain=6.0)
    inp.k[:, 100] *= np.float16(8)
    layer = tkv.QuantLayer(bits=4, capacity=2048)
    layer.append(to_new(inp.k), to_new(inp.v))
    ref = check_quant_cache(layer, 0, inp.k, inp.v)
    out = layer.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    assert attn_err(out[0], attention.quant_attention(inp.q, ref, SM)) <= TOL


@pytest.mark.parametrize("bits,g", MAIN_SETTINGS)
@pytest.mark.parametrize("scale", [64.0, 250.0])
def test_large_value_magnitudes(bits, g, scale):
    """Values of magnitude up to about 1000 (scalers of a few hundred): the fp16 operands of
    the matrix-core kernel must not overflow."""
    inp = make_layer(3000, seq=9)
    v = (inp.v.astype(np.float32) * scale).astype(np.float16)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=3008 + 64)
    layer.append(to_new(inp.k), to_new(v))
    ref = check_quant_cache(layer, 0, inp.k, v)
    out = layer.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    assert torch.isfinite(out).all()
    assert attn_err(out[0], attention.quant_attention(inp.q, ref, SM)) <= TOL


@pytest.mark.parametrize("bits,g", MAIN_SETTINGS)
@pytest.mark.parametrize("k_scale,q_scale", [(64.0, 1.0), (1.0, 64.0), (16.0, 16.0)])
def test_large_key_and_query_magnitudes(bits, g, k_scale, q_scale):
    """Keys in the thousands (outlier channels x 64) and large queries: the product of a query
    element and a key scaler must stay inside fp16 on its way to the matrix cores."""
    inp = make_layer(3000, seq=9)
    k = (inp.k.astype(np.float32) * k_scale).astype(np.float16)
    q = (inp.q.astype(np.float32) * q_scale).astype(np.float16)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=3008 + 64)
    layer.append(to_new(k), to_new(inp.v))
    ref = check_quant_cache(layer, 0, k, inp.v)
    out = layer.attn_decode(torch.from_numpy(q)[None].cuda(), SM)
    assert torch.isfinite(out).all()
    assert attn_err(out[0], attention.quant_attention(q, ref, SM)) <= TOL


def test_many_chunks(kernel_choice):
    """More split-K chunks than the usual cap of 64 (forced through the tuning hook): the
    cross-chunk merge then runs in several rounds."""
    if kernel_choice != "mfma":
        pytest.skip("chunk count of the matrix-core kernel")
    n = 16384 + 77
    inp = make_layer(n, config=1, layer=1, seq=31)
    layer = tkv.QuantLayer(bits=2, capacity=16384 + 128)
    layer.append(to_new(inp.k), to_new(inp.v))
    ref = quant.quantize_kv(inp.k, inp.v, bits=2, group=32, residual=128)
    q = torch.from_numpy(inp.q)[None].cuda()
    want = attention.quant_attention(inp.q, ref, SM)
    try:
        for target in (8 * 100, 8 * 256):
            tkv.debug_quant_attn_config(0, target)
            out = layer.attn_decode(q, SM)
            assert attn_err(out[0], want) <= TOL
    finally:
        tkv.debug_quant_attn_config(0, -1)


def test_read_sweep_runs_and_leaves_the_buffer_alone():
    """The measurement kernel of the benchmark: reads only."""
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    before = buf.clone()
    for wgs in (1, 256, 2048):
        tkv.debug_read_sweep(buf, wgs)
    tkv.debug_read_sweep(buf[: 4 * 13])          # shorter than one pass of the grid
    torch.cuda.synchronize()
    assert torch.equal(buf, before)


def test_stream_with_compute_unit_mask():
    """On a stream that may use only part of the machine the split-K launch sizes itself to
    that part; the result does not depend on it."""
    import ctypes as C
    hip = C.CDLL("libamdhip64.so")
    create = hip.hipExtStreamCreateWithCUMask
    create.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_uint32)]
    create.restype = C.c_int
    mask = (C.c_uint32 * 8)(0xFFFF0000, 0xFFFFFFFF, 0xFFFFFFFF, 0x0000FFFF, 0, 0, 0, 0)   # 96 units
    handle = C.c_void_p()
    if create(C.byref(handle), 8, mask) != 0 or not handle.value:
        pytest.skip("streams with a compute-unit mask are not available")
    stream = torch.cuda.ExternalStream(handle.value)
    try:
        inp = make_layer(5000, seq=12)
        layer = tkv.QuantLayer(bits=2, capacity=5056)
        layer.append(to_new(inp.k), to_new(inp.v))
        ref = check_quant_cache(layer, 0, inp.k, inp.v)
        q = torch.from_numpy(inp.q)[None].cuda()
        want = attention.quant_attention(inp.q, ref, SM)
        torch.cuda.synchronize()
        out_masked = layer.attn_decode(q, SM, stream=stream)
        stream.synchronize()
        out_masked = out_masked.clone()
        out_plain = layer.attn_decode(q, SM)
        torch.cuda.synchronize()
        assert attn_err(out_masked[0], want) <= TOL and attn_err(out_plain[0], want) <= TOL
    finally:
        torch.cuda.synchronize()
        hip.hipStreamDestroy.argtypes = [C.c_void_p]
        hip.hipStreamDestroy(handle)
