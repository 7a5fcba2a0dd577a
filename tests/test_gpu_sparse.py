"""GPU parity of the sparse path against the oracle (through the C ABI).
Top-K indices and counts: bit-exact.  Attention: <= 2e-3."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from oracle import attention, sparse
from synth import HeadShape, LayerInputs, make_layer, static_channels

from gpu_util import attn_err, to_new, to_new_batch

pytestmark = pytest.mark.gpu
TOL = 2e-3
SM = 1.0 / np.sqrt(128.0)


def _build(inp, *, top_k, capacity, n_channels=16, shape=None, n_sink=4, n_window=64):
    shape = shape or HeadShape(inp.q.shape[0], inp.k.shape[0], 128)
    layer = tkv.SparseLayer(n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, n_channels=n_channels,
                            top_k=top_k, n_sink=n_sink, n_window=n_window, capacity=capacity)
    ch = static_channels(inp.k, n_channels)
    layer.set_channels(ch[None])
    layer.append(to_new(inp.k), to_new(inp.v))
    return layer, ch


def _check_layer(layer, b, inp, ch, q_dev, out):
    d = layer.desc
    n = inp.k.shape[1]
    summ = sparse.key_summary(inp.k, ch)
    idx, cnt = sparse.estimate_topk(inp.q, summ, ch, n, top_k=d.top_k, n_sink=d.n_sink, n_window=d.n_window)
    torch.cuda.synchronize()
    got_idx = layer.topk_idx[b].cpu().numpy()
    got_cnt = layer.topk_count[b].cpu().numpy()
    assert np.array_equal(got_cnt, cnt)
    assert np.array_equal(got_idx, idx)
    want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, SM, n_sink=d.n_sink, n_window=d.n_window)
    err = attn_err(out[b], want)
    print(f"   n={n} err {err:.3e}", flush=True)
    assert err <= TOL


@pytest.mark.parametrize("n,top_k", [(4096, 128), (1, 128), (3, 16), (68, 16), (69, 16), (70, 128), (1500, 1024),
                                     (5000, 1024), (1024, 128), (1025, 128)])
def test_estimate_topk_gather_attention(n, top_k):
    print(f"case sparse n={n} k={top_k}", flush=True)
    inp = make_layer(n, config=0, layer=1, seq=n % 89)
    layer, ch = _build(inp, top_k=top_k, capacity=max(n, 64) + 37)
    # cache contents: summary, host rows, resident rows
    torch.cuda.synchronize()
    assert np.array_equal(layer.key_summary[0, :, :n].cpu().numpy().view(np.uint16),
                          sparse.key_summary(inp.k, ch).view(np.uint16))
    host = layer.kv_host[0, :, :n].numpy()
    assert np.array_equal(host[:, :, 0].view(np.uint16), inp.k.view(np.uint16))
    assert np.array_equal(host[:, :, 1].view(np.uint16), inp.v.view(np.uint16))
    q = torch.from_numpy(inp.q)[None].cuda()
    layer.estimate_topk(q)
    out = layer.gather_attn(q, SM)
    _check_layer(layer, 0, inp, ch, q, out)
    # the staged rows are the selected rows (the one-stream call above fetches them inside
    # the attention kernel and leaves the staging buffer alone: gather explicitly)
    layer.gather()
    torch.cuda.synchronize()
    cnt = int(layer.topk_count[0, 0])
    if cnt:
        sel = layer.topk_idx[0, 0, :cnt].cpu().numpy()
        st = layer.staging[0, 0, :cnt].cpu().numpy()
        assert np.array_equal(st[:, 0].view(np.uint16), inp.k[0, sel].view(np.uint16))
        assert np.array_equal(st[:, 1].view(np.uint16), inp.v[0, sel].view(np.uint16))


def test_ties_take_lowest_indices():
    """All-equal summaries -> all scores equal -> indices n_sink .. n_sink+k-1."""
    n, top_k = 3000, 128
    inp = make_layer(n, seq=3)
    ch = static_channels(inp.k, 16)
    for h in range(8):
        inp.k[h][:, ch[h]] = inp.k[h][0, ch[h]]
    layer = tkv.SparseLayer(top_k=top_k, capacity=n)
    layer.set_channels(ch[None])
    layer.append(to_new(inp.k), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    idx, cnt = layer.estimate_topk(q)
    torch.cuda.synchronize()
    assert (cnt.cpu().numpy() == top_k).all()
    assert np.array_equal(idx[0].cpu().numpy(), np.tile(np.arange(4, 4 + top_k, dtype=np.int32), (8, 1)))
    out = layer.gather_attn(q, SM)
    _check_layer(layer, 0, inp, ch, q, out)


def test_heavy_ties_quantized_scores():
    """Integer-valued keys/queries give many exactly equal scores at the threshold."""
    rng = np.random.default_rng(2)
    n = 4000
    inp = make_layer(n, seq=4)
    inp.k[:] = rng.integers(-2, 3, size=inp.k.shape).astype(np.float16)
    inp.q[:] = rng.integers(-2, 3, size=inp.q.shape).astype(np.float16)
    layer, ch = _build(inp, top_k=256, capacity=n)
    q = torch.from_numpy(inp.q)[None].cuda()
    layer.estimate_topk(q)
    out = layer.gather_attn(q, SM)
    _check_layer(layer, 0, inp, ch, q, out)


def test_two_streams_and_incremental_append():
    print("case sparse two streams", flush=True)
    n0, extra = 3000, 70
    inp = make_layer(n0 + extra, config=0, layer=1, seq=7)
    layer = tkv.SparseLayer(top_k=128, capacity=4096)
    ch = static_channels(inp.k, 16)
    layer.set_channels(ch[None])
    kd, vd = to_new(inp.k), to_new(inp.v)
    layer.append(kd[:, :n0].contiguous(), vd[:, :n0].contiguous())
    q = torch.from_numpy(inp.q)[None].cuda()
    side = torch.cuda.Stream()
    pos = n0
    for s in [1, 1, 5, 63]:
        layer.append(kd[:, pos:pos + s].contiguous(), vd[:, pos:pos + s].contiguous())
        pos += s
        layer.estimate_topk(q)
        out = layer.gather_attn(q, SM, gather_stream=side)
        sub = LayerInputs(inp.q, inp.k[:, :pos], inp.v[:, :pos], inp.outlier_channels, inp.dominant_tokens)
        _check_layer(layer, 0, sub, ch, q, out)


def test_ragged_batch():
    print("case sparse ragged", flush=True)
    lens = [900, 5, 2000, 68, 1311]
    inps = [make_layer(n, config=4, layer=2, seq=b) for b, n in enumerate(lens)]
    layer = tkv.SparseLayer(top_k=256, capacity=2048, batch=len(lens))
    chs = [static_channels(i.k, 16) for i in inps]
    layer.set_channels(np.stack(chs))
    layer.append(to_new_batch([i.k for i in inps], 2000), to_new_batch([i.v for i in inps], 2000), n_valid=lens)
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    layer.estimate_topk(q)
    out = layer.gather_attn(q, SM)
    for b, inp in enumerate(inps):
        _check_layer(layer, b, inp, chs[b], q, out)


@pytest.mark.parametrize("shape,n_channels", [(HeadShape(8, 8, 128), 16), (HeadShape(16, 8, 128), 8), (HeadShape(32, 8, 128), 12)])
def test_other_shapes(shape, n_channels):
    inp = make_layer(2500, shape=shape, seq=11)
    layer, ch = _build(inp, top_k=200, capacity=2500, n_channels=n_channels, shape=shape)
    q = torch.from_numpy(inp.q)[None].cuda()
    layer.estimate_topk(q)
    out = layer.gather_attn(q, SM)
    _check_layer(layer, 0, inp, ch, q, out)


@pytest.mark.parametrize("shape,n_channels", [(HeadShape(64, 8, 128), 16), (HeadShape(56, 8, 128), 16),
                                              (HeadShape(10, 2, 128), 12), (HeadShape(6, 1, 128), 8),
                                              (HeadShape(3, 1, 128), 16)])
def test_groups_of_up_to_eight_query_heads(shape, n_channels):
    """Groups of 5 to 8 query heads per KV head: the scores are summed over all of them (their
    channels read from LDS), the attention kernels hold eight heads per KV row.  Every form of the
    attention call: rows fetched inside the launch, gathered on a side stream, staged first."""
    print(f"case sparse Hq={shape.n_q_heads} Hkv={shape.n_kv_heads} d_s={n_channels}", flush=True)
    for n, top_k in ((6000, 512), (300, 64)):
        inp = make_layer(n, shape=shape, seq=5)
        layer, ch = _build(inp, top_k=top_k, capacity=n + 8, n_channels=n_channels, shape=shape)
        q = torch.from_numpy(inp.q)[None].cuda()
        layer.estimate_topk(q)
        _check_layer(layer, 0, inp, ch, q, layer.gather_attn(q, SM))
        side = torch.cuda.Stream()
        _check_layer(layer, 0, inp, ch, q, layer.gather_attn(q, SM, gather_stream=side.cuda_stream))
        layer.gather()
        _check_layer(layer, 0, inp, ch, q, layer.attn(q, SM))
        # tkv_sparse_decode: one launch for groups of up to 4, two launches behind the same call above
        layer.topk_idx.fill_(-7)
        _check_layer(layer, 0, inp, ch, q, layer.decode(q, SM))
        # ... and with the step's append: one more token, then the same checks on the grown prefix
        if n == 6000:
            rng = np.random.default_rng(n)
            extra_k = rng.standard_normal((shape.n_kv_heads, 1, 128)).astype(np.float16)
            extra_v = rng.standard_normal((shape.n_kv_heads, 1, 128)).astype(np.float16)
            grown = dataclasses.replace(inp, k=np.concatenate([inp.k, extra_k], axis=1),
                                        v=np.concatenate([inp.v, extra_v], axis=1))
            out = layer.decode(q, SM, to_new(extra_k), to_new(extra_v))
            _check_layer(layer, 0, grown, ch, q, out)


def test_ties_beyond_the_on_chip_list():
    """All scores equal at a length where the candidates (every token) do not fit the
    selection kernel's on-chip list: indices are still n_sink .. n_sink + k - 1."""
    n, top_k = 20000, 1024
    inp = make_layer(n, seq=33)
    ch = static_channels(inp.k, 16)
    k = inp.k.copy()
    for h in range(8):
        k[h][:, ch[h]] = np.float16(0.5)
    layer = tkv.SparseLayer(top_k=top_k, capacity=n)
    layer.set_channels(ch[None])
    layer.append(to_new(k), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    idx, cnt = layer.estimate_topk(q)
    torch.cuda.synchronize()
    want_idx, want_cnt = sparse.estimate_topk(inp.q, sparse.key_summary(k, ch), ch, n, top_k=top_k, n_sink=4, n_window=64)
    assert np.array_equal(cnt[0].cpu().numpy(), want_cnt)
    assert np.array_equal(idx[0].cpu().numpy(), want_idx)
    assert np.array_equal(want_idx[0, :top_k], np.arange(4, 4 + top_k))


@pytest.mark.parametrize("n0,steps", [(3000, [1] * 70 + [3, 8, 1]), (0, [1, 1, 2, 8, 1] * 15), (60, [1] * 12)])
def test_decode_steps_with_append_inside_the_scoring_launch(n0, steps):
    """tkv_sparse_append_estimate_topk: a decode loop that crosses the sink and window
    boundaries; after every step the selection and the attention are the oracle's for the
    whole prefix, and at the end the host cache and the summary hold every token."""
    print(f"case sparse fused append n0={n0}", flush=True)
    total = n0 + sum(steps)
    inp = make_layer(total, config=0, layer=1, seq=11)
    layer = tkv.SparseLayer(top_k=128, capacity=total + 5)
    ch = static_channels(inp.k, 16)
    layer.set_channels(ch[None])
    kd, vd = to_new(inp.k), to_new(inp.v)
    if n0:
        layer.append(kd[:, :n0].contiguous(), vd[:, :n0].contiguous())
    q = torch.from_numpy(inp.q)[None].cuda()
    pos = n0
    for i, s in enumerate(steps):
        layer.append_estimate_topk(kd[:, pos:pos + s].contiguous(), vd[:, pos:pos + s].contiguous(), q)
        pos += s
        assert int(layer.seq_len[0]) == pos
        out = layer.gather_attn(q, SM)
        if i % 7 == 0 or i >= len(steps) - 3:
            sub = LayerInputs(inp.q, inp.k[:, :pos], inp.v[:, :pos], inp.outlier_channels, inp.dominant_tokens)
            _check_layer(layer, 0, sub, ch, q, out)
    torch.cuda.synchronize()
    assert np.array_equal(layer.key_summary[0, :, :total].cpu().numpy().view(np.uint16),
                          sparse.key_summary(inp.k, ch).view(np.uint16))
    host = layer.kv_host[0, :, :total].numpy()
    assert np.array_equal(host[:, :, 0].view(np.uint16), inp.k.view(np.uint16))
    assert np.array_equal(host[:, :, 1].view(np.uint16), inp.v.view(np.uint16))
    # too many rows for the fused form
    with pytest.raises(tkv.TkvError):
        layer.append_estimate_topk(kd[:, :9].contiguous(), vd[:, :9].contiguous(), q)


@pytest.mark.parametrize("units", [224, 96, 8])
def test_streams_with_compute_unit_masks(units):
    """Scoring, Top-K, gather and attention on a stream that may use only part of the machine:
    the token split follows the stream's mask, the results do not depend on it."""
    import ctypes as C
    hip = C.CDLL("libamdhip64.so")
    create = hip.hipExtStreamCreateWithCUMask
    create.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_uint32)]
    create.restype = C.c_int
    bits = ((1 << 256) - 1) ^ ((1 << (256 - units)) - 1) if units >= 32 else (1 << units) - 1
    mask = (C.c_uint32 * 8)(*[(bits >> (32 * i)) & 0xFFFFFFFF for i in range(8)])
    handle = C.c_void_p()
    if create(C.byref(handle), 8, mask) != 0 or not handle.value:
        hip.hipGetLastError()
        pytest.skip("streams with a compute-unit mask are not available")
    stream = torch.cuda.ExternalStream(handle.value)
    try:
        n = 9000
        inp = make_layer(n, config=0, layer=1, seq=5)
        layer, ch = _build(inp, top_k=1024, capacity=n + 40)
        q = torch.from_numpy(inp.q)[None].cuda()
        out = torch.empty(1, inp.q.shape[0], 128, dtype=torch.float16, device="cuda")
        torch.cuda.synchronize()
        layer.estimate_topk(q, stream=stream)
        layer.gather_attn(q, SM, out=out, gather_stream=stream, compute_stream=stream)
        stream.synchronize()
        _check_layer(layer, 0, inp, ch, q, out)
    finally:
        torch.cuda.synchronize()
        hip.hipStreamDestroy.argtypes = [C.c_void_p]
        hip.hipStreamDestroy(handle)


def _only_topk(inp, k_mod, ch, top_k):
    n = inp.k.shape[1]
    layer = tkv.SparseLayer(top_k=top_k, capacity=n)
    layer.set_channels(ch[None])
    layer.append(to_new(k_mod), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    idx, cnt = layer.estimate_topk(q)
    torch.cuda.synchronize()
    want_idx, want_cnt = sparse.estimate_topk(inp.q, sparse.key_summary(k_mod, ch), ch, n, top_k=top_k,
                                              n_sink=4, n_window=64)
    assert np.array_equal(cnt[0].cpu().numpy(), want_cnt)
    assert np.array_equal(idx[0].cpu().numpy(), want_idx)
    # the same call again on the same workspace: histogram and counters were left clean
    idx, cnt = layer.estimate_topk(q)
    torch.cuda.synchronize()
    assert np.array_equal(idx[0].cpu().numpy(), want_idx)
    return want_idx


@pytest.mark.parametrize("n,top_k,spans", [
    (20000, 1024, [(2100, 2900)]),                 # one workgroup's share holds most of the Top-K
    (20000, 1024, [(0, 700), (19000, 20000)]),     # first and last share (sinks / window cut into them)
    (131072, 1024, [(70000, 70600), (4096, 4500)]),
    (131072, 4096, [(100000, 104000)]),
    (9000, 512, [(1000, 1010), (5000, 5400)]),
])
def test_topk_concentrated_in_few_shares(n, top_k, spans):
    """The scoring workgroups list their tokens down to a bin guessed from an even spread of the
    Top-K over the context.  Here the Top-K is far from evenly spread: tokens of a few short spans
    score several times higher than the rest, so the guess of the workgroups that own them stops
    short and the head's last workgroup has to rebuild their lists.  The result is the oracle's
    all the same."""
    print(f"case topk concentrated n={n} k={top_k} spans={spans}", flush=True)
    inp = make_layer(n, config=2, layer=4, seq=len(spans))
    ch = static_channels(inp.k, 16)
    k = inp.k.copy()
    for a, b in spans:
        # aligned with the summed query of each head's group on the critical channels: large positive scores
        for h in range(8):
            qsum = inp.q[4 * h:4 * h + 4].astype(np.float32).sum(axis=0)[ch[h]]
            boost = 3.0 * np.sign(qsum) * np.abs(k[h, a:b][:, ch[h]].astype(np.float32))
            k[h, a:b][:, ch[h]] = boost.astype(np.float16)
    idx = _only_topk(inp, k, ch, top_k)
    inside = sum(int(((idx[0] >= a) & (idx[0] < b)).sum()) for a, b in spans)
    print(f"   {inside} of {top_k} selected tokens of head 0 lie in the spans", flush=True)
    assert inside > top_k // 4


def test_topk_heavy_ties_concentrated():
    """Integer-valued scores (many exact ties at the threshold) with the large values packed into
    one span: rebuilt lists and the tie rule (lower index first) together."""
    rng = np.random.default_rng(12)
    n, top_k = 30000, 1024
    inp = make_layer(n, seq=44)
    ch = static_channels(inp.k, 16)
    k = inp.k.copy()
    k[:] = rng.integers(-1, 2, size=k.shape).astype(np.float16)
    k[:, 12000:13500] = rng.integers(1, 4, size=(8, 1500, 128)).astype(np.float16)
    inp.q[:] = rng.integers(0, 3, size=inp.q.shape).astype(np.float16)
    _only_topk(inp, k, ch, top_k)
