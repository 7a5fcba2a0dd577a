"""GPU parity of Stage 1 of the dynamic retrieval (Sec. 4.2: channel maxima, Eq. 10
channel selection, fetch of the critical key cache) and of Stage 2 over a channel-major
critical key cache, against the oracle (through the C ABI).  Channel lists, fetched keys,
Top-K indices and counts: bit-exact.  Attention: <= 2e-3."""
import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from oracle import attention, sparse
from synth import HeadShape, make_layer

from gpu_util import attn_err, to_new, to_new_batch

pytestmark = pytest.mark.gpu
TOL = 2e-3
SM = 1.0 / np.sqrt(128.0)


def _layer(inp, *, top_k, capacity, n_channels=16, resident=False, shape=None):
    shape = shape or HeadShape(inp.q.shape[0], inp.k.shape[0], 128)
    layer = tkv.SparseLayer(n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, n_channels=n_channels,
                            top_k=top_k, capacity=capacity)
    return layer, tkv.Stage1(layer, resident=resident)


def _append(layer, s1, k, v, pieces, both=False):
    """Append in the given piece sizes: Stage 1 buffers first, then the layer's own; or both
    through the combined entry point (short pieces then take its single-launch path)."""
    kd, vd = to_new(k), to_new(v)
    pos = 0
    for s in pieces:
        kn, vn = kd[:, pos:pos + s].contiguous(), vd[:, pos:pos + s].contiguous()
        if both:
            s1.append_both(kn, vn)
        else:
            s1.append(kn)
            layer.append(kn, vn)
        pos += s
    assert pos == k.shape[1]


def _check_stage1_buffers(s1, b, k):
    n = k.shape[1]
    torch.cuda.synchronize()
    assert np.array_equal(s1.k_absmax[b].cpu().numpy(), sparse.channel_absmax(k))
    got = s1.keys_cm[b, :, :, :n].cpu().numpy()                       # [Hkv, D, n]
    assert np.array_equal(got.view(np.uint16), np.ascontiguousarray(k.transpose(0, 2, 1)).view(np.uint16))


@pytest.mark.parametrize("resident", [False, True])
@pytest.mark.parametrize("n,top_k,pieces", [
    (4096, 128, [4096]), (1, 16, [1]), (70, 16, [70]), (1000, 128, [1, 63, 64, 65, 7, 800]),
    (5000, 1024, [4999, 1]), (4100, 1024, [3, 4097]), (300, 128, [200, 8, 9, 1, 1, 1, 2, 70, 8]),
])
def test_select_fetch_score_attend(resident, n, top_k, pieces):
    print(f"case stage1 n={n} k={top_k} resident={resident}", flush=True)
    inp = make_layer(n, config=0, layer=1, seq=n % 83)
    layer, s1 = _layer(inp, top_k=top_k, capacity=(max(n, 64) + 37 + 7) // 8 * 8, resident=resident)
    _append(layer, s1, inp.k, inp.v, pieces, both=(n % 2 == 0))
    torch.cuda.synchronize()
    host = layer.kv_host[0, :, :n].numpy()     # the layer's own cache, whichever entry point filled it
    assert np.array_equal(host[:, :, 0].view(np.uint16), inp.k.view(np.uint16))
    assert np.array_equal(host[:, :, 1].view(np.uint16), inp.v.view(np.uint16))
    _check_stage1_buffers(s1, 0, inp.k)
    # the query itself stands in for the predicted query of App. B
    q = torch.from_numpy(inp.q)[None].cuda()
    ch_dev = s1.select_channels(q)
    ch = sparse.select_channels(inp.q, sparse.channel_absmax(inp.k), 16)
    torch.cuda.synchronize()
    assert np.array_equal(ch_dev[0].cpu().numpy(), ch)
    summ = sparse.key_summary(inp.k, ch)                              # [Hkv, n, d_s]
    idx, cnt = sparse.estimate_topk(inp.q, summ, ch, n, top_k=top_k, n_sink=4, n_window=64)
    # fetched critical key cache, in both halves of the double buffer
    for buf in (0, 1):
        keys = s1.prefetch(buf)
        torch.cuda.synchronize()
        assert np.array_equal(keys[0, :, :, :n].cpu().numpy().view(np.uint16),
                              np.ascontiguousarray(summ.transpose(0, 2, 1)).view(np.uint16))
        layer.topk_idx.fill_(-7)
        s1.estimate_topk(q, buf)
        torch.cuda.synchronize()
        assert np.array_equal(layer.topk_count[0].cpu().numpy(), cnt)
        assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)
    if resident:  # scoring in place over the resident channel-major keys
        layer.topk_idx.fill_(-7)
        s1.estimate_topk(q, None)
        torch.cuda.synchronize()
        assert np.array_equal(layer.topk_count[0].cpu().numpy(), cnt)
        assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)
        # Stage 1 and Stage 2 in one call
        layer.topk_idx.fill_(-7)
        s1.channel_idx.fill_(-7)
        s1.select_estimate_topk(q, q)
        torch.cuda.synchronize()
        assert np.array_equal(s1.channel_idx[0].cpu().numpy(), ch)
        assert np.array_equal(layer.topk_count[0].cpu().numpy(), cnt)
        assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)
    else:
        with pytest.raises(tkv.TkvError):   # in-place scoring needs resident keys
            s1.select_estimate_topk(q, q)
    out = layer.gather_attn(q, SM)
    want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, SM, n_sink=4, n_window=64)
    assert attn_err(out[0], want) <= TOL


def test_dynamic_channels_follow_the_query():
    """A query concentrated on a few channels must pull those channels into the list,
    whatever the static statistics of the keys say (the point of Eq. 10)."""
    n = 2048
    inp = make_layer(n, config=0, layer=1, seq=5)
    layer, s1 = _layer(inp, top_k=128, capacity=2048 + 64)
    _append(layer, s1, inp.k, inp.v, [n])
    q = np.full_like(inp.q, np.float16(0.01))
    want_channels = [3, 17, 60, 101]
    q[:, want_channels] = np.float16(8.0)
    ch_dev = s1.select_channels(torch.from_numpy(q)[None].cuda())
    torch.cuda.synchronize()
    got = ch_dev[0].cpu().numpy()
    assert np.array_equal(got, sparse.select_channels(q, sparse.channel_absmax(inp.k), 16))
    for h in range(8):
        assert set(want_channels) <= set(got[h].tolist())


def test_ragged_batch_other_grouping_and_eight_channels():
    shape = HeadShape(16, 8, 128)
    lens = [700, 1, 2048, 333]
    inps = [make_layer(n, config=4, layer=1, seq=b, shape=shape) for b, n in enumerate(lens)]
    layer = tkv.SparseLayer(n_q_heads=16, n_kv_heads=8, n_channels=8, top_k=128, capacity=2048, batch=len(lens))
    s1 = tkv.Stage1(layer)
    kd = to_new_batch([i.k for i in inps], 2048)
    vd = to_new_batch([i.v for i in inps], 2048)
    s1.append(kd, n_valid=lens)
    layer.append(kd, vd, n_valid=lens)
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    ch_dev = s1.select_channels(q)
    keys = s1.prefetch(0)
    s1.estimate_topk(q, 0)
    out = layer.gather_attn(q, SM)
    torch.cuda.synchronize()
    for b, inp in enumerate(inps):
        n = lens[b]
        _check_stage1_buffers(s1, b, inp.k)
        ch = sparse.select_channels(inp.q, sparse.channel_absmax(inp.k), 8)
        assert np.array_equal(ch_dev[b].cpu().numpy(), ch)
        summ = sparse.key_summary(inp.k, ch)
        assert np.array_equal(keys[b, :, :, :n].cpu().numpy().view(np.uint16),
                              np.ascontiguousarray(summ.transpose(0, 2, 1)).view(np.uint16))
        idx, cnt = sparse.estimate_topk(inp.q, summ, ch, n, top_k=128, n_sink=4, n_window=64)
        assert np.array_equal(layer.topk_count[b].cpu().numpy(), cnt)
        assert np.array_equal(layer.topk_idx[b].cpu().numpy(), idx)
        want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, SM, n_sink=4, n_window=64)
        assert attn_err(out[b], want) <= TOL


@pytest.mark.parametrize("resident", [False, True])
def test_groups_of_eight_query_heads(resident):
    """Eq. 10 sums |q| over all eight heads of a group; Stage 2 over the fetched or resident
    channel-major keys."""
    shape = HeadShape(16, 2, 128)
    n = 3000
    inp = make_layer(n, config=4, layer=1, seq=3, shape=shape)
    layer, s1 = _layer(inp, top_k=256, capacity=n + 8, resident=resident, shape=shape)
    _append(layer, s1, inp.k, inp.v, [n - 1, 1], both=True)
    q = torch.from_numpy(inp.q)[None].cuda()
    if resident:
        s1.select_estimate_topk(q, q)
        ch_dev = s1.channel_idx
    else:
        ch_dev = s1.select_channels(q)
        s1.prefetch(0)
        s1.estimate_topk(q, 0)
    out = layer.gather_attn(q, SM)
    torch.cuda.synchronize()
    ch = sparse.select_channels(inp.q, sparse.channel_absmax(inp.k), 16)
    assert np.array_equal(ch_dev[0].cpu().numpy(), ch)
    idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, ch), ch, n, top_k=256, n_sink=4, n_window=64)
    assert np.array_equal(layer.topk_count[0].cpu().numpy(), cnt)
    assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)
    want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, SM, n_sink=4, n_window=64)
    assert attn_err(out[0], want) <= TOL


def test_the_papers_long_context_setting():
    """Sec. 5.1 / App. D: 12 critical channels, n_local = 128 (no separate sinks), n_topk = 896,
    channels re-selected from the query, keys fetched from the host copy."""
    n = 6000
    inp = make_layer(n, config=0, layer=1, seq=21)
    layer = tkv.SparseLayer(n_channels=12, top_k=896, n_sink=0, n_window=128, capacity=6000)
    s1 = tkv.Stage1(layer)
    _append(layer, s1, inp.k, inp.v, [5990, 8, 2], both=True)
    q = torch.from_numpy(inp.q)[None].cuda()
    ch_dev = s1.select_channels(q)
    s1.prefetch(0)
    s1.estimate_topk(q, 0)
    out = layer.gather_attn(q, SM)
    torch.cuda.synchronize()
    ch = sparse.select_channels(inp.q, sparse.channel_absmax(inp.k), 12)
    assert np.array_equal(ch_dev[0].cpu().numpy(), ch)
    idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, ch), ch, n, top_k=896, n_sink=0, n_window=128)
    assert np.array_equal(layer.topk_count[0].cpu().numpy(), cnt)
    assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)
    want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, SM, n_sink=0, n_window=128)
    assert attn_err(out[0], want) <= TOL
    # the same list through the token-major summary (static path with 12 channels)
    layer2 = tkv.SparseLayer(n_channels=12, top_k=896, n_sink=0, n_window=128, capacity=6000)
    layer2.set_channels(ch[None])
    layer2.append(to_new(inp.k), to_new(inp.v))
    layer2.estimate_topk(q)
    torch.cuda.synchronize()
    assert np.array_equal(layer2.topk_idx[0].cpu().numpy(), idx)


def test_argument_errors():
    inp = make_layer(100, seq=1)
    layer = tkv.SparseLayer(top_k=16, capacity=100)          # capacity not a multiple of 8
    with pytest.raises(tkv.TkvError):
        s1 = tkv.Stage1(layer)
        s1.append(to_new(inp.k))
