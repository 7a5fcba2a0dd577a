"""tkv_sparse_decode (append + scoring + Top-K + fetch + attention in one launch) against the
oracle, through the C ABI: indices bit-exact, attention <= 2e-3."""
import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from oracle import sparse
from synth import HeadShape, LayerInputs, make_layer, ragged_lengths, static_channels

from gpu_util import attn_err, to_new, to_new_batch

pytestmark = pytest.mark.gpu
TOL = 2e-3
SM = 1.0 / np.sqrt(128.0)


def _check(layer, b, inp, ch, out, n=None):
    d = layer.desc
    n = inp.k.shape[1] if n is None else n
    k, v = inp.k[:, :n], inp.v[:, :n]
    idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(k, ch), ch, n, top_k=d.top_k, n_sink=d.n_sink,
                                    n_window=d.n_window)
    torch.cuda.synchronize()
    assert np.array_equal(layer.topk_count[b].cpu().numpy(), cnt)
    assert np.array_equal(layer.topk_idx[b].cpu().numpy(), idx)
    want = sparse.sparse_attention(inp.q, k, v, idx, cnt, n, SM, n_sink=d.n_sink, n_window=d.n_window)
    err = attn_err(out[b], want)
    print(f"   n={n} err {err:.3e}", flush=True)
    assert err <= TOL


@pytest.mark.parametrize("n,top_k", [(4096, 128), (1, 128), (3, 16), (68, 16), (69, 16), (70, 128), (1500, 1024),
                                     (5000, 1024), (20000, 1024), (9000, 4096)])
def test_decode_without_append(n, top_k):
    print(f"case sparse decode n={n} k={top_k}", flush=True)
    inp = make_layer(n, config=0, layer=1, seq=n % 83)
    layer = tkv.SparseLayer(top_k=top_k, capacity=max(n, 64) + 37)
    ch = static_channels(inp.k, 16)
    layer.set_channels(ch[None])
    layer.append(to_new(inp.k), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    out = layer.decode(q, SM)
    _check(layer, 0, inp, ch, out)
    out2 = layer.decode(q, SM)          # same workspace again: counters were left clean
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    # the hint that warms up the next layer's key summary changes nothing (here: a second layer of
    # the same shape, whose summary must come through untouched)
    other = tkv.SparseLayer(top_k=top_k, capacity=max(n, 64) + 37)
    other.key_summary.view(-1)[:] = 0.5
    idx0 = layer.topk_idx.clone()
    out3 = layer.decode(q, SM, warm_next=other)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out3.view(torch.int16)) and torch.equal(idx0, layer.topk_idx)
    assert bool((other.key_summary == 0.5).all())


@pytest.mark.parametrize("n0,steps", [(3000, [1] * 70 + [3, 8, 1]), (0, [1, 1, 2, 8, 1] * 15), (60, [1] * 12)])
def test_decode_loop_with_append(n0, steps):
    """A decode loop that crosses the sink and window boundaries: after every step the selection
    and the attention are the oracle's for the whole prefix (the step's own tokens included: they
    are in the window), and at the end the host cache and the summary hold every token."""
    print(f"case sparse decode loop n0={n0}", flush=True)
    total = n0 + sum(steps)
    inp = make_layer(total, config=0, layer=1, seq=13)
    layer = tkv.SparseLayer(top_k=128, capacity=total + 5)
    ch = static_channels(inp.k, 16)
    layer.set_channels(ch[None])
    kd, vd = to_new(inp.k), to_new(inp.v)
    if n0:
        layer.append(kd[:, :n0].contiguous(), vd[:, :n0].contiguous())
    q = torch.from_numpy(inp.q)[None].cuda()
    pos = n0
    for i, s in enumerate(steps):
        out = layer.decode(q, SM, kd[:, pos:pos + s].contiguous(), vd[:, pos:pos + s].contiguous())
        pos += s
        assert int(layer.seq_len[0]) == pos
        if i % 7 == 0 or i >= len(steps) - 3:
            _check(layer, 0, inp, ch, out, n=pos)
    torch.cuda.synchronize()
    assert np.array_equal(layer.key_summary[0, :, :total].cpu().numpy().view(np.uint16),
                          sparse.key_summary(inp.k, ch).view(np.uint16))
    host = layer.kv_host[0, :, :total].numpy()
    assert np.array_equal(host[:, :, 0].view(np.uint16), inp.k.view(np.uint16))
    assert np.array_equal(host[:, :, 1].view(np.uint16), inp.v.view(np.uint16))
    # resident rows: the separate attention call reads them from kv_local
    layer.estimate_topk(q)
    out2 = layer.gather_attn(q, SM)
    _check(layer, 0, inp, ch, out2)


def test_decode_full_size_and_concentrated():
    """N = 131072, k = 1024, once as generated and once with the Top-K packed into two short
    spans (the selection's slow path) - followed by the fetch and the attention either way."""
    n, top_k = 131072, 1024
    print(f"case sparse decode full size n={n}", flush=True)
    inp = make_layer(n, config=2, layer=5, seq=3)
    ch = static_channels(inp.k, 16)
    for spans in ([], [(70000, 70600), (4096, 4500)]):
        k = inp.k.copy()
        for a, b in spans:
            for h in range(8):
                qsum = inp.q[4 * h:4 * h + 4].astype(np.float32).sum(axis=0)[ch[h]]
                k[h, a:b][:, ch[h]] = (3.0 * np.sign(qsum) * np.abs(k[h, a:b][:, ch[h]].astype(np.float32))).astype(np.float16)
        layer = tkv.SparseLayer(top_k=top_k, capacity=n + 16)
        layer.set_channels(ch[None])
        layer.append(to_new(k), to_new(inp.v))
        q = torch.from_numpy(inp.q)[None].cuda()
        new = make_layer(1, config=2, layer=6, seq=4)
        out = layer.decode(q, SM, to_new(new.k), to_new(new.v))
        full = LayerInputs(inp.q, np.concatenate([k, new.k], axis=1), np.concatenate([inp.v, new.v], axis=1),
                           inp.outlier_channels, inp.dominant_tokens)
        _check(layer, 0, full, ch, out)
        del layer


def test_decode_ragged_batch_and_other_shapes():
    lens = ragged_lengths(8, 4096, 8192).tolist()
    lens[2] = 0
    lens[5] = 37
    print(f"case sparse decode ragged lens={lens}", flush=True)
    nmax = max(lens)
    inps = [make_layer(max(n, 1), config=4, layer=3, seq=b) for b, n in enumerate(lens)]
    layer = tkv.SparseLayer(top_k=1024, capacity=8192 + 8, batch=8)
    chs = [static_channels(i.k, 16) for i in inps]
    layer.set_channels(np.stack(chs))
    layer.append(to_new_batch([i.k[:, :n] for i, n in zip(inps, lens)], nmax),
                 to_new_batch([i.v[:, :n] for i, n in zip(inps, lens)], nmax), n_valid=lens)
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    out = layer.decode(q, SM)
    torch.cuda.synchronize()
    for b, inp in enumerate(inps):
        if lens[b] == 0:
            assert (out[b] == 0).all() and int(layer.topk_count[b].sum()) == 0
            continue
        _check(layer, b, inp, chs[b], out, n=lens[b])
    for shape, ds in ((HeadShape(8, 8, 128), 16), (HeadShape(16, 8, 128), 8), (HeadShape(32, 8, 128), 12)):
        inp = make_layer(2500, shape=shape, seq=17)
        sl = tkv.SparseLayer(n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, n_channels=ds, top_k=200,
                             capacity=2500)
        ch = static_channels(inp.k, ds)
        sl.set_channels(ch[None])
        sl.append(to_new(inp.k), to_new(inp.v))
        out = sl.decode(torch.from_numpy(inp.q)[None].cuda(), SM)
        _check(sl, 0, inp, ch, out)
