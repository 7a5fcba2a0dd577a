"""Parity at the benchmark's full sizes, in the launch configuration bench.py times
(same library defaults): quantized layer at N = 32768 (2 and 4 bit) and N = 131072,
sparse layer at N = 131072 with k = 1024, batched ragged decode."""
import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from oracle import attention, quant, sparse
from synth import make_layer, ragged_lengths, static_channels

from gpu_util import attn_err, attn_err_elementwise, check_quant_cache, to_new, to_new_batch

pytestmark = pytest.mark.gpu
TOL = 2e-3
SM = 1.0 / np.sqrt(128.0)


@pytest.mark.parametrize("n,bits,g", [(32768, 2, 32), (32768, 4, 32), (131072, 2, 32), (131072, 1, 64), (32768, 2, 64)])
def test_quant_layer_full_size(n, bits, g):
    print(f"case full-size quant n={n} bits={bits} g={g}", flush=True)
    inp = make_layer(n, config=1, layer=0, seq=bits)
    layer = tkv.QuantLayer(bits=bits, group_size=g, capacity=n + 64)
    layer.append(to_new(inp.k), to_new(inp.v))
    ref = check_quant_cache(layer, 0, inp.k, inp.v)          # every code, scaler, zero-point
    out = layer.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    want = attention.quant_attention(inp.q, ref, SM)
    err = attn_err(out[0], want)
    print(f"   err {err:.3e} (element-wise with 2e-3 rms floor: {attn_err_elementwise(out[0], want):.3e})", flush=True)
    assert err <= TOL
    # one decoded token more: the single-token append path at full size
    new = make_layer(1, config=1, layer=1, seq=bits)
    layer.append(to_new(new.k), to_new(new.v))
    k2 = np.concatenate([inp.k, new.k], axis=1)
    v2 = np.concatenate([inp.v, new.v], axis=1)
    layer2 = tkv.QuantLayer(bits=bits, group_size=g, capacity=n + 64)
    layer2.append(to_new(k2), to_new(v2))
    a = layer.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    b = layer2.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    assert attn_err(a[0], b[0].float().cpu().numpy().astype(np.float64)) <= TOL
    # ... and a third through tkv_quant_decode (append inside the attention launch: what the
    # benchmark's chained step runs), against the oracle over the grown cache
    new3 = make_layer(1, config=1, layer=2, seq=bits)
    out3 = layer.decode(torch.from_numpy(inp.q)[None].cuda(), SM, to_new(new3.k), to_new(new3.v))
    k3 = np.concatenate([k2, new3.k], axis=1)
    v3 = np.concatenate([v2, new3.v], axis=1)
    ref3 = check_quant_cache(layer, 0, k3, v3)
    err3 = attn_err(out3[0], attention.quant_attention(inp.q, ref3, SM))
    print(f"   one-call step err {err3:.3e}", flush=True)
    assert err3 <= TOL


def test_sparse_layer_full_size():
    n, top_k = 131072, 1024
    print(f"case full-size sparse n={n}", flush=True)
    inp = make_layer(n, config=2, layer=0, seq=0)
    layer = tkv.SparseLayer(top_k=top_k, capacity=n)
    ch = static_channels(inp.k, 16)
    layer.set_channels(ch[None])
    layer.append(to_new(inp.k), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    layer.estimate_topk(q)
    out = layer.gather_attn(q, SM, gather_stream=torch.cuda.Stream())
    idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, ch), ch, n, top_k=top_k, n_sink=4, n_window=64)
    torch.cuda.synchronize()
    assert np.array_equal(layer.topk_count[0].cpu().numpy(), cnt)
    assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)
    want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, SM, n_sink=4, n_window=64)
    err = attn_err(out[0], want)
    print(f"   err {err:.3e} (element-wise with 2e-3 rms floor: {attn_err_elementwise(out[0], want):.3e})", flush=True)
    assert err <= TOL
    # a second call on the same workspace (self-cleaning counters) gives the same indices
    layer.estimate_topk(q)
    torch.cuda.synchronize()
    assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)


def test_stage1_full_size():
    """Dynamic channels at the full context: maxima, Eq. 10 list, fetched critical key cache
    (pinned-host channel-major keys), Stage 2 over it."""
    n, top_k = 131072, 1024
    print(f"case full-size stage 1 n={n}", flush=True)
    inp = make_layer(n, config=2, layer=1, seq=1)
    layer = tkv.SparseLayer(top_k=top_k, capacity=n)
    s1 = tkv.Stage1(layer)
    kd, vd = to_new(inp.k), to_new(inp.v)
    s1.append(kd)
    layer.append(kd, vd)
    q = torch.from_numpy(inp.q)[None].cuda()
    ch_dev = s1.select_channels(q)
    keys = s1.prefetch(1)
    s1.estimate_topk(q, 1)
    torch.cuda.synchronize()
    amax = sparse.channel_absmax(inp.k)
    assert np.array_equal(s1.k_absmax[0].cpu().numpy(), amax)
    ch = sparse.select_channels(inp.q, amax, 16)
    assert np.array_equal(ch_dev[0].cpu().numpy(), ch)
    summ = sparse.key_summary(inp.k, ch)
    assert np.array_equal(keys[0].cpu().numpy().view(np.uint16),
                          np.ascontiguousarray(summ.transpose(0, 2, 1)).view(np.uint16))
    idx, cnt = sparse.estimate_topk(inp.q, summ, ch, n, top_k=top_k, n_sink=4, n_window=64)
    assert np.array_equal(layer.topk_count[0].cpu().numpy(), cnt)
    assert np.array_equal(layer.topk_idx[0].cpu().numpy(), idx)


@pytest.mark.parametrize("lo,hi", [(4096, 8192), (16384, 32768)])
def test_batched_ragged_hybrid(lo, hi):
    """Batch 8, ragged lengths: the batched configuration at its own sizes (16384..32768
    tokens per sequence) and a scaled-down version."""
    lens = ragged_lengths(8, lo, hi).tolist()
    print(f"case batched ragged lens={lens}", flush=True)
    nmax = max(lens)
    inps = [make_layer(n, config=4, layer=0, seq=b) for b, n in enumerate(lens)]
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    kb, vb = to_new_batch([i.k for i in inps], nmax), to_new_batch([i.v for i in inps], nmax)
    ql = tkv.QuantLayer(bits=2, capacity=hi, batch=8)
    ql.append(kb, vb, n_valid=lens)
    out = ql.attn_decode(q, SM)
    sl = tkv.SparseLayer(top_k=1024, capacity=hi, batch=8)
    chs = [static_channels(i.k, 16) for i in inps]
    sl.set_channels(np.stack(chs))
    sl.append(kb, vb, n_valid=lens)
    sl.estimate_topk(q)
    out_s = sl.gather_attn(q, SM, gather_stream=torch.cuda.Stream())
    torch.cuda.synchronize()
    for b, inp in enumerate(inps):
        ref = check_quant_cache(ql, b, inp.k, inp.v)
        assert attn_err(out[b], attention.quant_attention(inp.q, ref, SM)) <= TOL
        idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, chs[b]), chs[b], lens[b],
                                        top_k=1024, n_sink=4, n_window=64)
        assert np.array_equal(sl.topk_idx[b].cpu().numpy(), idx)
        want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, lens[b], SM, n_sink=4, n_window=64)
        assert attn_err(out_s[b], want) <= TOL


def test_limits_of_the_descriptor():
    """Largest supported Top-K / window / residual."""
    n = 9000
    inp = make_layer(n, seq=21)
    sl = tkv.SparseLayer(top_k=4096, n_sink=16, n_window=1024, capacity=n)
    ch = static_channels(inp.k, 16)
    sl.set_channels(ch[None])
    sl.append(to_new(inp.k), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    sl.estimate_topk(q)
    out = sl.gather_attn(q, SM)
    idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, ch), ch, n, top_k=4096, n_sink=16, n_window=1024)
    torch.cuda.synchronize()
    assert np.array_equal(sl.topk_idx[0].cpu().numpy(), idx)
    want = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, SM, n_sink=16, n_window=1024)
    assert attn_err(out[0], want) <= TOL
    ql = tkv.QuantLayer(bits=4, residual=992, capacity=4096)
    inp = make_layer(3000, seq=22)
    ql.append(to_new(inp.k), to_new(inp.v))
    ref = quant.quantize_kv(inp.k, inp.v, bits=4, group=32, residual=992)
    check_quant_cache(ql, 0, inp.k, inp.v)
    out = ql.attn_decode(torch.from_numpy(inp.q)[None].cuda(), SM)
    assert attn_err(out[0], attention.quant_attention(inp.q, ref, SM)) <= TOL


def test_sixty_four_sequences():
    """The largest batch the ABI takes (64): more (sequence, head) problems than compute units."""
    rng = np.random.default_rng(64)
    lens = rng.integers(1, 1500, size=64).tolist()
    lens[3], lens[40] = 1500, 0
    print(f"case batch 64 lens={lens[:8]}...", flush=True)
    nmax = max(lens)
    inps = [make_layer(max(n, 1), config=4, layer=1, seq=100 + b) for b, n in enumerate(lens)]
    q = torch.from_numpy(np.stack([i.q for i in inps])).cuda()
    kb, vb = to_new_batch([i.k for i in inps], nmax), to_new_batch([i.v for i in inps], nmax)
    ql = tkv.QuantLayer(bits=2, capacity=1536, batch=64)
    ql.append(kb, vb, n_valid=lens)
    out = ql.attn_decode(q, SM)
    sl = tkv.SparseLayer(top_k=128, capacity=1536, batch=64)
    chs = [static_channels(i.k, 16) for i in inps]
    sl.set_channels(np.stack(chs))
    sl.append(kb, vb, n_valid=lens)
    sl.estimate_topk(q)
    out_s = sl.gather_attn(q, SM)
    torch.cuda.synchronize()
    for b, inp in enumerate(inps):
        n = lens[b]
        if n == 0:
            assert (out[b] == 0).all() and (out_s[b] == 0).all()
            assert int(sl.topk_count[b].sum()) == 0
            continue
        ref = check_quant_cache(ql, b, inp.k[:, :n], inp.v[:, :n])
        assert attn_err(out[b], attention.quant_attention(inp.q, ref, SM)) <= TOL
        idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k[:, :n], chs[b]), chs[b], n,
                                        top_k=128, n_sink=4, n_window=64)
        assert np.array_equal(sl.topk_count[b].cpu().numpy(), cnt)
        assert np.array_equal(sl.topk_idx[b].cpu().numpy(), idx)
        want = sparse.sparse_attention(inp.q, inp.k[:, :n], inp.v[:, :n], idx, cnt, n, SM, n_sink=4, n_window=64)
        assert attn_err(out_s[b], want) <= TOL


def test_dense_preference_full_size():
    """Offline identification at the full context: 64 query rows per head against 131072 keys."""
    from oracle import preference
    n, n_q, top_k = 131072, 64, 1024
    print(f"case full-size dense preference n={n}", flush=True)
    inp = make_layer(n, config=2, layer=3, seq=2)
    rng = np.random.default_rng(8)
    q_last = (inp.q[None].astype(np.float32) + 0.5 * rng.standard_normal((n_q, 32, 128))).astype(np.float16)
    dp = tkv.DensePreference(n_q=n_q, top_k=top_k, capacity=n)
    kd = torch.from_numpy(np.ascontiguousarray(inp.k.transpose(1, 0, 2)))[None].contiguous().cuda()
    out = dp.score(torch.from_numpy(q_last)[None].contiguous().cuda(), kd, SM)
    torch.cuda.synchronize()
    want = preference.dense_preference(q_last[:, :8], inp.k[:2], top_k, SM)     # two KV heads' worth of the oracle
    got = out[0, :8].cpu().numpy()
    print(f"   max |P - P_oracle| = {np.abs(got - want).max():.2e}", flush=True)
    assert np.abs(got - want).max() <= 1e-4 * n_q
