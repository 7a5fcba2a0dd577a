"""Prefill-side build of the caches in the overlapped order bench.py --prefill-offload times:
sparse layers' bulk appends (host rows, summaries, resident rows) on a side stream while the
other stream produces and quantizes the next layers.  Everything must come out bit for bit as
the oracle has it."""
import os
import sys

import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from oracle import sparse
from synth import make_layer, static_channels

from gpu_util import check_quant_cache

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("with_side_stream", [True, False])
def test_layer_by_layer_build_is_bit_exact(with_side_stream):
    n, kinds = 20000, ["q", "s", "s", "q", "s", "s"]
    print(f"case prefill build n={n} side={with_side_stream}", flush=True)
    inps = [make_layer(n, config=3, layer=l, seq=0) for l in range(len(kinds))]
    chans = [static_channels(i.k, 16) for i in inps]
    layers = []
    for l, kind in enumerate(kinds):
        if kind == "q":
            layers.append(tkv.QuantLayer(bits=2, capacity=n + 32))
        else:
            L = tkv.SparseLayer(top_k=128, capacity=n + 16)
            L.set_channels(chans[l][None])
            layers.append(L)
    pinned = [(torch.from_numpy(np.ascontiguousarray(i.k.transpose(1, 0, 2))[None]).pin_memory(),
               torch.from_numpy(np.ascontiguousarray(i.v.transpose(1, 0, 2))[None]).pin_memory()) for i in inps]

    def produce(l):
        # stands in for the prefill computation: the layer's K/V arrive on the current stream and
        # a little arithmetic runs on them before they are used
        k = pinned[l][0].to("cuda", non_blocking=True)
        v = pinned[l][1].to("cuda", non_blocking=True)
        return (k * 1).contiguous(), (v * 1).contiguous()

    side = torch.cuda.Stream() if with_side_stream else None
    bench.build_caches_overlapped(torch, layers, produce, side).synchronize()
    torch.cuda.synchronize()
    for l, (kind, L, inp) in enumerate(zip(kinds, layers, inps)):
        if kind == "q":
            check_quant_cache(L, 0, inp.k, inp.v)
            continue
        assert int(L.seq_len[0]) == n
        host = L.kv_host[0, :, :n].numpy()
        assert np.array_equal(host[:, :, 0].view(np.uint16), inp.k.view(np.uint16))
        assert np.array_equal(host[:, :, 1].view(np.uint16), inp.v.view(np.uint16))
        assert np.array_equal(L.key_summary[0, :, :n].cpu().numpy().view(np.uint16),
                              sparse.key_summary(inp.k, chans[l]).view(np.uint16))
        loc = L.kv_local[0].cpu().numpy()          # [Hkv][4 + 64][2][128]
        assert np.array_equal(loc[:, :4, 0].view(np.uint16), inp.k[:, :4].view(np.uint16))
        win = np.arange(n - 64, n)
        assert np.array_equal(loc[:, 4 + win % 64, 1].view(np.uint16), inp.v[:, win].view(np.uint16))
