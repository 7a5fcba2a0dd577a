"""Child process of tests/test_gpu_handoffs.py: runs the hot path of both layer kinds on
seeded inputs and saves every output to the .npz file named on the command line.  The parent
starts it with and without serialized, blocking kernel launches (environment variables that
must be set before the process touches the GPU)."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np  # noqa: E402
import torch  # noqa: E402

import paper_2505_19586_amd as tkv  # noqa: E402
from synth import make_layer, static_channels  # noqa: E402

from gpu_util import to_new  # noqa: E402

SM = 1.0 / np.sqrt(128.0)
out = {}
for n in (4096, 40000):
    # quantized layer (toy configuration: 2 bit, groups of 32, 128-token fp16 tail)
    inp = make_layer(n, config=0, layer=0, seq=0)
    ql = tkv.QuantLayer(bits=2, capacity=n + 64)
    ql.append(to_new(inp.k), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    out[f"quant_{n}"] = ql.attn_decode(q, SM).cpu().numpy().view(np.uint16)
    new = make_layer(40, config=0, layer=0, seq=1)
    for i in range(40):   # decode steps across a group boundary
        ql.append(to_new(new.k[:, i:i + 1]), to_new(new.v[:, i:i + 1]))
    out[f"quant_after_steps_{n}"] = ql.attn_decode(q, SM).cpu().numpy().view(np.uint16)
    out[f"quant_codes_{n}"] = ql.view("k_codes").cpu().numpy()
    # sparse layer (k = 128 in the toy configuration, 1024 in the longer one)
    inp = make_layer(n, config=0, layer=1, seq=0)
    sl = tkv.SparseLayer(top_k=128 if n == 4096 else 1024, capacity=n + 64)
    sl.set_channels(static_channels(inp.k, 16)[None])
    sl.append(to_new(inp.k), to_new(inp.v))
    q = torch.from_numpy(inp.q)[None].cuda()
    sl.estimate_topk(q)
    out[f"topk_idx_{n}"] = sl.topk_idx.cpu().numpy()
    out[f"sparse_two_streams_{n}"] = sl.gather_attn(q, SM, gather_stream=torch.cuda.Stream()).cpu().numpy().view(np.uint16)
    out[f"sparse_one_stream_{n}"] = sl.gather_attn(q, SM).cpu().numpy().view(np.uint16)
    new = make_layer(3, config=0, layer=1, seq=1)
    out[f"sparse_decode_{n}"] = sl.decode(q, SM, to_new(new.k), to_new(new.v)).cpu().numpy().view(np.uint16)
    out[f"topk_idx_after_decode_{n}"] = sl.topk_idx.cpu().numpy()
torch.cuda.synchronize()
np.savez(sys.argv[1], **out)
