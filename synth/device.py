"""Device-side draw of the same workload recipe as synth.workloads, for sizes where
numpy on the host would take minutes (30 layers x 512 MiB at 128k context).

Same structure - N(0,1) fp16 q/k/v, 4 key outlier channels x10 per KV head, 8
dominant tokens per KV head with key 0.8*q_dir + 0.2*noise - drawn with torch's
seeded generator on the GPU.  The values differ from the numpy recipe (different
generator); parity checks at these sizes copy the tensors back to the host and hand
those to the oracle.  No arithmetic of the method lives here.
"""
from __future__ import annotations

import math

import torch


def make_layer_device(n_tokens: int, *, n_q_heads=32, n_kv_heads=8, head_dim=128, seed=0,
                      n_outlier=4, outlier_gain=10.0, n_dominant=8, dominance_gain=1.0,
                      n_sink=4, n_window=64, device="cuda:0"):
    """Returns q [Hq, D], k [N, Hkv, D], v [N, Hkv, D] fp16 on the device (token-major,
    the layout the append entry points take)."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    grp = n_q_heads // n_kv_heads
    q = torch.randn(n_q_heads, head_dim, generator=g, device=device, dtype=torch.float32)
    k = torch.randn(n_tokens, n_kv_heads, head_dim, generator=g, device=device, dtype=torch.float32)
    v = torch.randn(n_tokens, n_kv_heads, head_dim, generator=g, device=device, dtype=torch.float32)
    for h in range(n_kv_heads):
        ch = torch.randperm(head_dim, generator=g, device=device)[:n_outlier]
        k[:, h, ch] *= outlier_gain
    lo, hi = n_sink, n_tokens - n_window
    if hi - lo >= n_dominant:
        for h in range(n_kv_heads):
            pos = torch.randperm(hi - lo, generator=g, device=device)[:n_dominant] + lo
            m = q[h * grp:(h + 1) * grp].mean(dim=0)
            q_dir = math.sqrt(head_dim) * m / m.norm() * dominance_gain
            noise = torch.randn(n_dominant, head_dim, generator=g, device=device)
            k[pos, h] = 0.8 * q_dir[None, :] + 0.2 * noise
    return q.half(), k.half(), v.half()


def static_channels_device(k: torch.Tensor, n_channels: int) -> torch.Tensor:
    """Per KV head the n_channels channels with the largest mean |k| (ascending)."""
    mean_abs = k.float().abs().mean(dim=0)          # [Hkv, D]
    idx = torch.topk(mean_abs, n_channels, dim=1).indices
    return torch.sort(idx, dim=1).values.to(torch.int32)
