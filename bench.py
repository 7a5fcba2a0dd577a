#!/usr/bin/env python3
"""Decode-attention benchmark of the hybrid KV cache on one MI355X.

Workload (default): the full 32-layer decode step at 128k context, batch 1, with
Llama-3.1-8B attention shapes: layers 0-1 quantization-friendly (2 bit, g = 32,
128-token fp16 tail), layers 2-31 sparsity-friendly (16 summary channels on the
GPU, Top-K 1024 + 4 sinks + 64-token window, full fp16 K/V in pinned host memory).
One step = every call of the hot path for every layer.  Metric: microseconds per
layer-token (step time / 32).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

N_LAYERS = 32
QUANT_LAYERS = (0, 1)
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--context", type=int, default=131072)
    ap.add_argument("--batch", type=int, default=1, help="sequences decoded together (configs[4]: 8)")
    ap.add_argument("--ragged", action="store_true",
                    help="sequence lengths uniform in [context/2, context] (configs[4]: --batch 8 --context 32768 --ragged)")
    ap.add_argument("--bits", type=int, default=2, help="code width of the quantized layers (1, 2, 4)")
    ap.add_argument("--group", type=int, default=32, help="quantization group (32, or the paper's 64)")
    ap.add_argument("--top-k", type=int, default=1024)
    ap.add_argument("--channels", type=int, default=16, help="critical channels d_s (8, 12, 16)")
    ap.add_argument("--n-sink", type=int, default=4)
    ap.add_argument("--n-window", type=int, default=64)
    ap.add_argument("--paper-setting", action="store_true",
                    help="the paper's long-context configuration (Sec. 5.1, App. D): 1 bit, groups of 64, "
                         "n_local 128, n_topk 896, 12 critical channels re-selected every step and fetched "
                         "from host memory")
    ap.add_argument("--host-layers", type=int, default=30,
                    help="distinct pinned host K/V caches (30 = one per sparse layer)")
    ap.add_argument("--dynamic-channels", choices=["off", "resident", "host"], default="off",
                    help="re-select the critical channels every step (Eq. 10): 'resident' scores in place over "
                         "channel-major keys kept on the GPU, 'host' fetches the critical key cache from a "
                         "pinned-host channel-major copy one layer ahead (the paper's design)")
    ap.add_argument("--no-warm-next", dest="warm_next", action="store_false",
                    help="chained schedule: tkv_sparse_decode without the hint that warms up the next layer's key summary")
    ap.add_argument("--identify", action="store_true",
                    help="instead of the decode step, time the offline identification of one layer (dense "
                         "preference score, Sec. 4.1) at --context with 64 query rows per head and k = --top-k")
    ap.add_argument("--per-call", choices=["quant", "sparse"], default=None,
                    help="instead of the decode step, time the entry points of ONE layer kind on their own over "
                         "many distinct caches (configs[1]: --per-call quant --context 32768 [--bits 4]; "
                         "configs[2]: --per-call sparse)")
    ap.add_argument("--prefill-offload", action="store_true",
                    help="instead of the decode step, time the prefill-side build of the 32 layers' caches at "
                         "--context: each sparse layer's K/V goes to pinned host memory on a side stream while the "
                         "compute stream produces (and, for quantized layers, quantizes) the next layers' K/V; "
                         "measured against a pinned device-to-host copy")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--schedule", choices=["chained", "overlapped"], default="chained",
                    help="chained (the headline): every call waits for the previous one, the only order a decoder "
                         "can run, since a layer's query depends on the layer before; overlapped: sparse-layer "
                         "gathers on side streams while the compute stream scores later layers (legal only because "
                         "the synthetic queries of different layers are independent; reported as other_schedule)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="chained schedule: tkv_sparse_append_estimate_topk + tkv_sparse_gather_attn per sparse layer "
                         "instead of the single tkv_sparse_decode launch")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the single-layer and batched configurations that the default run reports beside "
                         "the headline (the `configs` object of the JSON line)")
    ap.add_argument("--one-schedule", action="store_true", help="time only --schedule (profiling runs)")
    ap.add_argument("--lookahead", type=int, default=4,
                    help="overlapped schedule: sparse layers whose scoring runs ahead of the attention")
    ap.add_argument("--gather-streams", type=int, default=2,
                    help="overlapped schedule: side streams the gathers alternate between")
    ap.add_argument("--gather-cus", type=int, default=16,
                    help="overlapped schedule: compute units of the gather streams, split evenly (0 = no masks); the "
                         "compute stream gets what lies above the next multiple of 32 mask bits")
    return ap.parse_args()


def cu_masked_streams(n_gather_cus, n_streams=1, n_cus=256):
    """HIP streams with disjoint compute-unit masks, wrapped for torch: n_streams gather
    streams that split the first n_gather_cus mask bits evenly, and a compute stream on
    everything above the next multiple of 32 bits.  Mask bit i is a unit of shader engine
    i mod 32 (four engines per die), and a launch hands every engine the same share of its
    workgroups: only a mask that takes the same number of units from every engine (whole
    groups of 32 bits) leaves the compute stream a machine on which one-workgroup-per-unit
    launches still finish in one round; with 16 units taken from half of the engines every
    kernel of the compute stream ran about 1.5 times longer.  Returns ([gather streams],
    compute stream, destroy) or None if the runtime refuses."""
    import ctypes as C
    import torch
    per = n_gather_cus // max(n_streams, 1)
    reserved = -(-n_gather_cus // 32) * 32
    if n_streams < 1 or per < 8 or reserved >= n_cus:
        return None
    try:
        hip = C.CDLL("libamdhip64.so")
        fn = hip.hipExtStreamCreateWithCUMask
    except (OSError, AttributeError):
        return None
    fn.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_uint32)]
    fn.restype = C.c_int
    words = n_cus // 32
    gather_bits = [((1 << per) - 1) << (per * i) for i in range(n_streams)]
    compute_bits = ((1 << n_cus) - 1) ^ ((1 << reserved) - 1)
    out, handles = [], []
    for bits in gather_bits + [compute_bits]:
        mask = (C.c_uint32 * words)(*[(bits >> (32 * i)) & 0xFFFFFFFF for i in range(words)])
        h = C.c_void_p()
        if fn(C.byref(h), words, mask) != 0 or not h.value:
            hip.hipGetLastError()   # the refusal must not surface in a later launch check
            return None
        handles.append(h)
        out.append(torch.cuda.ExternalStream(h.value))

    def destroy():
        hip.hipStreamDestroy.argtypes = [C.c_void_p]
        for h in handles:
            hip.hipStreamDestroy(h)
    return out[:-1], out[-1], destroy


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(the path would shard by KV head, one host link per GPU)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2505_19586_amd as tkv
    from synth.device import make_layer_device, static_channels_device

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(tkv.library_path()):
        from paper_2505_19586_amd import build as b
        b.build_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.identify:
        print(json.dumps(identify(args, tkv, torch, dev)))
        return
    if args.prefill_offload:
        print(json.dumps(prefill_offload(args, tkv, torch, dev)))
        return
    if args.per_call:
        print(json.dumps(per_call(args, tkv, torch, dev)))
        return
    default_workload = (args.context == 131072 and args.batch == 1 and not args.ragged and not args.paper_setting
                        and args.dynamic_channels == "off" and (args.bits, args.group) == (2, 32))
    line = run_step(args, tkv, torch, dev)
    if default_workload and not args.no_configs:
        line["configs"] = other_configs(args, tkv, torch, dev)
    print(json.dumps(line))


def other_configs(args, tkv, torch, dev):
    """The benchmark's other workloads, measured in the same run (the headline stays the 32-layer
    step at 128k): single quantized layer at N = 32768 with 2 and 4 bit, single sparse layer at
    N = 131072, batched ragged decode (batch 8, lengths in [16384, 32768]).  Every call is timed
    with its data coming from HBM (round-robin over distinct caches)."""
    import copy
    import gc

    def fresh(**kw):
        a = copy.copy(args)
        for k, v in kw.items():
            setattr(a, k, v)
        return a

    def cleanup():
        gc.collect()
        torch.cuda.empty_cache()
        empty_host = getattr(torch._C, "_host_emptyCache", None)   # pinned blocks the finished configuration no longer needs
        if empty_host is not None:
            empty_host()

    out = {}
    cleanup()
    for bits in (2, 4):
        r = per_call(fresh(per_call="quant", context=32768, bits=bits, group=32), tkv, torch, dev)
        c = r["calls"]
        out["configs[1] quantized layer N=32768 %d bit" % bits] = {
            "quant_attn_us": r["value"], "algorithmic_bytes": r["roofline"]["algorithmic_bytes"],
            "GBs": r["roofline"]["achieved"], "frac_of_hbm_peak": r["roofline"]["frac"],
            "read_sweep_same_bytes_us": c["read_sweep_same_bytes_us"], "hot_in_cache_us": c["quant_attn_hot_in_cache_us"],
            "quantize_append_bulk_us": c["quantize_append_bulk_us"], "quantize_append_bulk_GBs": c["quantize_append_bulk_GBs"],
            "quantize_append_1_token_us": c["quantize_append_1_token_us"], "distinct_caches": c["distinct_caches"]}
        cleanup()
    r = per_call(fresh(per_call="sparse", context=131072), tkv, torch, dev)
    c = r["calls"]
    out["configs[2] sparse layer N=131072"] = {
        "estimate_topk_us": c["estimate_topk_us"], "estimate_topk_GBs": c["estimate_topk_GBs"],
        "estimate_topk_frac_of_hbm_peak": c["estimate_topk_frac_of_hbm"],
        "append_estimate_topk_us": c["append_estimate_topk_us"],
        "gather_alone_us": c["gather_alone_us"], "gather_GBs": r["roofline"]["achieved"],
        "gather_frac_of_h2d": r["roofline"]["frac"], "h2d_memcpy_GBs": c["h2d_memcpy_GBs"],
        "gather_attn_fused_us": c["gather_attn_fused_us"], "attention_over_staged_rows_us": c["attention_over_staged_rows_us"],
        "decode_fused_us": c.get("decode_fused_us"),
        "distinct_summaries": c["distinct_summaries"], "distinct_host_caches": c["distinct_host_caches"]}
    cleanup()
    b = run_step(fresh(batch=8, context=32768, ragged=True, steps=max(4, args.steps // 4), warmup=2,
                       no_cpu_baseline=True), tkv, torch, dev)
    out["configs[4] batched ragged decode, batch 8"] = {
        "workload": b["config"]["workload"], "schedule": b["config"]["schedule"], "ms_per_step": b["ms_per_step"],
        "us_per_layer_token": b["value"], "other_schedule": b["other_schedule"],
        "host_link": b["host_link"], "host_link_floor_ms": b["host_link_floor_ms"],
        "quant_attn_us": b["quant_attn_us"], "quant_attn_frac_of_hbm_peak": b["roofline"]["frac"],
        "quant_attn_bytes": b["roofline"]["algorithmic_bytes"], "estimate_topk_us": b["estimate_topk_us"],
        "gather_us": b["gather_us"], "distinct_host_caches": b["config"]["distinct_host_caches"]}
    cleanup()
    # off the decode path: which layers are quantization-friendly (Sec. 4.1), one layer of a 131072-token prompt
    i = identify(fresh(context=131072), tkv, torch, dev)
    out["offline identification, dense preference score of one layer at N=131072"] = {
        "workload": i["config"]["workload"], "ms_per_layer": i["value"], "TFLOPs": i["roofline"]["achieved"],
        "frac_of_fp16_mfma_peak": i["roofline"]["frac"], "workspace_MiB": i["workspace_MiB"]}
    cleanup()
    return out


def run_step(args, tkv, torch, dev):
    """The 32-layer decode step (configs[3]; with --batch / --ragged configs[4]); returns the JSON line."""
    import numpy as np

    from synth.device import make_layer_device, static_channels_device
    if args.paper_setting:
        args.bits, args.group, args.top_k, args.channels, args.n_sink, args.n_window = 1, 64, 896, 12, 0, 128
        if args.dynamic_channels == "off":
            args.dynamic_channels = "host"
    if args.dynamic_channels == "host":
        args.schedule = "chained"   # its own pipeline: the fetch of layer l+1 under layer l
    B = args.batch
    if B < 1 or B > 64:
        print("bench.py: --batch must be between 1 and 64", file=sys.stderr)
        sys.exit(2)
    if B > 1 and args.dynamic_channels != "off":
        print("bench.py: the dynamic-channel modes are timed at batch 1", file=sys.stderr)
        sys.exit(2)
    sparse_kw = dict(top_k=args.top_k, n_channels=args.channels, n_sink=args.n_sink, n_window=args.n_window, batch=B)
    N = args.context
    if args.ragged:
        from synth import ragged_lengths
        lens = [int(x) for x in ragged_lengths(B, N // 2, N)]
    else:
        lens = [N] * B
    tot = sum(lens)
    CAP = N + 64 * ((args.steps * 2 + args.warmup + 64 + 63) // 64)
    sm = 1.0 / np.sqrt(128.0)
    t_build = time.time()

    # ---- measured host-link ceiling: one pinned 1 GiB H2D copy
    pin = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
    dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    h2d = 0.0
    for _ in range(3):
        e0.record(); dst.copy_(pin, non_blocking=True); e1.record(); e1.synchronize()
        h2d = max(h2d, (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    # device-to-device copy of known size (1 GiB read + 1 GiB written): calibrates the
    # FETCH_SIZE / WRITE_SIZE counters when this script runs under rocprofv3 --pmc
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst.copy_(src)
    torch.cuda.synchronize()
    del pin, dst, src

    # ---- build the caches
    layers = []
    qs = []
    stage1 = {}
    host_pool = []
    sample = {}
    def make_batch(seed):
        """q [B][Hq][D], k and v [B][max len][Hkv][D] (rows past a sequence's length are not
        appended), channel lists [B][Hkv][d_s]"""
        qq, kk, vv, cc = [], [], [], []
        for b in range(B):
            q, k, v = make_layer_device(max(lens), seed=seed + 100000 * b, device=dev)
            qq.append(q); kk.append(k); vv.append(v)
            cc.append(static_channels_device(k[:lens[b]], args.channels))
        if B == 1:
            return qq[0][None].contiguous(), kk[0][None], vv[0][None], cc[0][None]
        return torch.stack(qq), torch.stack(kk), torch.stack(vv), torch.stack(cc)

    def host_sample(q, k, v):   # sequence 0 as the oracle takes it: [Hkv][n][D]
        return (q[0].cpu().numpy(), k[0, :lens[0]].permute(1, 0, 2).contiguous().cpu().numpy(),
                v[0, :lens[0]].permute(1, 0, 2).contiguous().cpu().numpy())

    for l in range(N_LAYERS):
        q, k, v, ch = make_batch(1000 + l)
        qs.append(q)
        if l in QUANT_LAYERS:
            L = tkv.QuantLayer(bits=args.bits, group_size=args.group, capacity=CAP, batch=B, device=dev)
            L.append(k, v, n_valid=lens)
            if l == 0:
                sample["quant"] = host_sample(q, k, v)
        else:
            si = l - len(QUANT_LAYERS)
            kv_host = None
            if si >= args.host_layers:
                kv_host = host_pool[si % args.host_layers]
            try:
                L = tkv.SparseLayer(capacity=CAP, device=dev, kv_host=kv_host, **sparse_kw)
            except RuntimeError:
                # no more pinned host memory: the remaining sparse layers share the host caches that
                # exist (only the selected rows of a cache are ever read); stated in the JSON line
                if kv_host is not None or not host_pool:
                    raise
                torch.cuda.synchronize()
                args.host_layers = len(host_pool)
                kv_host = host_pool[si % args.host_layers]
                L = tkv.SparseLayer(capacity=CAP, device=dev, kv_host=kv_host, **sparse_kw)
            if args.dynamic_channels != "off":   # Stage 1 buffers see the keys before the layer's own append
                shared = next(iter(stage1.values())).fetched if stage1 else None   # one double buffer for all layers
                stage1[l] = tkv.Stage1(L, resident=args.dynamic_channels == "resident", fetched=shared)
                stage1[l].append(k)
            if kv_host is None:
                host_pool.append(L.kv_host)
            L.set_channels(ch)
            if kv_host is None:
                L.append(k, v, n_valid=lens)
            else:  # aliased host cache: keep its rows, refresh only the GPU-side state
                tmp = tkv.SparseLayer(capacity=CAP, device=dev, **sparse_kw)
                tmp.set_channels(L.channel_idx)
                tmp.append(k, v, n_valid=lens)
                L.key_summary.copy_(tmp.key_summary); L.kv_local.copy_(tmp.kv_local); L.seq_len[:] = tmp.seq_len
                del tmp
            if l == len(QUANT_LAYERS):
                sample["sparse"] = host_sample(q, k, v) + (L.channel_idx[0].cpu().numpy(),)
        layers.append(L)
        del k, v
    torch.cuda.synchronize()
    t_build = time.time() - t_build

    outs = [torch.empty(B, 32, 128, dtype=torch.float16, device=dev) for _ in range(N_LAYERS)]
    g = torch.Generator(device=dev); g.manual_seed(7)
    new_k = [torch.randn(B, 1, 8, 128, generator=g, device=dev).half() for _ in range(N_LAYERS)]
    new_v = [torch.randn(B, 1, 8, 128, generator=g, device=dev).half() for _ in range(N_LAYERS)]
    def ev():
        return torch.cuda.Event(enable_timing=True)

    sparse_ids = [l for l in range(N_LAYERS) if l not in QUANT_LAYERS]

    def step_overlapped(compute, sides):
        """Software-pipelined enqueue.  The gathers alternate between the side streams, so the
        link already serves layer l+1's rows while layer l's gather drains and the next launch
        is set up (one stream alone leaves the link idle for ~10 us between two gathers); the
        compute stream runs append + scoring + selection `lookahead` sparse layers ahead of the
        attention, so that no gather ever waits for its indices.  Legal only because the
        synthetic queries of different layers are independent."""
        lookahead = args.lookahead
        done = {}      # layer -> event after which its staged rows are complete
        order = []     # sparse layers in flight, oldest first
        # the first sparse layers are scored before the quantized layers' attention, so that the
        # link is busy from the start of the step (gathers under quantized-layer compute)
        first = sparse_ids[:lookahead]
        sequence = first + [l for l in range(N_LAYERS) if l not in first]
        for l in sequence:
            L = layers[l]
            if l in QUANT_LAYERS:
                L.append(new_k[l], new_v[l])
                L.attn_decode(qs[l], sm, out=outs[l])
                continue
            if l in stage1:   # resident channel-major keys: Eq. 10 and the scoring in one call
                stage1[l].append_both(new_k[l], new_v[l])
                stage1[l].select_estimate_topk(qs[l], qs[l])
            else:
                L.append_estimate_topk(new_k[l], new_v[l], qs[l])
            side = sides[l % len(sides)]
            ready = torch.cuda.Event()
            ready.record(compute)
            side.wait_event(ready)
            L.gather(stream=side)
            done[l] = torch.cuda.Event()
            done[l].record(side)
            order.append(l)
            if len(order) > lookahead:
                pl = order.pop(0)
                compute.wait_event(done.pop(pl))
                layers[pl].attn(qs[pl], sm, out=outs[pl])
        for pl in order:
            compute.wait_event(done.pop(pl))
            layers[pl].attn(qs[pl], sm, out=outs[pl])

    fetch = {"stream": torch.cuda.Stream() if args.dynamic_channels == "host" else None}

    def step_dynamic():
        """Chained step with the critical channels re-selected per layer and step (Eq. 10).
        'resident': Stage 2 reads the listed rows of the GPU-resident channel-major keys.
        'host': Stage 1 of the next sparse layer (append, channel selection, fetch of its
        critical key cache into the other half of the double buffer) is enqueued one layer
        ahead, the fetch on its own stream (legal here because the synthetic queries of
        different layers are independent; a model would use the predicted query)."""
        compute = torch.cuda.current_stream()
        fetch_stream = fetch["stream"]
        fetched = {}

        def start_fetch(j):
            l = sparse_ids[j]
            stage1[l].append_both(new_k[l], new_v[l])
            stage1[l].select_channels(qs[l])
            a = torch.cuda.Event(); a.record(compute)
            fetch_stream.wait_event(a)
            stage1[l].prefetch(j % 2, stream=fetch_stream)
            b = torch.cuda.Event(); b.record(fetch_stream)
            fetched[l] = b

        if fetch_stream is not None:
            start_fetch(0)
        for l, L in enumerate(layers):
            if l in QUANT_LAYERS:
                L.append(new_k[l], new_v[l])
                L.attn_decode(qs[l], sm, out=outs[l])
                continue
            j = sparse_ids.index(l)
            if fetch_stream is None:
                stage1[l].append_both(new_k[l], new_v[l])
                stage1[l].select_estimate_topk(qs[l], qs[l])
            else:
                if j + 1 < len(sparse_ids):
                    start_fetch(j + 1)
                compute.wait_event(fetched[l])
                stage1[l].estimate_topk(qs[l], j % 2)
            L.gather_attn(qs[l], sm, out=outs[l])

    def step_chained(rec=None):
        """Every call of a layer waits for the previous one: what a real model allows."""
        if rec is None and args.dynamic_channels != "off":
            return step_dynamic()
        for l, L in enumerate(layers):
            if l in QUANT_LAYERS and rec is None and not args.separate_calls:
                # one call per quantized layer: the step's new token joins the cache (Eq. 2) in the
                # attention's launch (a launch of its own only when it completes a quantization group)
                L.decode(qs[l], sm, new_k[l], new_v[l], out=outs[l])
                continue
            if l in QUANT_LAYERS or rec is not None:
                L.append(new_k[l], new_v[l])      # Eq. 2: the step's new token joins the cache first
            if l in QUANT_LAYERS:
                if rec is not None:
                    a, b = ev(), ev(); a.record()
                L.attn_decode(qs[l], sm, out=outs[l])
                if rec is not None:
                    b.record(); rec["quant"].append((a, b))
            else:
                if rec is not None:
                    a, b = ev(), ev(); a.record()
                    L.estimate_topk(qs[l])
                    b.record(); rec["topk"].append((a, b))
                elif not args.separate_calls:
                    # one launch per sparse layer: append, scoring, Top-K, fetch of the rows, attention
                    # (the next sparse layer's key summary is read once meanwhile: it does not depend
                    # on that layer's query, and HBM is idle while this layer waits for the host link)
                    nxt = layers[l + 1] if args.warm_next and l + 1 < len(layers) else None
                    L.decode(qs[l], sm, new_k[l], new_v[l], out=outs[l],
                             warm_next=nxt if isinstance(nxt, tkv.SparseLayer) else None)
                    continue
                else:                 # the scoring launch also appends the step's new token
                    L.append_estimate_topk(new_k[l], new_v[l], qs[l])
                if rec is not None:   # per-call timing pass: the transfer on its own
                    g0, g1 = ev(), ev(); g0.record()
                    L.gather()
                    g1.record(); rec["gather"].append((g0, g1))
                    L.attn(qs[l], sm, out=outs[l])
                else:                 # one stream: the attention kernel fetches the rows itself
                    L.gather_attn(qs[l], sm, out=outs[l])

    def timed(schedule):
        """W untimed warm-up steps, then exactly K timed steps; returns ms per step (None if
        the schedule cannot be set up)."""
        import contextlib
        destroy = None
        if schedule == "chained":
            ctx, step = contextlib.nullcontext(), step_chained
            if args.dynamic_channels == "host":
                # the fetch of the critical key cache gets compute units of its own, like the gather
                masked = cu_masked_streams(args.gather_cus, 1)
                if masked is not None:
                    sides, compute, destroy = masked
                    fetch["stream"] = sides[0]
                    ctx = torch.cuda.stream(compute)
        else:
            # A kernel that shares compute units with the gather is slowed to the pace of the
            # host link (its memory instructions queue behind the gather's): the gather gets
            # compute units of its own and everything else the rest.
            masked = cu_masked_streams(args.gather_cus, args.gather_streams)
            if masked is None and args.gather_cus > 0:
                return None   # no streams with compute-unit masks here: plain overlap is slower than chaining
            if masked is None:
                sides, compute = [torch.cuda.Stream() for _ in range(args.gather_streams)], torch.cuda.current_stream()
                ctx = contextlib.nullcontext()
            else:
                sides, compute, destroy = masked
                ctx = torch.cuda.stream(compute)
            step = lambda: step_overlapped(compute, sides)
        with ctx:
            for _ in range(args.warmup):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) / args.steps * 1e3
        if destroy is not None:
            destroy()
        return ms

    ms_per_step = timed(args.schedule)
    if ms_per_step is None:   # the overlapped schedule could not be set up
        args.schedule = "chained"
        ms_per_step = timed("chained")
    other = "overlapped" if args.schedule == "chained" else "chained"
    ms_other = None if args.one_schedule or args.dynamic_channels == "host" else timed(other)

    # per-kernel durations with events on the launching stream (separate passes so the
    # events do not perturb the step time above)
    rec = {"quant": [], "topk": [], "gather": []}
    for _ in range(max(25, args.steps // 2)):   # >= 50 samples of every call
        step_chained(rec)
    torch.cuda.synchronize()
    samples = {k: np.array([a.elapsed_time(b) for a, b in v]) * 1e3 for k, v in rec.items() if v}  # us
    dur = {k: float(v.mean()) for k, v in samples.items()}
    spread = {k: {"n": int(v.size), "p10": float(np.percentile(v, 10)), "p50": float(np.percentile(v, 50)),
                  "p90": float(np.percentile(v, 90))} for k, v in samples.items()}

    # The dominant kernel on its own: launches back to back between ONE pair of events (an event
    # pair around a single launch adds 3-4 us of its own), over four distinct caches (> 256 MB
    # in total, so every sweep comes from HBM as it does inside the step).
    pool = [layers[l] for l in QUANT_LAYERS]
    for x in range(max(0, 4 - len(pool))):
        _, k, v, _ = make_batch(5000 + x)
        L = tkv.QuantLayer(bits=args.bits, group_size=args.group, capacity=CAP, batch=B, device=dev)
        L.append(k, v, n_valid=lens)
        pool.append(L)
        del k, v
    for L in pool:
        L.attn_decode(qs[0], sm, out=outs[0])
    e0, e1 = ev(), ev()
    rounds = 13   # 52 launches
    e0.record()
    for _ in range(rounds):
        for L in pool:
            L.attn_decode(qs[0], sm, out=outs[0])
    e1.record()
    torch.cuda.synchronize()
    dur["quant_in_step"] = dur["quant"]
    dur["quant"] = e0.elapsed_time(e1) * 1e3 / (rounds * len(pool))
    del pool
    dur["read_sweep"] = read_sweep_us(tkv, torch, dev, quant_bytes_of(args, lens), rounds)
    # the gather alone, the same way: every sparse layer's rows (distinct host caches), twice
    g0, g1 = ev(), ev()
    g0.record()
    for _ in range(2):
        for l in sparse_ids:
            layers[l].gather()
    g1.record()
    torch.cuda.synchronize()
    dur["gather_in_step"] = dur["gather"]
    dur["gather"] = g0.elapsed_time(g1) * 1e3 / (2 * len(sparse_ids))
    # scoring + Top-K alone, the same way: every sparse layer's summary (distinct, so each sweep comes
    # from HBM), twice
    for l in sparse_ids[:4]:
        layers[l].estimate_topk(qs[l])
    t0, t1 = ev(), ev()
    t0.record()
    for _ in range(2):
        for l in sparse_ids:
            layers[l].estimate_topk(qs[l])
    t1.record()
    torch.cuda.synchronize()
    dur["topk_in_step"] = dur["topk"]
    dur["topk"] = t0.elapsed_time(t1) * 1e3 / (2 * len(sparse_ids))

    quant_bytes = quant_bytes_of(args, lens)
    summary_bytes = 8 * tot * args.channels * 2
    gather_bytes = B * 8 * args.top_k * 512
    roof = {"bound": "hbm", "kernel": "tkv_quant_attn_decode", "achieved": quant_bytes / dur["quant"] / 1e3,
            "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "traffic": traffic_from_profile("quant_attn_mfma_kernel<2") if (N, B, args.bits, args.group) == (131072, 1, 2, 32) else None,
            "traffic_source": "profiles/bench_hybrid_step_128k_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                              "earlier run of this command, not measured in this run)",
            "algorithmic_bytes": quant_bytes,
            # a kernel that only streams the same number of bytes (tkv_debug_read_sweep), timed the same way
            "read_sweep_us": dur["read_sweep"], "read_sweep_GBs": quant_bytes / dur["read_sweep"] / 1e3,
            "time_vs_read_sweep": dur["quant"] / dur["read_sweep"]}
    roof["frac"] = roof["achieved"] / roof["peak"]
    extra = {
        "quant_attn_us": dur["quant"], "quant_attn_in_step_us": dur["quant_in_step"], "estimate_topk_us": dur["topk"], "estimate_topk_in_step_us": dur["topk_in_step"], "gather_us": dur["gather"], "gather_in_step_us": dur["gather_in_step"],
        "estimate_topk_GBs": summary_bytes / dur["topk"] / 1e3,
        "per_call_us": {"quant_attn": spread["quant"], "estimate_topk": spread["topk"], "gather": spread["gather"]},
        "other_schedule": None if ms_other is None else {
            "schedule": other, "ms_per_step": ms_other, "us_per_layer_token": ms_other * 1e3 / N_LAYERS / B,
            "note": "scoring runs %d sparse layers ahead of the attention: possible only because the synthetic "
                    "queries of different layers are independent, not a schedule a decoder can run" % args.lookahead
                    if other == "overlapped" else "every call waits for the previous one"},
        "host_link_floor_ms": len(sparse_ids) * gather_bytes / h2d / 1e6,
        "host_link": {"bound": "host_link", "kernel": "tkv_sparse_gather", "achieved": gather_bytes / dur["gather"] / 1e3,
                      "peak": h2d, "unit": "GB/s", "frac": gather_bytes / dur["gather"] / 1e3 / h2d,
                      "peak_source": "pinned 1 GiB hipMemcpy H2D measured in this run"},
    }

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(sample, lens[0], tot, args, sm)

    if B == 1:
        metric = "decode attention us per layer-token at %dk ctx" % (N // 1024)
        shape = f"configs[3]: 32-layer hybrid decode step, batch 1, N={N}"
    else:   # one step decodes one token of every sequence: B layer-tokens per layer
        metric = "decode attention us per layer-token, batch %d" % B
        shape = (f"configs[4]: 32-layer hybrid decode step, batch {B}, lengths "
                 + (f"uniform in [{N // 2}, {N}] ({tot} tokens in all)" if args.ragged else f"{N} each"))
    line = {
        "metric": metric, "value": ms_per_step * 1e3 / N_LAYERS / B,
        "unit": "us/layer-token", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{shape}, layers 0-1 {args.bits}-bit "
                               f"quantized (g={args.group}, W=128), layers 2-31 sparse (d_s={args.channels}, k={args.top_k}, "
                               f"{args.n_sink} sinks, {args.n_window} window)" + ("" if args.dynamic_channels == "off" else
                                               f", critical channels re-selected every step ({args.dynamic_channels})"),
                   "schedule": args.schedule,
                   **({"sparse_layer_calls": "tkv_sparse_append_estimate_topk + tkv_sparse_gather_attn" if args.separate_calls
                       else "tkv_sparse_decode (one launch)",
                       "quant_layer_calls": "tkv_quantize_append + tkv_quant_attn_decode" if args.separate_calls
                       else "tkv_quant_decode (one launch unless the token completes a group)"}
                      if args.schedule == "chained" and args.dynamic_channels == "off" else {}),
                   **({"gather_compute_units": args.gather_cus, "gather_streams": args.gather_streams}
                      if args.schedule == "overlapped" else {}),
                   "distinct_host_caches": len(host_pool),
                   "host_caches_note": None if len(host_pool) == len(sparse_ids) else
                   "pinned-memory fallback: %d sparse layers share %d pinned host caches" % (len(sparse_ids), len(host_pool)),
                   "build_s": round(t_build, 1)},
        "roofline": roof, "cpu_baseline": cpu, **extra,
    }
    del layers, stage1, host_pool, outs, qs
    return line


def identify(args, tkv, torch, dev):
    """Offline identification of one layer (not the headline): dense preference score of
    synthetic Gaussian queries and keys, timed over a few calls."""
    n, n_q = args.context, 64
    g = torch.Generator(device=dev)
    g.manual_seed(11)
    q_last = torch.randn(1, n_q, 32, 128, generator=g, device=dev).half()
    keys = torch.randn(1, n, 8, 128, generator=g, device=dev).half()
    dp = tkv.DensePreference(n_q=n_q, top_k=args.top_k, capacity=n, device=dev)
    sm = 128 ** -0.5
    for _ in range(max(1, args.warmup)):
        out = dp.score(q_last, keys, sm)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(3, args.steps // 4)
    e0.record()
    for _ in range(reps):
        out = dp.score(q_last, keys, sm)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    friendly, score = dp.classify(out[0], 0.2)
    flops = 2.0 * 32 * n_q * n * 128
    return {
        "metric": "offline identification ms per layer", "value": ms, "unit": "ms/layer", "n_gpus": 1,
        "higher_is_better": False, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"dense preference score, 32 query / 8 KV heads, n={n}, n_q={n_q}, k={args.top_k}"},
        "roofline": {"bound": "mfma", "achieved": flops / ms / 1e9, "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": flops / ms / 1e9 / 2500.0, "traffic": None},
        "layer_score": score, "quantization_friendly": friendly, "workspace_MiB": dp.workspace_bytes / 2 ** 20}


def build_caches_overlapped(torch, layers, produce, side):
    """Prefill-side build of the layers' caches, layer by layer (Sec. 4.2: the KV cache of a
    sparsity-friendly layer is offloaded to CPU memory layer by layer during prefill; Sec. 4.3:
    quantization-friendly layers are quantized on the spot).  produce(l) enqueues, on the current
    stream, whatever makes layer l's keys and values (here: synthetic generation, standing in for
    the prefill computation) and returns (k, v).  A quantized layer is quantized on the current
    stream; a sparse layer's bulk append - host rows, key summary, resident rows - runs on the
    `side` stream after the event that marks its inputs ready, so the device-to-host transfer of
    layer l overlaps the production of layers l+1, l+2, ...  side=None: everything on the current
    stream, one call after the other.  Returns the event after which every cache is complete."""
    import paper_2505_19586_amd as tkv
    compute = torch.cuda.current_stream()
    for l, L in enumerate(layers):
        k, v = produce(l)
        if isinstance(L, tkv.QuantLayer) or side is None:
            L.append(k, v)
            continue
        ready = torch.cuda.Event()
        ready.record(compute)
        side.wait_event(ready)
        L.append(k, v, stream=side.cuda_stream)
        k.record_stream(side)      # the inputs stay allocated until the side stream is through with them
        v.record_stream(side)
    done = torch.cuda.Event()
    if side is not None:
        done.record(side)
        compute.wait_event(done)
    done = torch.cuda.Event()
    done.record(compute)
    return done


def prefill_offload(args, tkv, torch, dev):
    """Times build_caches_overlapped for the 32-layer hybrid layout at --context (not the headline)."""
    from synth.device import make_layer_device, static_channels_device
    N = args.context
    # measured device-to-host ceiling: one pinned 1 GiB copy
    pin = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    d2h = 0.0
    for _ in range(3):
        e0.record(); pin.copy_(src, non_blocking=True); e1.record(); e1.synchronize()
        d2h = max(d2h, (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del pin, src
    kw = dict(top_k=args.top_k, n_channels=args.channels, n_sink=args.n_sink, n_window=args.n_window)
    host_pool = []

    def make_layers():
        layers = []
        for l in range(N_LAYERS):
            if l in QUANT_LAYERS:
                layers.append(tkv.QuantLayer(bits=args.bits, group_size=args.group, capacity=N, device=dev))
            else:
                si = l - len(QUANT_LAYERS)
                L = tkv.SparseLayer(capacity=N, device=dev, kv_host=host_pool[si] if si < len(host_pool) else None, **kw)
                if si >= len(host_pool):
                    host_pool.append(L.kv_host)
                layers.append(L)
        return layers

    chans = {}

    def produce_for(layers):
        def produce(l):
            _, k, v = make_layer_device(N, seed=3000 + l, device=dev)
            if isinstance(layers[l], tkv.SparseLayer):
                if l not in chans:
                    chans[l] = static_channels_device(k, args.channels)[None]
                layers[l].set_channels(chans[l])
            return k[None], v[None]
        return produce

    def run(side):
        layers = make_layers()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        build_caches_overlapped(torch, layers, produce_for(layers), side).synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        del layers
        return ms

    # A kernel that shares compute units with the offload is slowed to the pace of the host link
    # (its memory instructions queue behind the offload's stores to host memory), so the offload
    # stream gets a few compute units of its own and the compute stream the rest, as in the
    # overlapped decode schedule.
    import contextlib
    masked = cu_masked_streams(args.gather_cus, 1)
    if masked is not None:
        (side,), compute, destroy = masked
        ctx = torch.cuda.stream(compute)
    else:
        side, destroy, ctx = torch.cuda.Stream(), None, contextlib.nullcontext()
    with ctx:
        run(side)                           # warm-up: allocations, first launches, channel lists
        overlapped = min(run(side) for _ in range(2))
        serial = min(run(None) for _ in range(2))
    torch.cuda.synchronize()
    if destroy is not None:
        destroy()
    # what the compute stream does on its own (generation + quantization), without any offload
    layers = make_layers()
    produce = produce_for(layers)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for l in range(N_LAYERS):
        k, v = produce(l)
        if l in QUANT_LAYERS:
            layers[l].append(k, v)
    torch.cuda.synchronize()
    produce_ms = (time.perf_counter() - t0) * 1e3
    del layers
    n_sparse = N_LAYERS - len(QUANT_LAYERS)
    offload_bytes = n_sparse * 8 * N * 512
    return {"metric": "prefill-side cache build ms per 32-layer prompt", "value": overlapped, "unit": "ms", "n_gpus": 1,
            "higher_is_better": False, "dtype": "f16", "data": "synthetic",
            "config": {"workload": f"32-layer hybrid layout at N={N}: layers 0-1 quantized in bulk ({args.bits} bit, "
                                   f"g={args.group}), layers 2-31 offloaded to pinned host memory in bulk (512 B per "
                                   "token-head) with their key summaries and resident rows",
                       "schedule": "offload of layer l on a side stream under the production of layers l+1, ...",
                       "offload_compute_units": args.gather_cus if masked is not None else "no mask (shared with the compute stream)"},
            "roofline": {"bound": "host_link", "kernel": "tkv_sparse_append (bulk)", "achieved": offload_bytes / overlapped / 1e6,
                         "peak": d2h, "unit": "GB/s", "frac": offload_bytes / overlapped / 1e6 / d2h, "traffic": None,
                         "peak_source": "pinned 1 GiB hipMemcpy D2H measured in this run"},
            "serial_ms": serial, "production_and_quantization_alone_ms": produce_ms,
            "offload_bytes": offload_bytes, "link_floor_ms": offload_bytes / d2h / 1e6}


def quant_bytes_of(args, lens):
    """Algorithmic bytes of one tkv_quant_attn_decode call (Sec. 4.4, Table 2: b/8 bytes per
    code, one fp16 scaler and zero-point per group, for K and V; fp16 rows for the tail;
    query in, output out)."""
    nq = sum((n - 128) // args.group * args.group for n in lens)
    per_tok_head = 2 * 128 * args.bits // 8 + 2 * 2 * 2 * 128 // args.group
    return 8 * nq * per_tok_head + 8 * (sum(lens) - nq) * 512 + len(lens) * 2 * 32 * 128 * 2


def read_sweep_us(tkv, torch, dev, n_bytes, rounds):
    """Microseconds per launch of a kernel that only reads n_bytes, back to back between one
    pair of events, round-robin over four distinct buffers (every sweep from HBM)."""
    n16 = (n_bytes + 15) // 16 * 16
    bufs = [torch.empty(n16, dtype=torch.uint8, device=dev).fill_(x + 1) for x in range(4)]
    best = None
    for wgs in (256, 4096, 8192):     # the fastest of a few grid sizes is the reference
        for b in bufs:
            tkv.debug_read_sweep(b, wgs)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(rounds):
            for b in bufs:
                tkv.debug_read_sweep(b, wgs)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (rounds * len(bufs))
        best = us if best is None else min(best, us)
    return best


def per_call(args, tkv, torch, dev):
    """The entry points of one layer kind on their own (not the headline).  Launches go back
    to back between one pair of events, round-robin over enough distinct caches that every
    sweep comes from HBM (more than three times the 256 MB Infinity Cache where the layer's
    GPU-resident data is what is read); 'hot' repeats one cache instead."""
    from synth.device import make_layer_device, static_channels_device
    N, sm = args.context, 128 ** -0.5
    reps = max(3, args.steps // 4)

    def timed(fn, n_calls):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * n_calls)

    out = torch.empty(1, 32, 128, dtype=torch.float16, device=dev)
    g = torch.Generator(device=dev); g.manual_seed(7)
    k1 = torch.randn(1, 1, 8, 128, generator=g, device=dev).half()
    v1 = torch.randn(1, 1, 8, 128, generator=g, device=dev).half()
    calls = {}
    if args.per_call == "quant":
        nq = (N - 128) // args.group * args.group
        per_tok_head = 2 * 128 * args.bits // 8 + 2 * 2 * 2 * 128 // args.group
        qbytes = 8 * nq * per_tok_head + 8 * (N - nq) * 512 + 2 * 32 * 128 * 2
        n_caches = max(4, -(-3 * 256 * 2 ** 20 // qbytes))      # > 3 x 256 MB in all
        layers, qs, t_bulk = [], [], []
        for l in range(n_caches):
            q, k, v = make_layer_device(N, seed=1000 + l, device=dev)
            L = tkv.QuantLayer(bits=args.bits, group_size=args.group, capacity=N + 128, device=dev)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); L.append(k[None], v[None]); e1.record(); e1.synchronize()
            t_bulk.append(e0.elapsed_time(e1) * 1e3)
            layers.append(L); qs.append(q[None].contiguous())
            del k, v
        calls["quantize_append_bulk_us"] = float(sorted(t_bulk)[len(t_bulk) // 2])   # median; the first call pays for set-up
        calls["quantize_append_bulk_GBs"] = (8 * N * 512 + qbytes) / calls["quantize_append_bulk_us"] / 1e3
        cold = timed(lambda: [L.attn_decode(q, sm, out=out) for L, q in zip(layers, qs)], n_caches)
        hot = timed(lambda: [layers[0].attn_decode(qs[0], sm, out=out) for _ in range(n_caches)], n_caches)
        # 64 single-token appends on one cache: two of them complete a group and quantize it
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        layers[1].append(k1, v1); torch.cuda.synchronize()
        e0.record()
        for _ in range(64):
            layers[1].append(k1, v1)
        e1.record(); torch.cuda.synchronize()
        calls["quantize_append_1_token_us"] = e0.elapsed_time(e1) * 1e3 / 64
        calls["quant_attn_hot_in_cache_us"] = hot
        calls["read_sweep_same_bytes_us"] = read_sweep_us(tkv, torch, dev, qbytes, 13)
        calls["distinct_caches"] = n_caches
        value, roof = cold, {"bound": "hbm", "kernel": "tkv_quant_attn_decode", "achieved": qbytes / cold / 1e3,
                             "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": qbytes / cold / 1e3 / HBM_PEAK_GBS,
                             "traffic": None, "algorithmic_bytes": qbytes}
        workload = (f"configs[1]: single quantized layer, batch 1, N={N}, {args.bits} bit, g={args.group}, W=128; "
                    f"{n_caches} distinct caches round-robin")
        metric = "tkv_quant_attn_decode us per call"
    else:
        pin = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
        dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        h2d = 0.0
        for _ in range(3):
            e0.record(); dst.copy_(pin, non_blocking=True); e1.record(); e1.synchronize()
            h2d = max(h2d, (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        del pin, dst
        sbytes = 8 * N * args.channels * 2
        n_caches = max(8, -(-3 * 256 * 2 ** 20 // sbytes))
        kw = dict(top_k=args.top_k, n_channels=args.channels, n_sink=args.n_sink, n_window=args.n_window)
        layers, qs, spare_host = [], [], None
        for l in range(n_caches):
            q, k, v = make_layer_device(N, seed=2000 + l, device=dev)
            # eight distinct host K/V caches (4 GiB: only the selected rows are read), then aliased;
            # the GPU-resident summaries are all distinct
            L = tkv.SparseLayer(capacity=N + 128, device=dev, kv_host=layers[l % 8].kv_host if l >= 8 else None, **kw)
            L.set_channels(static_channels_device(k, args.channels)[None])
            if l < 8:
                L.append(k[None], v[None])
            else:   # build the GPU-side state through a throw-away layer whose host rows are not kept
                tmp = tkv.SparseLayer(capacity=N + 128, device=dev, kv_host=spare_host, **kw)
                spare_host = tmp.kv_host
                tmp.set_channels(L.channel_idx)
                tmp.append(k[None], v[None])
                L.key_summary.copy_(tmp.key_summary); L.kv_local.copy_(layers[l % 8].kv_local); L.seq_len[:] = tmp.seq_len
                del tmp
            layers.append(L); qs.append(q[None].contiguous())
            del k, v
        torch.cuda.synchronize()
        pairs = list(zip(layers, qs))
        t_topk = timed(lambda: [L.estimate_topk(q) for L, q in pairs], n_caches)
        t_fused = timed(lambda: [L.gather_attn(q, sm, out=out) for L, q in pairs], n_caches)
        t_gather = timed(lambda: [L.gather() for L, _ in pairs], n_caches)
        t_attn = timed(lambda: [L.attn(q, sm, out=out) for L, q in pairs], n_caches)
        t_app = timed(lambda: [L.append_estimate_topk(k1, v1, q) for L, q in pairs[:8]], 8)
        t_dec = timed(lambda: [L.decode(q, sm, k1, v1, out=out) for L, q in pairs[:8]], 8)
        gbytes = 8 * args.top_k * 512
        calls = {"estimate_topk_us": t_topk, "estimate_topk_GBs": sbytes / t_topk / 1e3,
                 "estimate_topk_frac_of_hbm": sbytes / t_topk / 1e3 / HBM_PEAK_GBS,
                 "gather_attn_fused_us": t_fused, "gather_alone_us": t_gather, "attention_over_staged_rows_us": t_attn,
                 "append_estimate_topk_us": t_app, "decode_fused_us": t_dec, "distinct_summaries": n_caches, "distinct_host_caches": 8,
                 "h2d_memcpy_GBs": h2d}
        value, roof = t_gather, {"bound": "host_link", "kernel": "tkv_sparse_gather", "achieved": gbytes / t_gather / 1e3,
                                 "peak": h2d, "unit": "GB/s", "frac": gbytes / t_gather / 1e3 / h2d, "traffic": None,
                                 "peak_source": "pinned 1 GiB hipMemcpy H2D measured in this run"}
        workload = (f"configs[2]: single sparse layer, batch 1, N={N}, d_s={args.channels}, k={args.top_k}, "
                    f"{args.n_sink} sinks, {args.n_window} window; {n_caches} distinct summaries, 8 distinct host caches")
        metric = "sparse gather us per call"
    return {"metric": metric, "value": value, "unit": "us/call", "n_gpus": 1, "higher_is_better": False,
            "dtype": "f16", "data": "synthetic", "config": {"workload": workload}, "roofline": roof, "calls": calls}


def traffic_from_profile(kernel: str):
    """HBM bytes per launch of `kernel` as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (summary committed under profiles/, already scaled by the copy-kernel calibration)."""
    path = os.path.join(ROOT, "profiles", "bench_hybrid_step_128k_hbm_traffic.md")
    try:
        for line in open(path):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 5 and cells[1].startswith(kernel):
                return float(cells[3]) * 1e6 + float(cells[4]) * 1024.0
    except (OSError, ValueError):
        pass
    return None


def cpu_baseline(sample, N, tot, args, sm):
    """The oracle as it stands on the host cores, on a bounded sample: one whole
    quantized layer and one whole sparse layer of one sequence (N tokens), a few repetitions
    each, weighted 2 : 30 over the 32 layers.  A batch is priced by its token count `tot`
    (the oracle's work is proportional to it) and reported per layer-token like `value`."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import attention, quant, sparse

    q, k, v = sample["quant"]
    t0 = time.perf_counter()
    c = quant.quantize_kv(k, v, bits=args.bits, group=args.group, residual=128)
    t_quantize = time.perf_counter() - t0
    reps = 6
    t0 = time.perf_counter()
    for _ in range(reps):
        attention.quant_attention(q, c, sm)
    t_quant = (time.perf_counter() - t0) / reps
    q, k, v, ch = sample["sparse"]
    summ = sparse.key_summary(k, ch)
    t0 = time.perf_counter()
    for _ in range(reps):
        idx, cnt = sparse.estimate_topk(q, summ, ch, N, top_k=args.top_k, n_sink=args.n_sink, n_window=args.n_window)
        sparse.sparse_attention(q, k, v, idx, cnt, N, sm, n_sink=args.n_sink, n_window=args.n_window)
    t_sparse = (time.perf_counter() - t0) / reps
    per_layer_token_us = (2 * t_quant + 30 * t_sparse) / 32 * 1e6 * (tot / N) / args.batch
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    cpu_model = ""
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                cpu_model = ln.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"value": per_layer_token_us, "unit": "us/layer-token", "cores": threads, "kind": "oracle",
            "cpu_model": cpu_model, "host_cpus": os.cpu_count(),
            "sample": ("" if args.batch == 1 else "sequence 0 of the batch, scaled by the batch's token count: ") +
                      "one whole quantized layer and one whole sparse layer (8 KV heads, 32 query heads) at N=%d, "
                      "%d repetitions each, weighted 2:30 over the 32 layers; quant attention %.2fs, sparse "
                      "estimate+topk+attention %.2fs per layer-token (quantizing the layer once: %.1fs, "
                      "not counted)" % (N, reps, t_quant, t_sparse, t_quantize)}


if __name__ == "__main__":
    main()
