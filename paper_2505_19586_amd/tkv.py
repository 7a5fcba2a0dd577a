"""ctypes binding of libtkv.so: same entry points as include/tkv.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels; there
is no CPU or PyTorch fallback - a missing library or GPU raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

TKV_MAX_BATCH = 64


class TkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().tkv_strerror(status).decode() if _LIB is not None else "?"
        super().__init__(f"{where}: {msg} ({status})")


def library_path() -> str:
    return os.path.join(_HERE, "libtkv.so")


class QuantDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("bits", C.c_int32), ("group_size", C.c_int32),
                ("residual", C.c_int32), ("capacity", C.c_int32), ("batch", C.c_int32)]


class QuantCache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero",
                                          "k_resid", "v_resid")] + [("seq_len_host", C.POINTER(C.c_int32))]


class SparseDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("n_channels", C.c_int32), ("top_k", C.c_int32),
                ("n_sink", C.c_int32), ("n_window", C.c_int32), ("capacity", C.c_int32), ("batch", C.c_int32)]


class SparseCache(C.Structure):
    _fields_ = [("key_summary", C.c_void_p), ("channel_idx", C.c_void_p), ("kv_host", C.c_void_p),
                ("kv_local", C.c_void_p), ("seq_len_host", C.POINTER(C.c_int32))]


class PrefDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("n_q", C.c_int32), ("top_k", C.c_int32), ("capacity", C.c_int32),
                ("batch", C.c_int32)]


class SparseStage1(C.Structure):
    _fields_ = [("k_absmax", C.c_void_p), ("keys_cm", C.c_void_p)]


def lib() -> C.CDLL:
    """Loads libtkv.so (built by paper_2505_19586_amd/build.py); raises if absent."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2505_19586_amd.build`")
        L = C.CDLL(path)
        L.tkv_strerror.restype = C.c_char_p
        L.tkv_strerror.argtypes = [C.c_int32]
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.tkv_quant_cache_sizes.argtypes = [C.POINTER(QuantDesc), C.POINTER(sz), C.POINTER(sz)]
        L.tkv_quantize_append.argtypes = [C.POINTER(QuantDesc), C.POINTER(QuantCache), vp, vp, i32, vp]
        L.tkv_quantize_append_ragged.argtypes = [C.POINTER(QuantDesc), C.POINTER(QuantCache), vp, vp, i32,
                                                 C.POINTER(i32), vp]
        L.tkv_sparse_append_ragged.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, i32,
                                               C.POINTER(i32), vp]
        L.tkv_quant_attn_decode.argtypes = [C.POINTER(QuantDesc), C.POINTER(QuantCache), vp, vp, C.c_float, vp, sz, vp]
        L.tkv_quant_decode.argtypes = [C.POINTER(QuantDesc), C.POINTER(QuantCache), vp, vp, i32, C.POINTER(i32), vp, vp,
                                       C.c_float, vp, sz, vp]
        L.tkv_quant_attn_decode_static.argtypes = [C.POINTER(QuantDesc), C.POINTER(QuantCache), vp, vp, C.c_float, vp]
        L.tkv_sparse_cache_sizes.argtypes = [C.POINTER(SparseDesc), C.POINTER(sz), C.POINTER(sz)]
        L.tkv_sparse_append.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, i32, vp]
        L.tkv_sparse_estimate_topk.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, vp, vp, sz, vp]
        L.tkv_sparse_gather_attn.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, vp, vp,
                                             C.c_float, vp, vp, sz, vp, vp]
        L.tkv_sparse_gather.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, vp, vp]
        L.tkv_sparse_attn.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, vp, vp, C.c_float,
                                      vp, sz, vp]
        L.tkv_sparse_stage1_sizes.argtypes = [C.POINTER(SparseDesc), C.POINTER(sz)]
        L.tkv_sparse_stage1_append.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), C.POINTER(SparseStage1),
                                               vp, i32, C.POINTER(i32), vp]
        L.tkv_sparse_select_channels.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseStage1), vp, vp, vp]
        L.tkv_sparse_prefetch_keys.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), C.POINTER(SparseStage1),
                                               vp, vp, vp]
        L.tkv_sparse_estimate_topk_cm.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, vp, i32,
                                                  vp, vp, vp, sz, vp]
        L.tkv_sparse_select_estimate_topk.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache),
                                                      C.POINTER(SparseStage1), vp, vp, vp, vp, vp, vp, sz, vp]
        L.tkv_sparse_append_dynamic.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), C.POINTER(SparseStage1),
                                                vp, vp, i32, C.POINTER(i32), vp]
        L.tkv_sparse_decode.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, i32, C.POINTER(i32),
                                        vp, vp, vp, vp, C.c_float, vp, vp, sz, vp]
        L.tkv_sparse_append_estimate_topk.argtypes = [C.POINTER(SparseDesc), C.POINTER(SparseCache), vp, vp, i32,
                                                      C.POINTER(i32), vp, vp, vp, vp, sz, vp]
        L.tkv_dense_preference_sizes.argtypes = [C.POINTER(PrefDesc), C.POINTER(sz)]
        L.tkv_dense_preference.argtypes = [C.POINTER(PrefDesc), vp, vp, i32, C.c_float, vp, vp, sz, vp]
        L.tkv_classify_layer.argtypes = [C.POINTER(C.c_float), i32, i32, C.c_float, C.POINTER(C.c_float)]
        L.tkv_debug_quant_attn_config.argtypes = [i32, i32]
        L.tkv_debug_quant_attn_config.restype = i32
        L.tkv_debug_read_sweep.argtypes = [vp, C.c_size_t, vp, i32, vp]
        L.tkv_debug_read_sweep.restype = i32
        for name in ("tkv_quant_cache_sizes", "tkv_quantize_append", "tkv_quant_attn_decode",
                     "tkv_quant_attn_decode_static",
                     "tkv_quantize_append_ragged", "tkv_sparse_append_ragged",
                     "tkv_sparse_cache_sizes", "tkv_sparse_append", "tkv_sparse_estimate_topk",
                     "tkv_sparse_gather_attn", "tkv_sparse_gather", "tkv_sparse_attn",
                     "tkv_sparse_stage1_sizes", "tkv_sparse_stage1_append", "tkv_sparse_select_channels",
                     "tkv_sparse_prefetch_keys", "tkv_sparse_estimate_topk_cm",
                     "tkv_sparse_select_estimate_topk", "tkv_sparse_append_dynamic",
                     "tkv_sparse_append_estimate_topk", "tkv_sparse_decode", "tkv_dense_preference_sizes", "tkv_dense_preference",
                     "tkv_classify_layer"):
            getattr(L, name).restype = C.c_int32
        _LIB = L
    return _LIB


def debug_quant_attn_config(kernel_choice: int = 0, target_blocks: int = 0) -> None:
    """0 = matrix-core kernel (default), 1 = reference kernel; see tkv.h."""
    _check(lib().tkv_debug_quant_attn_config(int(kernel_choice), int(target_blocks)), "tkv_debug_quant_attn_config")


def debug_read_sweep(buf: torch.Tensor, n_workgroups: int = 2048, stream=None) -> None:
    """Measurement aid: one plain read sweep over a device tensor (size a multiple of 16 bytes)."""
    assert buf.is_cuda and buf.is_contiguous()
    _check(lib().tkv_debug_read_sweep(buf.data_ptr(), buf.numel() * buf.element_size(), None, int(n_workgroups),
                                      _stream(stream)), "tkv_debug_read_sweep")


def _check(status: int, where: str) -> None:
    if status != 0:
        raise TkvError(status, where)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _require_gpu(device) -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("tkv needs an AMD GPU (gfx950); no CPU fallback exists")
    return torch.device(device)


class QuantLayer:
    """Buffers of one quantization-friendly layer plus the three entry points that
    act on them (tkv_quant_cache_sizes, tkv_quantize_append, tkv_quant_attn_decode)."""

    def __init__(self, *, n_q_heads=32, n_kv_heads=8, head_dim=128, bits=2, group_size=32, residual=128,
                 capacity, batch=1, device="cuda:0"):
        dev = _require_gpu(device)
        self.desc = QuantDesc(C.sizeof(QuantDesc), n_q_heads, n_kv_heads, head_dim, bits, group_size, residual,
                              capacity, batch)
        sizes = (C.c_size_t * 8)()
        ws = C.c_size_t()
        _check(lib().tkv_quant_cache_sizes(C.byref(self.desc), sizes, C.byref(ws)), "tkv_quant_cache_sizes")
        self.sizes = [int(s) for s in sizes]
        self.workspace_bytes = int(ws.value)
        names = ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_resid", "v_resid")
        self.buffers = {n: torch.zeros(max(s, 16), dtype=torch.uint8, device=dev) for n, s in zip(names, self.sizes)}
        # zero once: the arrival counters behind the partials must start at zero
        self.workspace = torch.zeros(self.workspace_bytes, dtype=torch.uint8, device=dev)
        self.seq_len = np.zeros(batch, dtype=np.int32)
        self.cache = QuantCache(*[self.buffers[n].data_ptr() for n in names],
                                self.seq_len.ctypes.data_as(C.POINTER(C.c_int32)))
        self.device = dev

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, n_valid=None, stream=None) -> None:
        """k_new, v_new: fp16 [B, n_new, Hkv, D] on the device; n_valid: optional
        per-sequence row counts (padded batch)."""
        d = self.desc
        assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16
        assert k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
        assert tuple(k_new.shape) == tuple(v_new.shape) and k_new.shape[0] == d.batch
        assert tuple(k_new.shape[2:]) == (d.n_kv_heads, d.head_dim)
        if n_valid is None:
            _check(lib().tkv_quantize_append(C.byref(d), C.byref(self.cache), k_new.data_ptr(), v_new.data_ptr(),
                                             int(k_new.shape[1]), _stream(stream)), "tkv_quantize_append")
        else:
            nv = np.ascontiguousarray(n_valid, dtype=np.int32)
            assert nv.shape == (d.batch,)
            _check(lib().tkv_quantize_append_ragged(C.byref(d), C.byref(self.cache), k_new.data_ptr(),
                                                    v_new.data_ptr(), int(k_new.shape[1]),
                                                    nv.ctypes.data_as(C.POINTER(C.c_int32)), _stream(stream)),
                   "tkv_quantize_append_ragged")

    def attn_decode(self, q: torch.Tensor, sm_scale: float, out: torch.Tensor | None = None, stream=None):
        d = self.desc
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (d.batch, d.n_q_heads, d.head_dim)
        if out is None:
            out = torch.empty_like(q)
        _check(lib().tkv_quant_attn_decode(C.byref(d), C.byref(self.cache), q.data_ptr(), out.data_ptr(),
                                           float(sm_scale), self.workspace.data_ptr(), self.workspace_bytes,
                                           _stream(stream)), "tkv_quant_attn_decode")
        return out

    def decode(self, q: torch.Tensor, sm_scale: float, k_new: torch.Tensor, v_new: torch.Tensor, n_valid=None,
               out: torch.Tensor | None = None, stream=None):
        """tkv_quant_decode: the step's append and the attention over the grown cache in one call
        (one launch unless the new tokens complete a quantization group)."""
        d = self.desc
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (d.batch, d.n_q_heads, d.head_dim)
        assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16
        assert k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
        assert tuple(k_new.shape) == tuple(v_new.shape) and k_new.shape[0] == d.batch
        assert tuple(k_new.shape[2:]) == (d.n_kv_heads, d.head_dim)
        nv = None
        if n_valid is not None:
            nv = np.ascontiguousarray(n_valid, dtype=np.int32)
            assert nv.shape == (d.batch,)
        if out is None:
            out = torch.empty_like(q)
        _check(lib().tkv_quant_decode(C.byref(d), C.byref(self.cache), k_new.data_ptr(), v_new.data_ptr(),
                                      int(k_new.shape[1]),
                                      None if nv is None else nv.ctypes.data_as(C.POINTER(C.c_int32)),
                                      q.data_ptr(), out.data_ptr(), float(sm_scale), self.workspace.data_ptr(),
                                      self.workspace_bytes, _stream(stream)), "tkv_quant_decode")
        return out

    def attn_decode_static(self, q: torch.Tensor, sm_scale: float, out: torch.Tensor, stream=None):
        """tkv_quant_attn_decode_static: no workspace, nothing allocated (the caller passes `out`)."""
        d = self.desc
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        assert out.dtype == torch.float16 and out.is_cuda and out.is_contiguous() and out.shape == q.shape
        assert tuple(q.shape) == (d.batch, d.n_q_heads, d.head_dim)
        _check(lib().tkv_quant_attn_decode_static(C.byref(d), C.byref(self.cache), q.data_ptr(), out.data_ptr(),
                                                  float(sm_scale), _stream(stream)), "tkv_quant_attn_decode_static")
        return out

    # typed views of the raw buffers (for tests)
    def view(self, name: str) -> torch.Tensor:
        d = self.desc
        bh = (d.batch, d.n_kv_heads)
        j = d.capacity // 32   # codes and value scalers / zero-points: blocks of 32 tokens
        buf = self.buffers[name]
        if name in ("k_codes", "v_codes"):
            return buf.view(torch.int32).view(*bh, j, 128 * d.bits)
        if name in ("k_scale", "k_zero"):
            return buf.view(torch.float16).view(*bh, d.capacity // d.group_size, 128)
        if name in ("v_scale", "v_zero"):
            return buf.view(torch.float16).view(*bh, j, 128 // d.group_size, 32)
        return buf.view(torch.float16).view(*bh, d.residual + d.group_size, 128)


class SparseLayer:
    """Buffers of one sparsity-friendly layer (GPU key summary, pinned host K/V,
    resident sink/window rows) and the entry points that act on them."""

    def __init__(self, *, n_q_heads=32, n_kv_heads=8, head_dim=128, n_channels=16, top_k=1024, n_sink=4,
                 n_window=64, capacity, batch=1, device="cuda:0", kv_host: torch.Tensor | None = None):
        dev = _require_gpu(device)
        self.desc = SparseDesc(C.sizeof(SparseDesc), n_q_heads, n_kv_heads, head_dim, n_channels, top_k, n_sink,
                               n_window, capacity, batch)
        sizes = (C.c_size_t * 4)()
        ws = C.c_size_t()
        _check(lib().tkv_sparse_cache_sizes(C.byref(self.desc), sizes, C.byref(ws)), "tkv_sparse_cache_sizes")
        self.sizes = [int(s) for s in sizes]
        self.workspace_bytes = int(ws.value)
        self.key_summary = torch.zeros(self.sizes[0] // 2, dtype=torch.float16, device=dev).view(
            batch, n_kv_heads, capacity, n_channels)
        self.channel_idx = torch.zeros(batch, n_kv_heads, n_channels, dtype=torch.int32, device=dev)
        if kv_host is None:
            kv_host = torch.empty(self.sizes[2] // 2, dtype=torch.float16, pin_memory=True)
        assert kv_host.is_pinned() and kv_host.numel() * 2 >= self.sizes[2]
        self.kv_host = kv_host.view(-1)[: self.sizes[2] // 2].view(batch, n_kv_heads, capacity, 2, head_dim)
        self.kv_local = torch.zeros(batch, n_kv_heads, n_sink + n_window, 2, head_dim, dtype=torch.float16, device=dev)
        # zero once: the Top-K histogram and counters must start at zero (each call leaves them zero)
        self.workspace = torch.zeros(self.workspace_bytes, dtype=torch.uint8, device=dev)
        self.staging = torch.empty(batch, n_kv_heads, top_k, 2, head_dim, dtype=torch.float16, device=dev)
        self.topk_idx = torch.empty(batch, n_kv_heads, top_k, dtype=torch.int32, device=dev)
        self.topk_count = torch.zeros(batch, n_kv_heads, dtype=torch.int32, device=dev)
        self.seq_len = np.zeros(batch, dtype=np.int32)
        self.cache = SparseCache(self.key_summary.data_ptr(), self.channel_idx.data_ptr(), self.kv_host.data_ptr(),
                                 self.kv_local.data_ptr(), self.seq_len.ctypes.data_as(C.POINTER(C.c_int32)))
        self.device = dev

    def set_channels(self, channel_idx) -> None:
        if not isinstance(channel_idx, torch.Tensor):
            channel_idx = torch.from_numpy(np.ascontiguousarray(channel_idx, dtype=np.int32))
        self.channel_idx.copy_(channel_idx.to(torch.int32).reshape(self.channel_idx.shape))

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, n_valid=None, stream=None) -> None:
        d = self.desc
        assert k_new.dtype == torch.float16 and k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
        assert tuple(k_new.shape) == tuple(v_new.shape) and k_new.shape[0] == d.batch
        assert tuple(k_new.shape[2:]) == (d.n_kv_heads, d.head_dim)
        if n_valid is None:
            _check(lib().tkv_sparse_append(C.byref(d), C.byref(self.cache), k_new.data_ptr(), v_new.data_ptr(),
                                           int(k_new.shape[1]), _stream(stream)), "tkv_sparse_append")
        else:
            nv = np.ascontiguousarray(n_valid, dtype=np.int32)
            assert nv.shape == (d.batch,)
            _check(lib().tkv_sparse_append_ragged(C.byref(d), C.byref(self.cache), k_new.data_ptr(),
                                                  v_new.data_ptr(), int(k_new.shape[1]),
                                                  nv.ctypes.data_as(C.POINTER(C.c_int32)), _stream(stream)),
                   "tkv_sparse_append_ragged")

    def estimate_topk(self, q: torch.Tensor, stream=None):
        d = self.desc
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (d.batch, d.n_q_heads, d.head_dim)
        _check(lib().tkv_sparse_estimate_topk(C.byref(d), C.byref(self.cache), q.data_ptr(),
                                              self.topk_idx.data_ptr(), self.topk_count.data_ptr(),
                                              self.workspace.data_ptr(), self.workspace_bytes, _stream(stream)),
               "tkv_sparse_estimate_topk")
        return self.topk_idx, self.topk_count

    def append_estimate_topk(self, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor, n_valid=None,
                             stream=None):
        """A decode step's append and estimate_topk in one call (at most 8 new tokens)."""
        d = self.desc
        assert k_new.dtype == torch.float16 and k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
        assert tuple(k_new.shape) == tuple(v_new.shape) and k_new.shape[0] == d.batch
        assert tuple(k_new.shape[2:]) == (d.n_kv_heads, d.head_dim)
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (d.batch, d.n_q_heads, d.head_dim)
        nv = None
        if n_valid is not None:
            nv = np.ascontiguousarray(n_valid, dtype=np.int32)
            assert nv.shape == (d.batch,)
        _check(lib().tkv_sparse_append_estimate_topk(
            C.byref(d), C.byref(self.cache), k_new.data_ptr(), v_new.data_ptr(), int(k_new.shape[1]),
            None if nv is None else nv.ctypes.data_as(C.POINTER(C.c_int32)), q.data_ptr(),
            self.topk_idx.data_ptr(), self.topk_count.data_ptr(), self.workspace.data_ptr(), self.workspace_bytes,
            _stream(stream)), "tkv_sparse_append_estimate_topk")
        return self.topk_idx, self.topk_count

    def decode(self, q: torch.Tensor, sm_scale: float, k_new: torch.Tensor | None = None,
               v_new: torch.Tensor | None = None, n_valid=None, out: torch.Tensor | None = None, stream=None,
               warm_next: "SparseLayer | None" = None):
        """tkv_sparse_decode: the step's append (if k_new is given), scoring, Top-K, fetch of the
        selected rows and attention in one launch.  warm_next: the sparse layer (same shape) whose
        decode is the stream's next call: its key summary is read once while this call waits for
        the host link."""
        d = self.desc
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (d.batch, d.n_q_heads, d.head_dim)
        n_new, kp, vp_, nv = 0, None, None, None
        if k_new is not None:
            assert k_new.dtype == torch.float16 and k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
            assert tuple(k_new.shape) == tuple(v_new.shape) and k_new.shape[0] == d.batch
            assert tuple(k_new.shape[2:]) == (d.n_kv_heads, d.head_dim)
            n_new, kp, vp_ = int(k_new.shape[1]), k_new.data_ptr(), v_new.data_ptr()
            if n_valid is not None:
                nv = np.ascontiguousarray(n_valid, dtype=np.int32)
                assert nv.shape == (d.batch,)
        if out is None:
            out = torch.empty_like(q)
        warm_ptr = None
        if warm_next is not None:
            assert bytes(warm_next.desc) == bytes(d), "warm_next must have this layer's descriptor"
            warm_ptr = warm_next.key_summary.data_ptr()
        _check(lib().tkv_sparse_decode(
            C.byref(d), C.byref(self.cache), kp, vp_, n_new,
            None if nv is None else nv.ctypes.data_as(C.POINTER(C.c_int32)), q.data_ptr(),
            self.topk_idx.data_ptr(), self.topk_count.data_ptr(), out.data_ptr(), float(sm_scale),
            warm_ptr, self.workspace.data_ptr(), self.workspace_bytes, _stream(stream)),
            "tkv_sparse_decode")
        return out

    def gather_attn(self, q: torch.Tensor, sm_scale: float, out: torch.Tensor | None = None,
                    gather_stream=None, compute_stream=None):
        d = self.desc
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        if out is None:
            out = torch.empty_like(q)
        cs = _stream(compute_stream)
        gs = cs if gather_stream is None else _stream(gather_stream)
        _check(lib().tkv_sparse_gather_attn(C.byref(d), C.byref(self.cache), q.data_ptr(), self.topk_idx.data_ptr(),
                                            self.topk_count.data_ptr(), out.data_ptr(), float(sm_scale),
                                            self.staging.data_ptr(), self.workspace.data_ptr(),
                                            self.workspace_bytes, gs, cs), "tkv_sparse_gather_attn")
        return out

    def gather(self, stream=None) -> None:
        _check(lib().tkv_sparse_gather(C.byref(self.desc), C.byref(self.cache), self.topk_idx.data_ptr(),
                                       self.topk_count.data_ptr(), self.staging.data_ptr(), _stream(stream)),
               "tkv_sparse_gather")

    def attn(self, q: torch.Tensor, sm_scale: float, out: torch.Tensor | None = None, stream=None):
        if out is None:
            out = torch.empty_like(q)
        _check(lib().tkv_sparse_attn(C.byref(self.desc), C.byref(self.cache), q.data_ptr(),
                                     self.topk_count.data_ptr(), self.staging.data_ptr(), out.data_ptr(),
                                     float(sm_scale), self.workspace.data_ptr(), self.workspace_bytes,
                                     _stream(stream)), "tkv_sparse_attn")
        return out


class Stage1:
    """Stage 1 buffers of one sparsity-friendly layer (tkv_sparse_stage1): running
    channel maxima, a channel-major copy of the keys (pinned host memory, or device
    memory with resident=True) and two buffers for the fetched critical key cache."""

    def __init__(self, layer: SparseLayer, resident: bool = False, keys_cm: torch.Tensor | None = None,
                 fetched: list | None = None):
        self.layer = layer
        d = layer.desc
        sizes = (C.c_size_t * 2)()
        _check(lib().tkv_sparse_stage1_sizes(C.byref(d), sizes), "tkv_sparse_stage1_sizes")
        self.k_absmax = torch.zeros(d.batch, d.n_kv_heads, d.head_dim, dtype=torch.float32, device=layer.device)
        if keys_cm is None:
            if resident:
                keys_cm = torch.zeros(int(sizes[1]) // 2, dtype=torch.float16, device=layer.device)
            else:
                keys_cm = torch.zeros(int(sizes[1]) // 2, dtype=torch.float16, pin_memory=True)
        assert keys_cm.numel() * 2 >= int(sizes[1])
        self.resident = keys_cm.is_cuda
        self.keys_cm = keys_cm.view(-1)[: int(sizes[1]) // 2].view(d.batch, d.n_kv_heads, d.head_dim, d.capacity)
        self.channel_idx = torch.zeros(d.batch, d.n_kv_heads, d.n_channels, dtype=torch.int32, device=layer.device)
        if fetched is None:   # double buffer (Sec. 4.2); layers of the same shape may share one pair
            fetched = [torch.zeros(d.batch, d.n_kv_heads, d.n_channels, d.capacity, dtype=torch.float16,
                                   device=layer.device) for _ in range(2)]
        assert len(fetched) == 2 and all(tuple(f.shape) == (d.batch, d.n_kv_heads, d.n_channels, d.capacity)
                                         for f in fetched)
        self.fetched = fetched
        self.s1 = SparseStage1(self.k_absmax.data_ptr(), self.keys_cm.data_ptr())

    def append(self, k_new: torch.Tensor, n_valid=None, stream=None) -> None:
        """Call before layer.append with the same rows."""
        d = self.layer.desc
        assert k_new.dtype == torch.float16 and k_new.is_cuda and k_new.is_contiguous()
        assert k_new.shape[0] == d.batch and tuple(k_new.shape[2:]) == (d.n_kv_heads, d.head_dim)
        nv = None
        if n_valid is not None:
            nv = np.ascontiguousarray(n_valid, dtype=np.int32)
            assert nv.shape == (d.batch,)
        _check(lib().tkv_sparse_stage1_append(C.byref(d), C.byref(self.layer.cache), C.byref(self.s1),
                                              k_new.data_ptr(), int(k_new.shape[1]),
                                              None if nv is None else nv.ctypes.data_as(C.POINTER(C.c_int32)),
                                              _stream(stream)), "tkv_sparse_stage1_append")

    def append_both(self, k_new: torch.Tensor, v_new: torch.Tensor, n_valid=None, stream=None) -> None:
        """Stage 1 buffers and the layer's own cache in one call (tkv_sparse_append_dynamic)."""
        L = self.layer
        d = L.desc
        assert k_new.dtype == torch.float16 and k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
        assert tuple(k_new.shape) == tuple(v_new.shape) and k_new.shape[0] == d.batch
        assert tuple(k_new.shape[2:]) == (d.n_kv_heads, d.head_dim)
        nv = None
        if n_valid is not None:
            nv = np.ascontiguousarray(n_valid, dtype=np.int32)
            assert nv.shape == (d.batch,)
        _check(lib().tkv_sparse_append_dynamic(C.byref(d), C.byref(L.cache), C.byref(self.s1), k_new.data_ptr(),
                                               v_new.data_ptr(), int(k_new.shape[1]),
                                               None if nv is None else nv.ctypes.data_as(C.POINTER(C.c_int32)),
                                               _stream(stream)), "tkv_sparse_append_dynamic")

    def select_estimate_topk(self, q_hat: torch.Tensor, q: torch.Tensor, stream=None):
        """Eq. 10 and Stage 2 in one call over the resident channel-major keys."""
        L = self.layer
        d = L.desc
        for t in (q_hat, q):
            assert t.dtype == torch.float16 and t.is_cuda and t.is_contiguous()
            assert tuple(t.shape) == (d.batch, d.n_q_heads, d.head_dim)
        _check(lib().tkv_sparse_select_estimate_topk(C.byref(d), C.byref(L.cache), C.byref(self.s1), q_hat.data_ptr(),
                                                     q.data_ptr(), self.channel_idx.data_ptr(), L.topk_idx.data_ptr(),
                                                     L.topk_count.data_ptr(), L.workspace.data_ptr(),
                                                     L.workspace_bytes, _stream(stream)),
               "tkv_sparse_select_estimate_topk")
        return L.topk_idx, L.topk_count

    def select_channels(self, q_hat: torch.Tensor, stream=None) -> torch.Tensor:
        d = self.layer.desc
        assert q_hat.dtype == torch.float16 and q_hat.is_cuda and q_hat.is_contiguous()
        assert tuple(q_hat.shape) == (d.batch, d.n_q_heads, d.head_dim)
        _check(lib().tkv_sparse_select_channels(C.byref(d), C.byref(self.s1), q_hat.data_ptr(),
                                                self.channel_idx.data_ptr(), _stream(stream)),
               "tkv_sparse_select_channels")
        return self.channel_idx

    def prefetch(self, buf: int = 0, stream=None) -> torch.Tensor:
        """Fetch the rows of the current channel list into double-buffer half `buf`."""
        _check(lib().tkv_sparse_prefetch_keys(C.byref(self.layer.desc), C.byref(self.layer.cache), C.byref(self.s1),
                                              self.channel_idx.data_ptr(), self.fetched[buf].data_ptr(),
                                              _stream(stream)), "tkv_sparse_prefetch_keys")
        return self.fetched[buf]

    def estimate_topk(self, q: torch.Tensor, buf: int | None = 0, stream=None):
        """Stage 2 over the fetched buffer `buf`, or (buf=None, resident keys only) in place
        over the channel-major keys."""
        L = self.layer
        d = L.desc
        assert q.dtype == torch.float16 and q.is_cuda and q.is_contiguous()
        if buf is None:
            assert self.resident, "in-place scoring needs device-resident channel-major keys"
            keys, rows = self.keys_cm, d.head_dim
        else:
            keys, rows = self.fetched[buf], d.n_channels
        _check(lib().tkv_sparse_estimate_topk_cm(C.byref(d), C.byref(L.cache), q.data_ptr(),
                                                 self.channel_idx.data_ptr(), keys.data_ptr(), int(rows),
                                                 L.topk_idx.data_ptr(), L.topk_count.data_ptr(),
                                                 L.workspace.data_ptr(), L.workspace_bytes, _stream(stream)),
               "tkv_sparse_estimate_topk_cm")
        return L.topk_idx, L.topk_count


class DensePreference:
    """Offline identification of a layer (tkv_dense_preference, tkv_classify_layer)."""

    def __init__(self, *, n_q_heads=32, n_kv_heads=8, head_dim=128, n_q=64, top_k=1024, capacity, batch=1,
                 device="cuda:0"):
        dev = _require_gpu(device)
        self.desc = PrefDesc(C.sizeof(PrefDesc), n_q_heads, n_kv_heads, head_dim, n_q, top_k, capacity, batch)
        ws = C.c_size_t()
        _check(lib().tkv_dense_preference_sizes(C.byref(self.desc), C.byref(ws)), "tkv_dense_preference_sizes")
        self.workspace_bytes = int(ws.value)
        self.workspace = torch.zeros(self.workspace_bytes, dtype=torch.uint8, device=dev)
        self.device = dev

    def score(self, q_last: torch.Tensor, k: torch.Tensor, sm_scale: float, stream=None) -> torch.Tensor:
        """q_last fp16 [B, n_q, Hq, D], k fp16 [B, n, Hkv, D] -> float32 [B, Hq] (Eq. 8 per head)."""
        d = self.desc
        for t in (q_last, k):
            assert t.dtype == torch.float16 and t.is_cuda and t.is_contiguous()
        assert tuple(q_last.shape) == (d.batch, d.n_q, d.n_q_heads, d.head_dim)
        assert k.shape[0] == d.batch and tuple(k.shape[2:]) == (d.n_kv_heads, d.head_dim)
        out = torch.empty(d.batch, d.n_q_heads, dtype=torch.float32, device=self.device)
        _check(lib().tkv_dense_preference(C.byref(d), q_last.data_ptr(), k.data_ptr(), int(k.shape[1]),
                                          float(sm_scale), out.data_ptr(), self.workspace.data_ptr(),
                                          self.workspace_bytes, _stream(stream)), "tkv_dense_preference")
        return out

    def classify(self, p_heads: torch.Tensor, tau: float = 0.2):
        """Eq. 9 for one sequence: (True if quantization-friendly, layer score)."""
        p = np.ascontiguousarray(p_heads.detach().float().cpu().numpy().reshape(-1), dtype=np.float32)
        score = C.c_float()
        r = lib().tkv_classify_layer(p.ctypes.data_as(C.POINTER(C.c_float)), int(p.size), int(self.desc.n_q),
                                     float(tau), C.byref(score))
        if r < 0:
            raise TkvError(r, "tkv_classify_layer")
        return bool(r), float(score.value)
