"""The C-ABI library loads, exports every symbol include/*.h declares, and reports
argument errors without touching a GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2505_19586_amd as tkv
from paper_2505_19586_amd import build as tkv_build
from paper_2505_19586_amd.tkv import QuantCache, QuantDesc, SparseCache, SparseDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(tkv.library_path()):
        tkv_build.build_library()
    return tkv.lib()


def _declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(tkv_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_debug_hooks_are_not_in_the_product_header():
    text = open(os.path.join(ROOT, "include", "tkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert "tkv_debug_" not in text
    assert "tkv_debug_read_sweep" in open(os.path.join(ROOT, "include", "tkv_debug.h")).read()


def test_every_declared_symbol_is_exported(L):
    names = _declared_functions()
    for required in ("tkv_quantize_append", "tkv_quant_attn_decode", "tkv_sparse_estimate_topk",
                     "tkv_sparse_gather_attn"):
        assert required in names
    for n in names:
        assert hasattr(L, n), n


def test_strerror(L):
    assert L.tkv_strerror(0) == b"ok"
    seen = {L.tkv_strerror(s) for s in range(-6, 1)}
    assert len(seen) == 7
    assert b"unknown" in L.tkv_strerror(-99)


def _qdesc(**kw):
    d = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, bits=2, group_size=32, residual=128, capacity=4096, batch=1)
    d.update(kw)
    return QuantDesc(C.sizeof(QuantDesc), d["n_q_heads"], d["n_kv_heads"], d["head_dim"], d["bits"],
                     d["group_size"], d["residual"], d["capacity"], d["batch"])


def _sdesc(**kw):
    d = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, n_channels=16, top_k=128, n_sink=4, n_window=64,
             capacity=4096, batch=1)
    d.update(kw)
    return SparseDesc(C.sizeof(SparseDesc), d["n_q_heads"], d["n_kv_heads"], d["head_dim"], d["n_channels"],
                      d["top_k"], d["n_sink"], d["n_window"], d["capacity"], d["batch"])


def test_quant_sizes_follow_table2(L):
    """Sec. 4.4 Table 2: 2*n*h*d_h*(b/16 + 2/g) fp16 elements."""
    for bits, g, per_tok_head in ((2, 32, 96), (4, 32, 160), (1, 64, 48), (2, 64, 80)):
        d = _qdesc(bits=bits, group_size=g, capacity=131072)
        sizes = (C.c_size_t * 8)()
        ws = C.c_size_t()
        assert L.tkv_quant_cache_sizes(C.byref(d), sizes, C.byref(ws)) == 0
        total = sum(sizes[:6])
        assert total == per_tok_head * 131072 * 8
        assert total == int(2 * 131072 * 8 * 128 * (bits / 16 + 2 / g) * 2)
        assert sizes[6] == sizes[7] == 8 * (128 + g) * 128 * 2
        assert ws.value > 0


def test_sparse_sizes(L):
    d = _sdesc(capacity=131072, top_k=1024)
    sizes = (C.c_size_t * 4)()
    ws = C.c_size_t()
    assert L.tkv_sparse_cache_sizes(C.byref(d), sizes, C.byref(ws)) == 0
    assert sizes[0] == 131072 * 8 * 16 * 2              # one buffer of Table 2's 2*n*h*d_s elements
    assert sizes[2] == 512 * 1024 * 1024
    assert sizes[3] == 8 * 68 * 2 * 128 * 2


@pytest.mark.parametrize("kw,status", [
    (dict(bits=3), -2), (dict(bits=8), -2), (dict(bits=0), -1), (dict(head_dim=64), -2), (dict(group_size=16), -2),
    (dict(group_size=128), -2), (dict(group_size=64, residual=96), -1), (dict(group_size=64, capacity=4096 + 32), -1),
    (dict(residual=1024), -2), (dict(bits=1, group_size=64), 0), (dict(bits=1), 0), (dict(bits=4, group_size=64), 0),
    (dict(n_q_heads=30), -1), (dict(n_q_heads=64), 0), (dict(n_q_heads=56), 0), (dict(n_q_heads=72), -2),
    (dict(batch=0), -1), (dict(batch=65), -2),
    (dict(capacity=100), -1), (dict(residual=100), -1), (dict(residual=0), -2), (dict(capacity=0), -1),
])
def test_quant_desc_errors(L, kw, status):
    d = _qdesc(**kw)
    assert L.tkv_quant_cache_sizes(C.byref(d), None, None) == status


def test_bad_struct_size_and_null(L):
    d = _qdesc()
    d.struct_size = 12
    assert L.tkv_quant_cache_sizes(C.byref(d), None, None) == -1
    assert L.tkv_quant_cache_sizes(None, None, None) == -1
    s = _sdesc()
    s.struct_size = 0
    assert L.tkv_sparse_cache_sizes(C.byref(s), None, None) == -1


@pytest.mark.parametrize("kw,status", [
    (dict(n_channels=10), -2), (dict(n_channels=12), 0), (dict(n_channels=0), -1), (dict(top_k=0), -1), (dict(top_k=5000), -2),
    (dict(n_window=0), -1), (dict(n_sink=-1), -1), (dict(head_dim=96), -2),
    (dict(n_q_heads=64), 0), (dict(n_q_heads=24), 0), (dict(n_q_heads=72), -2),   # groups of up to 8
])
def test_sparse_desc_errors(L, kw, status):
    assert L.tkv_sparse_cache_sizes(C.byref(_sdesc(**kw)), None, None) == status


def test_call_errors_before_any_gpu_work(L):
    d = _qdesc(capacity=64 * 32)
    lens = (C.c_int32 * 1)(2040)
    fake = 0x1000
    cache = QuantCache(*([fake] * 8), lens)
    # NULL inputs
    assert L.tkv_quantize_append(C.byref(d), C.byref(cache), None, fake, 4, None) == -1
    assert L.tkv_quantize_append(C.byref(d), None, fake, fake, 4, None) == -1
    # capacity
    assert L.tkv_quantize_append(C.byref(d), C.byref(cache), fake, fake, 9, None) == -3
    assert lens[0] == 2040
    # n_new == 0 is a no-op, negative is invalid
    assert L.tkv_quantize_append(C.byref(d), C.byref(cache), fake, fake, 0, None) == 0
    assert L.tkv_quantize_append(C.byref(d), C.byref(cache), fake, fake, -1, None) == -1
    # ragged: n_valid > n_new
    nv = (C.c_int32 * 1)(5)
    assert L.tkv_quantize_append_ragged(C.byref(d), C.byref(cache), fake, fake, 4, nv, None) == -1
    # workspace too small / NULL
    assert L.tkv_quant_attn_decode(C.byref(d), C.byref(cache), fake, fake, 0.1, fake, 16, None) == -4
    assert L.tkv_quant_attn_decode(C.byref(d), C.byref(cache), fake, None, 0.1, fake, 1 << 30, None) == -1
    # the decode step in one call: the append's and the attention's checks, nothing enqueued, lengths kept
    L.tkv_quant_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    qd = lambda *a: L.tkv_quant_decode(C.byref(d), C.byref(cache), *a)
    assert qd(None, fake, 1, None, fake, fake, 0.1, fake, 1 << 30, None) == -1
    assert qd(fake, fake, -1, None, fake, fake, 0.1, fake, 1 << 30, None) == -1
    assert qd(fake, fake, 1, None, None, fake, 0.1, fake, 1 << 30, None) == -1
    assert qd(fake, fake, 1, None, fake, fake, 0.1, None, 1 << 30, None) == -1
    assert qd(fake, fake, 1, None, fake, fake, 0.1, fake, 16, None) == -4
    assert qd(fake, fake, 9, None, fake, fake, 0.1, fake, 1 << 30, None) == -3
    assert qd(fake, fake, 4, C.addressof(nv), fake, fake, 0.1, fake, 1 << 30, None) == -1
    assert lens[0] == 2040
    lens[0] = 5000
    assert L.tkv_quant_attn_decode(C.byref(d), C.byref(cache), fake, fake, 0.1, fake, 1 << 30, None) == -3

    s = _sdesc()
    slens = (C.c_int32 * 1)(4090)
    sc = SparseCache(fake, fake, fake, fake, slens)
    assert L.tkv_sparse_append(C.byref(s), C.byref(sc), fake, fake, 10, None) == -3
    assert L.tkv_sparse_estimate_topk(C.byref(s), C.byref(sc), fake, fake, fake, fake, 8, None) == -4
    assert L.tkv_sparse_estimate_topk(C.byref(s), C.byref(sc), None, fake, fake, fake, 1 << 30, None) == -1
    assert L.tkv_sparse_gather_attn(C.byref(s), C.byref(sc), fake, fake, fake, fake, 0.1, fake, fake, 8,
                                    None, None) == -4
    assert L.tkv_sparse_gather_attn(C.byref(s), C.byref(sc), fake, fake, fake, None, 0.1, fake, fake, 1 << 30,
                                    None, None) == -1
    assert L.tkv_sparse_attn(C.byref(s), C.byref(sc), fake, fake, fake, fake, 0.1, fake, 8, None) == -4
    # a plain (unpinned) host pointer is rejected, never dereferenced
    import numpy as np
    plain = np.zeros(1024, np.uint8)
    sc2 = SparseCache(fake, fake, plain.ctypes.data, fake, slens)
    assert L.tkv_sparse_gather(C.byref(s), C.byref(sc2), fake, fake, fake, None) in (-5, -6)


def test_read_sweep_argument_errors(L):
    fake = 0x1000
    assert L.tkv_debug_read_sweep(None, 1024, None, 256, None) == -1
    assert L.tkv_debug_read_sweep(fake, 0, None, 256, None) == -1
    assert L.tkv_debug_read_sweep(fake, 1000, None, 256, None) == -1        # not a multiple of 16
    assert L.tkv_debug_read_sweep(fake + 4, 1024, None, 256, None) == -1    # misaligned
    assert L.tkv_debug_read_sweep(fake, 1024, None, 0, None) == -1
    assert L.tkv_debug_read_sweep(fake, 1024, None, 1 << 20, None) == -1


def test_stage1_and_fused_entry_points_validate_before_any_gpu_work(L):
    from paper_2505_19586_amd.tkv import SparseCache, SparseStage1
    fake = C.c_void_p(0x1000)
    s = _sdesc()                                   # capacity 4096
    lens = (C.c_int32 * 1)(4090)
    sc = SparseCache(fake, fake, fake, fake, lens)
    s1 = SparseStage1(fake, fake)
    sizes = (C.c_size_t * 2)()
    assert L.tkv_sparse_stage1_sizes(C.byref(s), sizes) == 0
    assert sizes[0] == 8 * 128 * 4 and sizes[1] == 8 * 128 * 4096 * 2
    assert L.tkv_sparse_stage1_sizes(C.byref(s), None) == -1
    # capacity
    assert L.tkv_sparse_stage1_append(C.byref(s), C.byref(sc), C.byref(s1), fake, 10, None, None) == -3
    assert L.tkv_sparse_append_dynamic(C.byref(s), C.byref(sc), C.byref(s1), fake, fake, 10, None, None) == -3
    assert L.tkv_sparse_append_estimate_topk(C.byref(s), C.byref(sc), fake, fake, 7, None, fake, fake, fake, fake,
                                             1 << 30, None) == -3
    assert lens[0] == 4090                         # nothing was appended
    # too many rows for the fused decode-step form, NULL arguments, channel-major shape rules
    assert L.tkv_sparse_append_estimate_topk(C.byref(s), C.byref(sc), fake, fake, 9, None, fake, fake, fake, fake,
                                             1 << 30, None) == -1
    assert L.tkv_sparse_select_channels(C.byref(s), C.byref(s1), None, fake, None) == -1
    assert L.tkv_sparse_select_channels(C.byref(s), None, fake, fake, None) == -1
    assert L.tkv_sparse_prefetch_keys(C.byref(s), C.byref(sc), C.byref(s1), None, fake, None) == -1
    assert L.tkv_sparse_estimate_topk_cm(C.byref(s), C.byref(sc), fake, fake, fake, 7, fake, fake, fake, 1 << 30,
                                         None) == -1          # rows_per_head must be d_s or 128
    assert L.tkv_sparse_estimate_topk_cm(C.byref(s), C.byref(sc), fake, fake, fake, 16, fake, fake, fake, 8,
                                         None) == -4          # workspace too small
    odd = _sdesc(capacity=4100)                                # channel-major rows need capacity % 8 == 0
    assert L.tkv_sparse_estimate_topk_cm(C.byref(odd), C.byref(sc), fake, fake, fake, 16, fake, fake, fake,
                                         1 << 30, None) == -1
    assert L.tkv_sparse_stage1_append(C.byref(odd), C.byref(sc), C.byref(s1), fake, 1, None, None) == -1


def test_dense_preference_validation_and_host_classification(L):
    from paper_2505_19586_amd.tkv import PrefDesc
    fake = C.c_void_p(0x1000)

    def desc(**kw):
        d = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, n_q=64, top_k=1024, capacity=4096, batch=1)
        d.update(kw)
        return PrefDesc(C.sizeof(PrefDesc), d["n_q_heads"], d["n_kv_heads"], d["head_dim"], d["n_q"], d["top_k"],
                        d["capacity"], d["batch"])
    ws = C.c_size_t()
    assert L.tkv_dense_preference_sizes(C.byref(desc()), C.byref(ws)) == 0 and ws.value > 4 * 256 * 4096
    for kw, status in ((dict(n_q=20), -2), (dict(n_q=0), -1), (dict(top_k=5000), -2), (dict(head_dim=64), -2),
                       (dict(n_q_heads=30), -1), (dict(capacity=0), -1)):
        assert L.tkv_dense_preference_sizes(C.byref(desc(**kw)), C.byref(ws)) == status
    assert L.tkv_dense_preference_sizes(C.byref(desc()), None) == -1
    d = desc()
    assert L.tkv_dense_preference(C.byref(d), fake, fake, 5000, 0.1, fake, fake, 1 << 40, None) == -3   # n > capacity
    assert L.tkv_dense_preference(C.byref(d), fake, fake, 100, 0.1, fake, fake, 8, None) == -4          # workspace
    assert L.tkv_dense_preference(C.byref(d), None, fake, 100, 0.1, fake, fake, 1 << 40, None) == -1
    # Eq. 9 on the host: mean over heads of P / n_q against tau
    p = (C.c_float * 4)(8.0, 16.0, 24.0, 32.0)            # n_q = 64 -> shares 0.125 .. 0.5, mean 0.3125
    score = C.c_float()
    assert L.tkv_classify_layer(p, 4, 64, 0.2, C.byref(score)) == 1 and abs(score.value - 0.3125) < 1e-7
    assert L.tkv_classify_layer(p, 4, 64, 0.4, None) == 0
    assert L.tkv_classify_layer(None, 4, 64, 0.2, None) == -1
    assert L.tkv_classify_layer(p, 0, 64, 0.2, None) == -1


def test_binding_refuses_to_run_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        tkv.QuantLayer(capacity=4096)
    with pytest.raises(RuntimeError):
        tkv.SparseLayer(capacity=4096)


def test_library_leaves_the_callers_last_error_alone(L):
    """An earlier HIP error of the calling program is neither reported as the library's nor
    erased by it: argument checks and size helpers make no HIP call that could do either."""
    hip = C.CDLL("libamdhip64.so")
    hip.hipSetDevice.argtypes = [C.c_int]
    assert hip.hipSetDevice(12345) != 0                 # the caller's own error
    d = _qdesc()
    sizes = (C.c_size_t * 8)()
    assert L.tkv_quant_cache_sizes(C.byref(d), sizes, None) == 0
    assert L.tkv_quant_attn_decode(C.byref(d), None, None, None, C.c_float(1.0), None, 0, None) == -1
    sd = _sdesc()
    assert L.tkv_sparse_estimate_topk(C.byref(sd), None, None, None, None, None, 0, None) == -1
    assert hip.hipGetLastError() != 0                   # still there for the caller to read
