"""MI355X-native decode attention for TailorKV's hybrid KV cache (arxiv 2505.19586).

Thin ctypes binding over libtkv.so (hand-written HIP for gfx950).  PyTorch is used
only for device memory and streams.
"""
from .tkv import (  # noqa: F401
    DensePreference, QuantDesc, QuantLayer, SparseDesc, SparseLayer, Stage1, TkvError, debug_quant_attn_config, debug_read_sweep, lib, library_path,
)
