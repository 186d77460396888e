"""kvx: compressed-KV streaming attention step (XStreamVGGT hot path) for MI355X.

Thin ctypes binding over libkvx.so; every step of the path runs in the library's HIP
kernels.  PyTorch is used by callers only for device memory and streams.
"""
from .binding import (  # noqa: F401
    KV_BF16, KV_F32, KV_COMPRESSED, KV_UNCOMPRESSED_BF16, KV_META_F32, KV_META_F16, KV_ATTEND_THEN_PRUNE, KV_PRUNE_THEN_ATTEND, KV_LAYOUT_COMPACT, KV_LAYOUT_SLOTS, KERNEL_NAMES,
    KvConfig, KvStats, KvError, KvHandle, load_library, library_path, probe_mfma_bf16, probe_copy,
)
