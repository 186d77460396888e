"""ctypes binding of the C ABI declared in include/kvx.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

KV_BF16, KV_F32 = 0, 1
KV_COMPRESSED, KV_UNCOMPRESSED_BF16 = 0, 1
KV_META_F32, KV_META_F16 = 0, 1
KV_ATTEND_THEN_PRUNE, KV_PRUNE_THEN_ATTEND = 0, 1
KV_LAYOUT_COMPACT, KV_LAYOUT_SLOTS = 0, 1
KERNEL_NAMES = ["attention", "combine", "pool", "score", "select", "rebuild_k", "rebuild_v"]

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    return os.path.join(_HERE, "libkvx.so")


class KvConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_streams", "n_layers", "n_heads", "head_dim", "tokens_per_frame", "n_special", "pool_group",
        "budget_tokens", "k_bits", "k_group", "v_bits", "v_group", "in_dtype", "out_dtype", "mode", "max_frames")] + [
        ("softmax_scale", C.c_float), ("meta_format", C.c_int32), ("max_frames_per_step", C.c_int32), ("order", C.c_int32), ("layout", C.c_int32)]


class KvStepItem(C.Structure):
    _fields_ = [("stream", C.c_int32), ("layer", C.c_int32), ("q", C.c_void_p), ("k", C.c_void_p),
                ("v", C.c_void_p), ("out", C.c_void_p)]


class KvStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "bytes_allocated", "bytes_k_codes", "bytes_k_meta", "bytes_v_codes", "bytes_v_meta", "bytes_ids",
        "bytes_scratch", "bytes_live_per_cache", "frames_seen_total", "tokens_dropped_total",
        "k_groups_rebuilt_total")] + [(n, C.c_int32) for n in ("cache_len_min", "cache_len_max", "n_caches", "nonfinite_flag")] + [
        ("zp_range_warnings", C.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class KvExport(C.Structure):
    _fields_ = [("cache_len", C.c_int32), ("frames_seen", C.c_int32), ("last_keep_len", C.c_int32),
                ("last_scores_len", C.c_int32), ("ids", C.c_void_p), ("k_codes", C.c_void_p), ("k_scale", C.c_void_p),
                ("k_zero", C.c_void_p), ("v_codes", C.c_void_p), ("v_scale", C.c_void_p), ("v_zero", C.c_void_p),
                ("last_keep", C.c_void_p), ("last_scores", C.c_void_p), ("capacity_tokens", C.c_int32)]


class KvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"kvx error {code}: {msg}")
        self.code = code


_lib = None


def load_library():
    """Load libkvx.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(path)
    P = C.c_void_p
    lib.kv_init.argtypes = [C.POINTER(KvConfig), C.POINTER(P)]
    lib.kv_step.argtypes = [P, C.c_int32, C.c_int32, P, P, P, C.c_int64, C.c_int64, P, P]
    lib.kv_step_frames.argtypes = [P, C.c_int32, C.c_int32, C.c_int32, P, P, P, C.c_int64, C.c_int64, P, P]
    lib.kv_step_static.argtypes = [P, C.c_int32, C.c_int32, P, P, P, C.c_int64, C.c_int64, P, P]
    lib.kv_step_batched.argtypes = [P, C.c_int32, C.POINTER(KvStepItem), C.c_int64, C.c_int64, P]
    lib.kv_stats.argtypes = [P, C.POINTER(KvStats)]
    lib.kv_export.argtypes = [P, C.c_int32, C.c_int32, C.POINTER(KvExport)]
    lib.kv_reset.argtypes = [P, C.c_int32, C.c_int32]
    lib.kv_set_stream_tokens.argtypes = [P, C.c_int32, C.c_int32]
    lib.kv_import.argtypes = [P, C.c_int32, C.c_int32, C.POINTER(KvExport)]
    lib.kv_destroy.argtypes = [P]
    lib.kv_destroy.restype = None
    lib.kv_last_error.argtypes = [P]
    lib.kv_last_error.restype = C.c_char_p
    lib.kv_set_timing.argtypes = [P, C.c_uint32]
    lib.kv_read_timing.argtypes = [P, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.kv_set_option.argtypes = [P, C.c_char_p, C.c_int64]
    lib.kv_probe_mfma_bf16.argtypes = [C.c_int32, C.c_int32, P, C.POINTER(C.c_double)]
    lib.kv_probe_copy.argtypes = [C.c_int64, C.c_int32, P, C.POINTER(C.c_double)]
    for name in ("kv_init", "kv_step", "kv_step_frames", "kv_step_static", "kv_step_batched", "kv_stats", "kv_export", "kv_reset", "kv_set_stream_tokens", "kv_set_timing",
                 "kv_read_timing", "kv_set_option", "kv_probe_mfma_bf16", "kv_probe_copy", "kv_import"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def probe_mfma_bf16(iters: int = 50000, repeats: int = 3, hip_stream: int = 0) -> float:
    """kv_probe_mfma_bf16: TFLOP/s of a register-resident bf16 matrix-instruction loop on every compute unit."""
    out = C.c_double(0.0)
    rc = load_library().kv_probe_mfma_bf16(iters, repeats, hip_stream, C.byref(out))
    if rc != 0:
        raise KvError(rc, "kv_probe_mfma_bf16 failed")
    return out.value


def probe_copy(nbytes: int = 1 << 30, repeats: int = 3, hip_stream: int = 0) -> float:
    """kv_probe_copy: GB/s (read + written) of a streaming device-to-device copy of nbytes bytes."""
    out = C.c_double(0.0)
    rc = load_library().kv_probe_copy(nbytes, repeats, hip_stream, C.byref(out))
    if rc != 0:
        raise KvError(rc, "kv_probe_copy failed")
    return out.value


class KvHandle:
    """Owner of one kv_handle.  Tensors passed to step() only supply data_ptr() and strides."""

    def __init__(self, **cfg):
        self.lib = load_library()
        c = KvConfig()
        defaults = dict(n_streams=1, n_layers=1, head_dim=64, pool_group=16, k_bits=4, k_group=64, v_bits=4, v_group=64,
                        in_dtype=KV_BF16, out_dtype=None, mode=KV_COMPRESSED, max_frames=0, softmax_scale=0.0, budget_tokens=0,
                        meta_format=KV_META_F32, max_frames_per_step=1, order=KV_ATTEND_THEN_PRUNE, layout=KV_LAYOUT_COMPACT)
        defaults.update(cfg)
        if defaults["out_dtype"] is None:
            defaults["out_dtype"] = defaults["in_dtype"]
        for k, v in defaults.items():
            setattr(c, k, v)
        self.cfg = c
        self._h = C.c_void_p()
        rc = self.lib.kv_init(C.byref(c), C.byref(self._h))
        if rc != 0:
            raise KvError(rc, self.lib.kv_last_error(None).decode())

    def _check(self, rc):
        if rc != 0:
            raise KvError(rc, self.lib.kv_last_error(self._h).decode())

    @staticmethod
    def _strides(t):
        assert t.dim() == 3 and t.stride(2) == 1, "q/k/v/out must be [n, H, d] with contiguous channels"
        return t.stride(0), t.stride(1)

    def step(self, q, k, v, out, stream: int = 0, layer: int = 0, hip_stream: int = 0):
        ts, hs = self._strides(q)
        for t in (k, v):
            assert self._strides(t) == (ts, hs) and t.dtype == q.dtype
        assert self._strides(out) == (ts, hs)
        self._check(self.lib.kv_step(self._h, stream, layer, q.data_ptr(), k.data_ptr(), v.data_ptr(), ts, hs,
                                     out.data_ptr(), hip_stream))

    def step_frames(self, n_frames: int, q, k, v, out, stream: int = 0, layer: int = 0, hip_stream: int = 0):
        """kv_step_frames: q, k, v, out hold n_frames consecutive frames, [n_frames * n, H, d]."""
        ts, hs = self._strides(q)
        for t in (k, v):
            assert self._strides(t) == (ts, hs) and t.dtype == q.dtype
        assert self._strides(out) == (ts, hs)
        self._check(self.lib.kv_step_frames(self._h, stream, layer, n_frames, q.data_ptr(), k.data_ptr(), v.data_ptr(), ts, hs,
                                            out.data_ptr(), hip_stream))

    def step_static(self, q, k, v, out, stream: int = 0, layer: int = 0, hip_stream: int = 0):
        """kv_step_static: kv_step with the attention partials in the library's static device array."""
        ts, hs = self._strides(q)
        for t in (k, v):
            assert self._strides(t) == (ts, hs) and t.dtype == q.dtype
        assert self._strides(out) == (ts, hs)
        self._check(self.lib.kv_step_static(self._h, stream, layer, q.data_ptr(), k.data_ptr(), v.data_ptr(), ts, hs,
                                            out.data_ptr(), hip_stream))

    def step_batched(self, items, hip_stream: int = 0):
        """items: list of (stream, layer, q, k, v, out)."""
        arr = (KvStepItem * len(items))()
        ts, hs = self._strides(items[0][2])
        for i, (s, l, q, k, v, o) in enumerate(items):
            for t in (q, k, v, o):
                assert self._strides(t) == (ts, hs)
            arr[i] = KvStepItem(s, l, q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr())
        self._check(self.lib.kv_step_batched(self._h, len(items), arr, ts, hs, hip_stream))

    def stats(self) -> dict:
        s = KvStats()
        self._check(self.lib.kv_stats(self._h, C.byref(s)))
        return s.as_dict()

    def export(self, stream: int = 0, layer: int = 0) -> dict:
        c = self.cfg
        H, d = c.n_heads, c.head_dim
        cap = c.budget_tokens
        G = -(-cap // c.k_group)
        ngv = d // c.v_group
        bufs = dict(
            ids=np.zeros(cap, np.int32), k_codes=np.zeros((H, cap, d), np.uint8), k_scale=np.zeros((H, G, d), np.float32),
            k_zero=np.zeros((H, G, d), np.int32), v_codes=np.zeros((H, cap, d), np.uint8),
            v_scale=np.zeros((H, cap, ngv), np.float32), v_zero=np.zeros((H, cap, ngv), np.int32),
            last_keep=np.zeros(cap, np.int32), last_scores=np.zeros(cap, np.float32))
        x = KvExport()
        x.capacity_tokens = cap
        for name, a in bufs.items():
            setattr(x, name, a.ctypes.data)
        self._check(self.lib.kv_export(self._h, stream, layer, C.byref(x)))
        T = x.cache_len
        Gt = -(-T // c.k_group)
        # the library packs each [H, T, ...] part densely for the exported length T
        out = dict(cache_len=T, frames_seen=x.frames_seen)
        out["ids"] = bufs["ids"][:T].copy()
        out["k_codes"] = bufs["k_codes"].reshape(-1)[:H * T * d].reshape(H, T, d).copy()
        out["v_codes"] = bufs["v_codes"].reshape(-1)[:H * T * d].reshape(H, T, d).copy()
        out["k_scale"] = bufs["k_scale"].reshape(-1)[:H * Gt * d].reshape(H, Gt, d).copy()
        out["k_zero"] = bufs["k_zero"].reshape(-1)[:H * Gt * d].reshape(H, Gt, d).copy()
        out["v_scale"] = bufs["v_scale"].reshape(-1)[:H * T * ngv].reshape(H, T, ngv).copy()
        out["v_zero"] = bufs["v_zero"].reshape(-1)[:H * T * ngv].reshape(H, T, ngv).copy()
        out["last_keep"] = bufs["last_keep"][:x.last_keep_len].copy() if x.last_keep_len else None
        out["last_scores"] = bufs["last_scores"][:x.last_scores_len].copy() if x.last_keep_len else None
        return out

    def import_state(self, state: dict, stream: int = 0, layer: int = 0):
        """kv_import: load what export() returned (of this or another handle with the same configuration)."""
        arrs = dict(ids=(np.int32, state["ids"]), k_codes=(np.uint8, state["k_codes"]), k_scale=(np.float32, state["k_scale"]),
                    k_zero=(np.int32, state["k_zero"]), v_codes=(np.uint8, state["v_codes"]),
                    v_scale=(np.float32, state["v_scale"]), v_zero=(np.int32, state["v_zero"]))
        x = KvExport()
        x.cache_len = int(state["cache_len"])
        x.frames_seen = int(state["frames_seen"])
        x.capacity_tokens = x.cache_len
        keep = []
        for name, (dt, a) in arrs.items():
            a = np.ascontiguousarray(a, dtype=dt)
            keep.append(a)
            setattr(x, name, a.ctypes.data)
        self._check(self.lib.kv_import(self._h, stream, layer, C.byref(x)))

    def set_stream_tokens(self, stream: int, tokens_per_frame: int):
        self._check(self.lib.kv_set_stream_tokens(self._h, stream, tokens_per_frame))

    def reset(self, stream: int = -1, layer: int = -1):
        self._check(self.lib.kv_reset(self._h, stream, layer))

    def set_timing(self, mask: int):
        self._check(self.lib.kv_set_timing(self._h, mask))

    def read_timing(self) -> dict:
        ms = (C.c_float * len(KERNEL_NAMES))()
        cnt = (C.c_int32 * len(KERNEL_NAMES))()
        self._check(self.lib.kv_read_timing(self._h, ms, cnt))
        return {n: (float(ms[i]), int(cnt[i])) for i, n in enumerate(KERNEL_NAMES)}

    def set_option(self, name: str, value: int):
        self._check(self.lib.kv_set_option(self._h, name.encode(), value))

    def close(self):
        if self._h:
            self.lib.kv_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
