"""The C-ABI library loads, exports every function include/kvx.h declares, and rejects bad
configurations before touching the GPU (these run without one)."""
import ctypes as C
import os
import re

import pytest

import paper_2601_01204_amd as kvx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "kvx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kv_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = kvx.load_library()
    names = _declared_functions()
    assert {"kv_init", "kv_step", "kv_step_frames", "kv_step_static", "kv_set_stream_tokens", "kv_step_batched", "kv_stats", "kv_export", "kv_reset", "kv_destroy",
            "kv_last_error", "kv_set_timing", "kv_read_timing", "kv_set_option", "kv_import", "kv_probe_mfma_bf16",
            "kv_probe_copy"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in kvx.h but not exported by libkvx.so"


def _cfg(**kw):
    base = dict(n_streams=1, n_layers=1, n_heads=4, head_dim=64, tokens_per_frame=69, n_special=5, pool_group=16,
                budget_tokens=256, k_bits=4, k_group=64, v_bits=4, v_group=64, in_dtype=kvx.KV_BF16,
                out_dtype=kvx.KV_BF16, mode=kvx.KV_COMPRESSED, max_frames=0, softmax_scale=0.0, meta_format=0, max_frames_per_step=1, order=0, layout=0)
    base.update(kw)
    c = kvx.KvConfig()
    for k, v in base.items():
        setattr(c, k, v)
    return c


@pytest.mark.parametrize("bad,code", [
    (dict(budget_tokens=137), -1),          # below two frames: first and current frame could not both stay
    (dict(k_bits=3), -1),
    (dict(v_bits=16), -1),
    (dict(k_group=48), -1),
    (dict(v_group=16), -1),
    (dict(head_dim=128), -1),
    (dict(n_heads=0), -1),
    (dict(n_heads=65), -1),
    (dict(n_special=70), -1),
    (dict(pool_group=0), -1),
    (dict(in_dtype=7), -1),
    (dict(out_dtype=-1), -1),
    (dict(mode=5), -1),
    (dict(mode=kvx.KV_UNCOMPRESSED_BF16, max_frames=0), -1),
    (dict(softmax_scale=-1.0), -1),
    (dict(n_streams=0), -1),
    (dict(budget_tokens=40000), -3),
    (dict(meta_format=2), -1),
    (dict(order=2), -1),
    (dict(layout=2), -1),
    (dict(layout=1, mode=kvx.KV_UNCOMPRESSED_BF16, max_frames=4), -1),
    (dict(max_frames_per_step=-1), -1),
    (dict(max_frames_per_step=3, budget_tokens=4 * 69 - 1), -1),   # first frame + a full chunk must fit the budget
    (dict(max_frames_per_step=2, order=1), -1),
    (dict(meta_format=1, k_bits=8), -1),          # 16-bit metadata: 2- or 4-bit keys
    (dict(meta_format=1, in_dtype=kvx.KV_F32), -1),
])
def test_bad_configurations_are_rejected_with_a_message(bad, code):
    lib = kvx.load_library()
    h = C.c_void_p()
    cfg = _cfg(**bad)
    rc = lib.kv_init(C.byref(cfg), C.byref(h))
    assert rc == code
    assert not h.value
    assert len(lib.kv_last_error(None)) > 10


def test_null_arguments():
    lib = kvx.load_library()
    h = C.c_void_p()
    assert lib.kv_init(None, C.byref(h)) == -1
    assert lib.kv_init(C.byref(_cfg()), None) == -1
    lib.kv_destroy(None)                      # allowed
    assert lib.kv_stats(None, None) == -1
    assert lib.kv_reset(None, 0, 0) == -1
    assert lib.kv_import(None, 0, 0, None) == -1
    assert lib.kv_step(None, 0, 0, None, None, None, 64, 64, None, None) == -1


def test_config_struct_matches_header():
    """Field order of the ctypes struct follows the header (a mismatch would shift every field)."""
    text = open(os.path.join(ROOT, "include", "kvx.h")).read()
    body = re.search(r"typedef struct kv_config \{(.*?)\} kv_config;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|float)\s+(\w+);", body)
    assert fields == [n for n, _ in kvx.KvConfig._fields_]
    body = re.search(r"typedef struct kv_stats_t \{(.*?)\} kv_stats_t;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|int64_t)\s+(\w+);", body)
    assert fields == [n for n, _ in kvx.KvStats._fields_]
