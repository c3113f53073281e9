"""The C-ABI library loads, exports what the header declares, and validates configurations
without touching a GPU.  CPU only (no compute calls)."""
import ctypes
import os
import re

import pytest

from paper_2405_01814_amd import lamina

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(lamina_\w+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = lamina.load()
    names = header_functions()
    assert set(names) == set(lamina.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_binding_struct_layouts_match_the_header():
    # field order and types as declared; sizes as a C compiler lays them out
    assert ctypes.sizeof(lamina.lamina_attn_config) == 11 * 4
    assert ctypes.sizeof(lamina.lamina_call_params) == 8 + 5 * 8 + 8 + 3 * 8
    assert lamina.lamina_call_params.kv_stride_req.offset == 8
    assert lamina.lamina_call_params.k_scale.offset == 56


def good_cfg(**kw):
    c = lamina.lamina_attn_config(32, 8, 128, lamina.LAMINA_BF16, lamina.LAMINA_F32, 0,
                                  64, 4096, 0, 0.0, 0)
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_workspace_query_follows_the_partitioning():
    assert lamina.lamina_attn_workspace_bytes(good_cfg(num_splits=1)) == 0
    assert lamina.lamina_attn_workspace_bytes(good_cfg(num_splits=8)) == 64 * 32 * 8 * 129 * 4 + 272
    c = good_cfg(max_batch=16, max_seq_len=131072, num_splits=64)
    assert lamina.lamina_attn_workspace_bytes(c) == 16 * 32 * 64 * 129 * 4 + 80
    # balanced shares: two pieces per work-group of the largest grid plus a 16-byte record each
    c = good_cfg(max_batch=64, max_seq_len=8192, num_splits=0)
    assert lamina.lamina_attn_workspace_bytes(c) == 2048 * 4 * 129 * 4 + 1024 * 16
    assert lamina.lamina_attn_workspace_bytes(good_cfg(head_dim=64)) == 0      # invalid cfg


@pytest.mark.parametrize("field,value,code", [
    ("num_q_heads", 0, lamina.LAMINA_ERR_INVALID_ARG),
    ("num_q_heads", 30, lamina.LAMINA_ERR_INVALID_ARG),          # not a multiple of 8
    ("max_batch", 0, lamina.LAMINA_ERR_INVALID_ARG),
    ("max_seq_len", -1, lamina.LAMINA_ERR_INVALID_ARG),
    ("kv_dtype", 7, lamina.LAMINA_ERR_INVALID_ARG),
    ("out_dtype", lamina.LAMINA_FP8_E4M3, lamina.LAMINA_ERR_INVALID_ARG),
    ("num_splits", -2, lamina.LAMINA_ERR_INVALID_ARG),
    ("softmax_scale", float("nan"), lamina.LAMINA_ERR_INVALID_ARG),
    ("head_dim", 64, lamina.LAMINA_ERR_UNSUPPORTED),
    ("block_size", 32, lamina.LAMINA_ERR_UNSUPPORTED),
    ("num_kv_heads", 1, lamina.LAMINA_ERR_UNSUPPORTED),           # group size 32
])
def test_create_rejects_bad_configs_before_any_gpu_work(field, value, code):
    rc, h = lamina.lamina_attn_create(good_cfg(**{field: value}))
    assert rc == code and not h.value
    assert lamina.lamina_attn_last_error(None) != ""


def test_null_arguments_are_errors_not_crashes():
    lib = lamina.load()
    assert lib.lamina_attn_create(None, None) == lamina.LAMINA_ERR_INVALID_ARG
    h = ctypes.c_void_p()
    assert lib.lamina_attn_create(None, ctypes.byref(h)) == lamina.LAMINA_ERR_INVALID_ARG
    assert lib.lamina_attn_destroy(None) == lamina.LAMINA_OK
    assert lib.lamina_decode_attention(None, None, None, None, None, None, None, None,
                                       None) == lamina.LAMINA_ERR_INVALID_ARG
    assert lib.lamina_attn_num_splits(None) == 0
