"""CPU oracle for the decode attention operator -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  The product path (the HIP library and its Python binding) never
does, and this package never imports the product.

Three independent evaluators live here:

* :func:`decode_attention` -- the fp64 two-pass definition, in C (``lamina_oracle.c``),
  over the same bit patterns the GPU reads (paper Sec. 2.1 starred equation; GQA per
  Sec. 2.2.2).
* :mod:`oracle.naive` -- the partial-result definitions ``A_q(I)``, ``S_q(I)`` of
  Sec. 4.2.2 taken literally (no max shift, one output element at a time), pure Python.
* :mod:`oracle.splitmerge` -- partial results over arbitrary index sets and the
  divide-and-conquer combination of Sec. 4.2.2, in both the paper's ``A*S`` form and
  the log-sum-exp form.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lamina_oracle.c")
_LIB = os.path.join(_HERE, "liblamina_oracle.so")
_LIB_SANITIZED = os.path.join(_HERE, "liblamina_oracle_san.so")
# Set to 1 to make this package load the AddressSanitizer + UndefinedBehaviorSanitizer build of
# the C oracle.  The process must then have been started with the ASan runtime preloaded
# (see sanitizer_env); tests/test_oracle_sanitized.py runs the pin set that way.
SANITIZE_ENV = "LAMINA_ORACLE_SANITIZE"
_lib = None


class _Layout(ctypes.Structure):
    _fields_ = [
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("kv_is_fp8", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("block_table_stride", ctypes.c_int32),
        ("stride_req", ctypes.c_int64),
        ("stride_head", ctypes.c_int64),
        ("stride_tok", ctypes.c_int64),
        ("pool_stride_block", ctypes.c_int64),
        ("pool_stride_head", ctypes.c_int64),
        ("scale", ctypes.c_double),
    ]


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the C oracle with gcc (strict IEEE: no fast-math) and return the path.
    sanitize=True builds a second library with AddressSanitizer and
    UndefinedBehaviorSanitizer (any finding aborts), host code only."""
    lib = _LIB_SANITIZED if sanitize else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        flags = (["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                  "-fno-omit-frame-pointer"] if sanitize else ["-O2"])
        cmd = ["gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", lib, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return lib


def sanitizer_env() -> dict:
    """Environment for a child process that loads the sanitized oracle: the ASan runtime has to
    be in the process before anything else allocates, so it is preloaded (ahead of whatever is
    preloaded already); leak checking is off because the interpreter itself never frees
    everything."""
    env = dict(os.environ)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True,
                          capture_output=True, text=True).stdout.strip()
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env[SANITIZE_ENV] = "1"
    return env


def sanitized() -> bool:
    """True if this process runs the sanitizer build of the C oracle."""
    return os.environ.get(SANITIZE_ENV, "") == "1"


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build(sanitize=sanitized()))
        lib.oracle_decode_attention.restype = ctypes.c_int
        lib.oracle_decode_attention.argtypes = [
            ctypes.POINTER(_Layout), ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
            ctypes.c_void_p]
        lib.oracle_e4m3fn_decode.restype = ctypes.c_double
        lib.oracle_e4m3fn_decode.argtypes = [ctypes.c_uint8]
        lib.oracle_e4m3fn_encode.restype = ctypes.c_uint8
        lib.oracle_e4m3fn_encode.argtypes = [ctypes.c_double]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C oracle's OpenMP loop will use."""
    return int(_load().oracle_num_threads())


def e4m3fn_decode(byte: int) -> float:
    return float(_load().oracle_e4m3fn_decode(int(byte) & 0xFF))


def e4m3fn_encode(x: float) -> int:
    return int(_load().oracle_e4m3fn_encode(float(x)))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def decode_attention(q, k_cache, v_cache, seq_lens, *, num_kv_heads, scale,
                     block_table=None, block_size=0, k_scale=None, v_scale=None,
                     pairs=None):
    """fp64 two-pass decode attention over host tensors.

    q            torch bf16 [R][Hq][D]
    k_cache/v    contiguous mode: torch bf16 (or float8_e4m3fn / uint8) [R][Hkv][Lmax][D],
                 any strides with unit stride on D; paged mode (block_size > 0): pool
                 [num_blocks][Hkv][block_size][D]
    seq_lens     torch int32 [R]
    block_table  torch int32 [R][stride] (paged only)
    k_scale/v    torch fp32 [R][Hkv] (fp8 only)
    pairs        optional int array [[r, h], ...]: evaluate only those rows
    Returns (out float64 [rows][D], lse float64 [rows]); rows = all R*Hq in order when
    pairs is None (then reshaped to [R][Hq][D] and [R][Hq]).
    """
    lib = _load()
    assert q.dtype == torch.bfloat16 and q.is_contiguous() and q.dim() == 3
    R, Hq, D = q.shape
    fp8 = k_cache.dtype in (torch.float8_e4m3fn, torch.uint8)
    assert fp8 or k_cache.dtype == torch.bfloat16
    assert v_cache.dtype == k_cache.dtype and v_cache.shape == k_cache.shape
    assert all(a == b for a, b, n in zip(v_cache.stride(), k_cache.stride(), k_cache.shape)
               if n > 1), "K and V must share one layout"
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and k_cache.shape[3] == D
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous()
    L = _Layout()
    L.num_q_heads, L.num_kv_heads, L.head_dim = Hq, int(num_kv_heads), D
    L.kv_is_fp8 = 1 if fp8 else 0
    L.block_size = int(block_size)
    L.scale = float(scale)
    if block_size:
        assert block_table is not None and block_table.dtype == torch.int32
        assert block_table.dim() == 2 and block_table.stride(1) == 1
        assert k_cache.shape[2] == block_size and k_cache.stride(2) == D
        L.block_table_stride = block_table.stride(0)
        L.pool_stride_block, L.pool_stride_head = k_cache.stride(0), k_cache.stride(1)
    else:
        L.stride_req, L.stride_head, L.stride_tok = (k_cache.stride(0), k_cache.stride(1),
                                                     k_cache.stride(2))
    if fp8:
        assert k_scale.dtype == torch.float32 and k_scale.is_contiguous()
        assert v_scale.dtype == torch.float32 and v_scale.is_contiguous()
    if pairs is not None:
        pairs_np = np.ascontiguousarray(np.asarray(pairs, dtype=np.int32).reshape(-1, 2))
        n = pairs_np.shape[0]
        pairs_ptr = ctypes.c_void_p(pairs_np.ctypes.data)
    else:
        n = R * Hq
        pairs_ptr = ctypes.c_void_p(0)
    out = np.empty((n, D), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = lib.oracle_decode_attention(
        ctypes.byref(L), R, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens),
        _ptr(block_table), _ptr(k_scale), _ptr(v_scale), pairs_ptr, n,
        ctypes.c_void_p(out.ctypes.data), ctypes.c_void_p(lse.ctypes.data))
    if rc != 0:
        raise ValueError("oracle_decode_attention rejected its arguments")
    if pairs is None:
        return out.reshape(R, Hq, D), lse.reshape(R, Hq)
    return out, lse
