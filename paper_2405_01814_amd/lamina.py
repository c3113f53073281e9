"""ctypes binding over the C ABI of ``include/lamina_attn.h``.

Argument marshalling only: every step of the operator runs in the HIP kernels of
``liblamina_attn.so``.  PyTorch appears only as the owner of device memory and streams.
There is no CPU fallback: if the library is missing and cannot be built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SRCS = [os.path.join(_HERE, "csrc", "lamina_attn.hip"),
         os.path.join(_HERE, "csrc", "lamina_seqno.hip"),
         os.path.join(_HERE, "csrc", "lamina_probe.hip")]
_INC = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_HERE, "liblamina_attn.so")

LAMINA_OK = 0
LAMINA_ERR_INVALID_ARG = -1
LAMINA_ERR_UNSUPPORTED = -2
LAMINA_ERR_HIP = -3
LAMINA_ERR_WORKSPACE = -4
LAMINA_BF16, LAMINA_FP8_E4M3, LAMINA_F32 = 0, 1, 2
LAMINA_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ("lamina_attn_create", "lamina_decode_attention", "lamina_attn_destroy",
           "lamina_attn_last_error", "lamina_attn_workspace_bytes", "lamina_attn_num_splits",
           "lamina_attn_split_tokens", "lamina_attn_count_partials", "lamina_append_kv",
           "lamina_fold_new_token", "lamina_fold_new_token_and_append",
           "lamina_decode_attention_static",
           "lamina_seqno_alloc", "lamina_seqno_free", "lamina_seqno_wait", "lamina_seqno_signal",
           "lamina_probe_stream_read", "lamina_probe_valu_attention")

LAMINA_SEQNO_REACHED = 0
LAMINA_SEQNO_TIMED_OUT = 1

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


class lamina_attn_config(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
                ("out_dtype", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("max_batch", ctypes.c_int32), ("max_seq_len", ctypes.c_int32),
                ("num_splits", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("device", ctypes.c_int32)]


class lamina_call_params(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32),
                ("kv_stride_req", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
                ("kv_stride_tok", ctypes.c_int64),
                ("pool_stride_block", ctypes.c_int64), ("pool_stride_head", ctypes.c_int64),
                ("block_table_stride", ctypes.c_int32),
                ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
                ("stream", ctypes.c_void_p)]


TRACE_LIB_PATH = os.path.join(_HERE, "liblamina_attn_trace.so")
HOSTSAN_LIB_PATH = os.path.join(_HERE, "liblamina_attn_hostsan.so")
HOSTSAN_ENV = "LAMINA_HOST_SANITIZE"
# AddressSanitizer + UBSan on the HOST half of the library only (argument checks, planning,
# launch set-up); the device code is compiled as always.
HOSTSAN_FLAGS = ["-Xarch_host", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                 "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]


def build_library(verbose: bool = False, trace: bool = False, host_sanitize: bool = False) -> str:
    """Compile the HIP library for gfx950 in-tree with hipcc; returns its path.  trace=True builds
    the timeline variant (-DLAMINA_TRACE: the kernels stamp the device clock at a few points and
    lamina_trace_read returns the stamps) next to the ordinary one; only `bench.py --timeline`
    uses it.  host_sanitize=True builds a variant whose host code runs under ASan + UBSan (its
    process must preload the sanitizer runtime, see host_sanitizer_env); only tests use it."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    out = HOSTSAN_LIB_PATH if host_sanitize else (TRACE_LIB_PATH if trace else LIB_PATH)
    cmd = [hipcc, *HIPCC_FLAGS, *(HOSTSAN_FLAGS if host_sanitize else []),
           *(["-DLAMINA_TRACE"] if trace else []), "-I", _INC, "-o", out, *_SRCS]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return out


_lib = None


def library_is_stale() -> bool:
    """True if no built library exists or a source or header it is built from is newer."""
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    csrc = os.path.join(_HERE, "csrc")
    deps = list(_SRCS) + [os.path.join(d, f) for d in (_INC, csrc) for f in sorted(os.listdir(d))
                          if f.endswith(".h")]
    return any(os.path.getmtime(d) > built for d in deps)


def host_sanitized() -> bool:
    """True if this process is to run the host-sanitized build of the library."""
    return os.environ.get(HOSTSAN_ENV, "") == "1"


def host_sanitizer_env() -> dict:
    """Environment for a child process that loads the host-sanitized library: the compiler's ASan
    runtime (which also carries the UBSan handlers) has to be in the process first, so it is
    preloaded ahead of whatever is preloaded already; leak checking is off because neither the
    interpreter nor the GPU runtime free everything at exit."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    rt = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], check=True,
                        capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        raise RuntimeError("the compiler's AddressSanitizer runtime was not found: " + rt)
    env = dict(os.environ)
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:protect_shadow_gap=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env[HOSTSAN_ENV] = "1"
    return env


def use_trace_library() -> None:
    """Make this process load the timeline build instead of the ordinary library (must be called
    before the first load()); builds it if it is missing or older than its sources."""
    global LIB_PATH
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    LIB_PATH = TRACE_LIB_PATH
    if library_is_stale():
        build_library(trace=True)


def lamina_trace_read(words: int):
    """Timeline build only: the device-side stamp array as a numpy uint64 vector."""
    import numpy as np
    lib = load()
    buf = np.zeros(words, dtype=np.uint64)
    lib.lamina_trace_read.restype = ctypes.c_int
    lib.lamina_trace_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    rc = lib.lamina_trace_read(buf.ctypes.data, words)
    if rc != 0:
        raise RuntimeError(f"lamina_trace_read: hip error {rc}")
    return buf


def load():
    """Load the built library, building it first if it is missing or older than any of its
    sources or headers (an edited kernel must never be tested through an old binary)."""
    global _lib, LIB_PATH
    if _lib is not None:
        return _lib
    if host_sanitized() and LIB_PATH != HOSTSAN_LIB_PATH:
        LIB_PATH = HOSTSAN_LIB_PATH
    if library_is_stale():
        build_library(trace=LIB_PATH == TRACE_LIB_PATH, host_sanitize=LIB_PATH == HOSTSAN_LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp = ctypes.c_void_p
    lib.lamina_attn_create.restype = ctypes.c_int
    lib.lamina_attn_create.argtypes = [ctypes.POINTER(lamina_attn_config), ctypes.POINTER(vp)]
    lib.lamina_decode_attention.restype = ctypes.c_int
    lib.lamina_decode_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp,
                                            ctypes.POINTER(lamina_call_params)]
    lib.lamina_attn_destroy.restype = ctypes.c_int
    lib.lamina_attn_destroy.argtypes = [vp]
    lib.lamina_attn_last_error.restype = ctypes.c_char_p
    lib.lamina_attn_last_error.argtypes = [vp]
    lib.lamina_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.lamina_attn_workspace_bytes.argtypes = [ctypes.POINTER(lamina_attn_config)]
    lib.lamina_attn_num_splits.restype = ctypes.c_int
    lib.lamina_attn_num_splits.argtypes = [vp]
    lib.lamina_attn_split_tokens.restype = ctypes.c_int
    lib.lamina_attn_split_tokens.argtypes = [vp]
    lib.lamina_attn_count_partials.restype = ctypes.c_int64
    lib.lamina_attn_count_partials.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32]
    lib.lamina_append_kv.restype = ctypes.c_int
    lib.lamina_append_kv.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(lamina_call_params)]
    u64p, i32p = ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_int32)
    lib.lamina_seqno_alloc.restype = ctypes.c_int
    lib.lamina_seqno_alloc.argtypes = [ctypes.POINTER(u64p), ctypes.POINTER(i32p)]
    lib.lamina_seqno_free.restype = ctypes.c_int
    lib.lamina_seqno_free.argtypes = [u64p, i32p]
    lib.lamina_seqno_wait.restype = ctypes.c_int
    lib.lamina_seqno_wait.argtypes = [u64p, ctypes.c_uint64, ctypes.c_uint32, i32p, vp]
    lib.lamina_seqno_signal.restype = ctypes.c_int
    lib.lamina_seqno_signal.argtypes = [u64p, ctypes.c_uint64, vp]
    lib.lamina_fold_new_token.restype = ctypes.c_int
    lib.lamina_fold_new_token.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp,
                                          ctypes.POINTER(lamina_call_params)]
    lib.lamina_fold_new_token_and_append.restype = ctypes.c_int
    lib.lamina_fold_new_token_and_append.argtypes = [vp] * 12 + [ctypes.POINTER(lamina_call_params)]
    lib.lamina_decode_attention_static.restype = ctypes.c_int
    lib.lamina_decode_attention_static.argtypes = [ctypes.POINTER(lamina_attn_config), vp, vp, vp,
                                                   vp, vp, vp, vp,
                                                   ctypes.POINTER(lamina_call_params)]
    lib.lamina_probe_stream_read.restype = ctypes.c_int
    lib.lamina_probe_stream_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp]
    lib.lamina_probe_valu_attention.restype = ctypes.c_int
    lib.lamina_probe_valu_attention.argtypes = [vp] * 6 + [ctypes.c_int] * 4 + [ctypes.c_int64] * 3 + [
        ctypes.c_float, ctypes.c_int, vp]
    _lib = lib
    return lib


class LaminaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"lamina error {code}: {msg}")
        self.code = code


# ---- same names as the C ABI -------------------------------------------------------------

def lamina_attn_create(cfg: lamina_attn_config):
    """Returns (status, handle).  handle is a c_void_p (None-valued on failure)."""
    h = ctypes.c_void_p()
    rc = load().lamina_attn_create(ctypes.byref(cfg), ctypes.byref(h))
    return rc, h


def lamina_decode_attention(h, q, k_cache, v_cache, seq_lens, block_table, out, lse,
                            params: lamina_call_params) -> int:
    """Pointers are integers (device addresses) or None."""
    return load().lamina_decode_attention(h, q, k_cache, v_cache, seq_lens, block_table, out,
                                          lse, ctypes.byref(params) if params is not None else None)


def lamina_decode_attention_static(cfg: lamina_attn_config, q, k_cache, v_cache, seq_lens,
                                   block_table, out, lse, params: lamina_call_params) -> int:
    """The call that allocates nothing: cfg in place of a handle, partial results in the
    library's static scratch area.  Pointers are integers (device addresses) or None."""
    return load().lamina_decode_attention_static(
        ctypes.byref(cfg) if cfg is not None else None, q, k_cache, v_cache, seq_lens,
        block_table, out, lse, ctypes.byref(params) if params is not None else None)


def lamina_append_kv(h, k_new, v_new, k_cache, v_cache, positions, block_table,
                     params: lamina_call_params) -> int:
    return load().lamina_append_kv(h, k_new, v_new, k_cache, v_cache, positions, block_table,
                                   ctypes.byref(params) if params is not None else None)


def lamina_fold_new_token(h, q, k_new, v_new, out_prev, lse_prev, out, lse,
                          params: lamina_call_params) -> int:
    return load().lamina_fold_new_token(h, q, k_new, v_new, out_prev, lse_prev, out, lse,
                                        ctypes.byref(params) if params is not None else None)


def lamina_fold_new_token_and_append(h, q, k_new, v_new, out_prev, lse_prev, out, lse, k_cache,
                                     v_cache, positions, block_table,
                                     params: lamina_call_params) -> int:
    return load().lamina_fold_new_token_and_append(
        h, q, k_new, v_new, out_prev, lse_prev, out, lse, k_cache, v_cache, positions,
        block_table, ctypes.byref(params) if params is not None else None)


def lamina_attn_destroy(h) -> int:
    return load().lamina_attn_destroy(h)


def lamina_attn_last_error(h=None) -> str:
    s = load().lamina_attn_last_error(h)
    return s.decode() if s else ""


def lamina_attn_workspace_bytes(cfg: lamina_attn_config) -> int:
    return int(load().lamina_attn_workspace_bytes(ctypes.byref(cfg)))


# ---- convenience wrapper over torch tensors ---------------------------------------------

def lamina_seqno_alloc():
    """Returns (status, seqno pointer, status-word pointer); both ctypes pointers into pinned memory."""
    sq, st = ctypes.POINTER(ctypes.c_uint64)(), ctypes.POINTER(ctypes.c_int32)()
    rc = load().lamina_seqno_alloc(ctypes.byref(sq), ctypes.byref(st))
    return rc, sq, st


def lamina_seqno_free(seqno, status=None) -> int:
    return load().lamina_seqno_free(seqno, status)


def lamina_seqno_wait(seqno, target: int, timeout_us: int, status, stream) -> int:
    return load().lamina_seqno_wait(seqno, target, timeout_us, status, stream)


def lamina_seqno_signal(seqno, value: int, stream) -> int:
    return load().lamina_seqno_signal(seqno, value, stream)


def lamina_probe_stream_read(buf, nbytes: int, nontemporal: bool, work_groups: int, sink,
                             stream) -> int:
    """Read-only streaming pass over nbytes of device memory at address buf (integers)."""
    return load().lamina_probe_stream_read(buf, nbytes, 1 if nontemporal else 0, work_groups,
                                           sink, stream)


def lamina_probe_valu_attention(q, k_cache, v_cache, seq_lens, out, lse, batch: int,
                                num_q_heads: int, num_kv_heads: int, max_seq_len: int,
                                kv_stride_req: int, kv_stride_head: int, kv_stride_tok: int,
                                softmax_scale: float, work_groups: int, stream) -> int:
    """The operator on the vector ALU only (measurement aid); pointers are integers."""
    return load().lamina_probe_valu_attention(q, k_cache, v_cache, seq_lens, out, lse, batch,
                                              num_q_heads, num_kv_heads, max_seq_len,
                                              kv_stride_req, kv_stride_head, kv_stride_tok,
                                              softmax_scale, work_groups, stream)


def valu_attention(q, k_cache, v_cache, seq_lens, num_kv_heads: int, max_seq_len: int,
                   out=None, lse=None, stream=None, work_groups: int = 0):
    """Tensor-level wrapper of lamina_probe_valu_attention for bf16 contiguous caches
    [R][Hkv][L][128] (any strides that are multiples of 8 elements); returns (out, lse)."""
    import torch
    R, Hq, D = q.shape
    assert D == 128 and q.dtype == torch.bfloat16 and q.is_contiguous()
    assert k_cache.dtype == torch.bfloat16 and k_cache.stride() == v_cache.stride()
    assert k_cache.stride(3) == 1 and seq_lens.dtype == torch.int32
    if out is None:
        out = torch.empty((R, Hq, D), device=q.device, dtype=torch.float32)
    if lse is None:
        lse = torch.empty((R, Hq), device=q.device, dtype=torch.float32)
    st = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = lamina_probe_valu_attention(q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(),
                                     seq_lens.data_ptr(), out.data_ptr(), lse.data_ptr(), R, Hq,
                                     num_kv_heads, max_seq_len, k_cache.stride(0),
                                     k_cache.stride(1), k_cache.stride(2), 0.0, work_groups,
                                     st.cuda_stream)
    if rc != LAMINA_OK:
        raise LaminaError(rc, "lamina_probe_valu_attention")
    return out, lse


class Seqno:
    """A sequence number in pinned memory plus a status word for bounded waits (Sec. 4.1,
    device-side polling).  `value` / `status` read and write the words from the host."""

    def __init__(self):
        rc, self._seqno, self._status = lamina_seqno_alloc()
        if rc != LAMINA_OK:
            self._seqno = None
            raise LaminaError(rc, "lamina_seqno_alloc")

    @property
    def value(self) -> int:
        return int(self._seqno[0])

    @value.setter
    def value(self, v: int):
        self._seqno[0] = v                     # an aligned 64-bit store (x86: release ordering)

    @property
    def status(self) -> int:
        return int(self._status[0])

    def wait(self, target: int, timeout_us: int = 0, stream=None) -> None:
        """Enqueue a bounded wait for value >= target on `stream` (a torch stream or None)."""
        rc = lamina_seqno_wait(self._seqno, target, timeout_us, self._status, _stream_handle(stream))
        if rc != LAMINA_OK:
            raise LaminaError(rc, "lamina_seqno_wait")

    def signal(self, value: int, stream=None) -> None:
        rc = lamina_seqno_signal(self._seqno, value, _stream_handle(stream))
        if rc != LAMINA_OK:
            raise LaminaError(rc, "lamina_seqno_signal")

    def close(self):
        if getattr(self, "_seqno", None) is not None:
            lamina_seqno_free(self._seqno, self._status)
            self._seqno = None


def _stream_handle(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


_DTYPES = {"bf16": LAMINA_BF16, "fp8": LAMINA_FP8_E4M3, "f32": LAMINA_F32}


class DecodeAttention:
    """One handle = one attention layer-share.  Tensors are torch CUDA tensors."""

    def __init__(self, num_q_heads, num_kv_heads, max_batch, max_seq_len, *, kv_dtype="bf16",
                 out_dtype="f32", block_size=0, num_splits=0, softmax_scale=0.0, device=0,
                 head_dim=128):
        self.cfg = lamina_attn_config(num_q_heads, num_kv_heads, head_dim, _DTYPES[kv_dtype],
                                      _DTYPES[out_dtype], block_size, max_batch, max_seq_len,
                                      num_splits, softmax_scale, device)
        rc, self.handle = lamina_attn_create(self.cfg)
        if rc != LAMINA_OK:
            self.handle = None
            raise LaminaError(rc, lamina_attn_last_error(None))
        self.out_dtype = out_dtype
        self.num_splits = int(load().lamina_attn_num_splits(self.handle))
        self.split_tokens = int(load().lamina_attn_split_tokens(self.handle))

    def count_partials(self, seq_lens) -> int:
        """Per-head partial results a call with these (host) lengths writes and merges."""
        import numpy as np
        lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
        n = int(load().lamina_attn_count_partials(
            self.handle, lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), int(lens.size)))
        if n < 0:
            raise LaminaError(n, "lamina_attn_count_partials")
        return n

    def close(self):
        if getattr(self, "handle", None) is not None:
            lamina_attn_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def params_for(self, q, k_cache, block_table=None, k_scale=None, v_scale=None, stream=None):
        import torch
        p = lamina_call_params()
        p.batch = q.shape[0]
        if self.cfg.block_size:
            p.pool_stride_block, p.pool_stride_head = k_cache.stride(0), k_cache.stride(1)
            p.block_table_stride = block_table.stride(0)
        else:
            p.kv_stride_req, p.kv_stride_head, p.kv_stride_tok = (
                k_cache.stride(0), k_cache.stride(1), k_cache.stride(2))
        p.k_scale = k_scale.data_ptr() if k_scale is not None else None
        p.v_scale = v_scale.data_ptr() if v_scale is not None else None
        if stream is None:
            stream = torch.cuda.current_stream(q.device)
        p.stream = stream.cuda_stream or None
        return p

    def __call__(self, q, k_cache, v_cache, seq_lens, block_table=None, k_scale=None,
                 v_scale=None, out=None, lse=None, stream=None, want_lse=True):
        import torch
        R, Hq, D = q.shape
        if out is None:
            out = torch.empty((R, Hq, D), device=q.device,
                              dtype=torch.float32 if self.out_dtype == "f32" else torch.bfloat16)
        if lse is None and want_lse:
            lse = torch.empty((R, Hq), device=q.device, dtype=torch.float32)
        p = self.params_for(q, k_cache, block_table, k_scale, v_scale, stream)
        rc = lamina_decode_attention(
            self.handle, q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(),
            seq_lens.data_ptr(), block_table.data_ptr() if block_table is not None else None,
            out.data_ptr(), lse.data_ptr() if lse is not None else None, p)
        if rc != LAMINA_OK:
            raise LaminaError(rc, lamina_attn_last_error(self.handle))
        return out, lse

    def append_kv(self, k_new, v_new, k_cache, v_cache, positions, block_table=None,
                  k_scale=None, v_scale=None, stream=None):
        """Write the new token's rows (bf16 [R][Hkv][128]) into the cache at positions[r]."""
        p = self.params_for(k_new, k_cache, block_table, k_scale, v_scale, stream)
        rc = lamina_append_kv(self.handle, k_new.data_ptr(), v_new.data_ptr(), k_cache.data_ptr(),
                              v_cache.data_ptr(), positions.data_ptr(),
                              block_table.data_ptr() if block_table is not None else None, p)
        if rc != LAMINA_OK:
            raise LaminaError(rc, lamina_attn_last_error(self.handle))

    def fold_new_token(self, q, k_new, v_new, out_prev, lse_prev, out=None, lse=None,
                       k_scale=None, v_scale=None, stream=None):
        """Combine a result over the previous tokens with the single new token."""
        import torch
        R, Hq, D = q.shape
        if out is None:
            out = torch.empty((R, Hq, D), device=q.device,
                              dtype=torch.float32 if self.out_dtype == "f32" else torch.bfloat16)
        if lse is None:
            lse = torch.empty((R, Hq), device=q.device, dtype=torch.float32)
        p = lamina_call_params()
        p.batch = R
        p.k_scale = k_scale.data_ptr() if k_scale is not None else None
        p.v_scale = v_scale.data_ptr() if v_scale is not None else None
        if stream is None:
            stream = torch.cuda.current_stream(q.device)
        p.stream = stream.cuda_stream or None
        rc = lamina_fold_new_token(self.handle, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                   out_prev.data_ptr(), lse_prev.data_ptr(), out.data_ptr(),
                                   lse.data_ptr(), p)
        if rc != LAMINA_OK:
            raise LaminaError(rc, lamina_attn_last_error(self.handle))
        return out, lse

    def fold_new_token_and_append(self, q, k_new, v_new, out_prev, lse_prev, k_cache, v_cache,
                                  positions, block_table=None, out=None, lse=None, k_scale=None,
                                  v_scale=None, stream=None):
        """fold_new_token and append_kv in one launch."""
        import torch
        R, Hq, D = q.shape
        if out is None:
            out = torch.empty((R, Hq, D), device=q.device,
                              dtype=torch.float32 if self.out_dtype == "f32" else torch.bfloat16)
        if lse is None:
            lse = torch.empty((R, Hq), device=q.device, dtype=torch.float32)
        p = self.params_for(q, k_cache, block_table, k_scale, v_scale, stream)
        rc = lamina_fold_new_token_and_append(
            self.handle, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), out_prev.data_ptr(),
            lse_prev.data_ptr(), out.data_ptr(), lse.data_ptr(), k_cache.data_ptr(),
            v_cache.data_ptr(), positions.data_ptr(),
            block_table.data_ptr() if block_table is not None else None, p)
        if rc != LAMINA_OK:
            raise LaminaError(rc, lamina_attn_last_error(self.handle))
        return out, lse
