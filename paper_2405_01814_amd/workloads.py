"""Seeded synthetic decode-attention batches.

This module only draws random numbers and lays tensors out in memory; it holds none of
the operator's arithmetic.  It serves the GPU library's tests, the CPU oracle's tests
and the benchmark alike, and imports neither of them.

The five named workloads stand in for the serving workloads of the paper's evaluation
(Sec. 6: production traces that carry sequence lengths only, replayed with dummy
tokens; Table "Notations": batch 1..1024, sequence length 128..32768; the fixed
4096-token contexts of the latency-breakdown experiment).  Only the shapes and the
length mix matter to a bandwidth-bound operator, so values are i.i.d. N(0,1) rounded
to the storage type, which makes the scaled scores ~N(0,1): a flat softmax with no
sparsity to exploit.

Storage-type conversions use PyTorch CPU casts (round-to-nearest-even), a library
routine that belongs to neither side of the parity check.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

BASE_SEED = 240501814
HEAD_DIM = 128
BF16_NAN_BITS = 0x7FC0
FP8_NAN_BITS = 0x7F


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int                  # 1..5, selects the seed
    batch: int                  # R
    num_q_heads: int            # Hq
    num_kv_heads: int           # Hkv
    len_recipe: tuple           # ("uniform", lo, hi) | ("fixed", n) | ("lognormal", median, sigma, lo, hi)
    kv_dtype: str = "bf16"      # "bf16" | "fp8"
    block_size: int = 0         # 0 contiguous, 16 paged
    num_splits: int = 0         # 0 = library default
    head_dim: int = HEAD_DIM

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


WORKLOADS = {
    "tiny": Workload("tiny", 1, 4, 8, 2, ("uniform", 16, 256)),
    "llama3_8b_ctx4096": Workload("llama3_8b_ctx4096", 2, 64, 32, 8, ("fixed", 4096)),
    "llama3_70b_headshare_paged": Workload(
        "llama3_70b_headshare_paged", 3, 256, 8, 1,
        ("lognormal", 2048, 1.0, 128, 32768), block_size=16),
    "longctx_split64": Workload("longctx_split64", 4, 16, 32, 8, ("fixed", 131072),
                                num_splits=64),
    "fp8_paged": Workload("fp8_paged", 5, 128, 64, 8, ("uniform", 1024, 16384),
                          kv_dtype="fp8", block_size=16),
    # Multi-head attention (G = 1) shapes of the paper's other two evaluation models
    # (Table "Large language models used for evaluation": LLaMA-65B d = 8192, LLaMA-33B
    # d = 6656, both G = 1), as one attention device's head-level share (Sec. 5).
    "llama_65b_mha_ctx4096": Workload("llama_65b_mha_ctx4096", 6, 64, 8, 8, ("fixed", 4096)),
    "llama_33b_mha_paged": Workload("llama_33b_mha_paged", 7, 256, 13, 13,
                                    ("lognormal", 1024, 0.8, 128, 16384), block_size=16),
}


def draw_lens(w: Workload, batch: int | None = None) -> np.ndarray:
    """Context lengths (tokens attended, current token included), int32 [R]."""
    R = w.batch if batch is None else batch
    rng = np.random.default_rng(np.random.SeedSequence([w.seed, 0]))
    kind = w.len_recipe[0]
    if kind == "fixed":
        lens = np.full(R, w.len_recipe[1])
    elif kind == "uniform":
        lens = rng.integers(w.len_recipe[1], w.len_recipe[2] + 1, size=R)
    elif kind == "lognormal":
        _, median, sigma, lo, hi = w.len_recipe
        lens = np.clip(np.rint(np.exp(rng.normal(math.log(median), sigma, size=R))), lo, hi)
    else:
        raise ValueError(kind)
    return lens.astype(np.int32)


def _normal(seed, stream, r, shape):
    rng = np.random.default_rng(np.random.SeedSequence([seed, stream, r]))
    return torch.from_numpy(rng.standard_normal(shape, dtype=np.float32))


def _store(x, kv_dtype, scale_rg=None):
    """float32 [Hkv][n][D] -> storage dtype; fp8 divides by the per-head scale first."""
    if kv_dtype == "bf16":
        return x.to(torch.bfloat16)
    y = (x / scale_rg.view(-1, 1, 1)).clamp_(-448.0, 448.0)
    return y.to(torch.float8_e4m3fn)


def generate(w: Workload, lens: np.ndarray | None = None, threads: int = 8,
             pool_spare: float = 0.10, poison: bool = True) -> dict:
    """Build one batch on the host.  Returns a dict of torch CPU tensors:

    q [R][Hq][D] bf16; seq_lens [R] int32;
    contiguous: k, v [R][Hkv][Lmax][D] (rows >= len poisoned with NaN);
    paged: k, v pools [num_blocks][Hkv][16][D], block_table [R][max_blocks] int32
           (-1 beyond ceil(len/16)); spare blocks and last-block tails poisoned;
    fp8: k_scale, v_scale [R][Hkv] fp32, dequantised value = decode(byte) * scale.
    """
    lens = draw_lens(w) if lens is None else np.asarray(lens, dtype=np.int32)
    R, Hq, Hkv, D = len(lens), w.num_q_heads, w.num_kv_heads, w.head_dim
    seed = w.seed
    fp8 = w.kv_dtype == "fp8"
    st_dtype = torch.float8_e4m3fn if fp8 else torch.bfloat16
    nan_bits = FP8_NAN_BITS if fp8 else BF16_NAN_BITS
    int_view = torch.uint8 if fp8 else torch.int16

    q = torch.stack([_normal(seed, 1, r, (Hq, D)) for r in range(R)]).to(torch.bfloat16)
    out = {"q": q, "seq_lens": torch.from_numpy(lens.copy()), "workload": w,
           "max_seq_len": int(lens.max()) if R else 0}
    if fp8:
        rng = np.random.default_rng(np.random.SeedSequence([seed, 4]))
        lo, hi = math.log(1.0 / 32.0), math.log(1.0 / 8.0)
        out["k_scale"] = torch.from_numpy(np.exp(rng.uniform(lo, hi, (R, Hkv))).astype(np.float32))
        out["v_scale"] = torch.from_numpy(np.exp(rng.uniform(lo, hi, (R, Hkv))).astype(np.float32))

    def fresh(shape):
        t = torch.empty(shape, dtype=st_dtype)
        if poison:
            t.view(int_view).fill_(nan_bits)
        else:
            t.view(int_view).zero_()
        return t

    if w.block_size == 0:
        Lmax = max(int(lens.max()), 1) if R else 1
        k, v = fresh((R, Hkv, Lmax, D)), fresh((R, Hkv, Lmax, D))

        def fill(r):
            n = int(lens[r])
            if n == 0:
                return
            ks = out["k_scale"][r] if fp8 else None
            vs = out["v_scale"][r] if fp8 else None
            k[r, :, :n] = _store(_normal(seed, 2, r, (Hkv, n, D)), w.kv_dtype, ks)
            v[r, :, :n] = _store(_normal(seed, 3, r, (Hkv, n, D)), w.kv_dtype, vs)
    else:
        bs = w.block_size
        nblk = (lens.astype(np.int64) + bs - 1) // bs
        used = int(nblk.sum())
        total = used + max(int(math.ceil(used * pool_spare)), 1)
        rng = np.random.default_rng(np.random.SeedSequence([seed, 5]))
        ids = rng.permutation(total)[:used].astype(np.int32)
        starts = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
        max_blocks = max(int(nblk.max()), 1) if R else 1
        bt = np.full((R, max_blocks), -1, dtype=np.int32)
        for r in range(R):
            bt[r, :nblk[r]] = ids[starts[r]:starts[r + 1]]
        out["block_table"] = torch.from_numpy(bt)
        k, v = fresh((total, Hkv, bs, D)), fresh((total, Hkv, bs, D))

        def fill(r):
            n, nb = int(lens[r]), int(nblk[r])
            if n == 0:
                return
            ks = out["k_scale"][r] if fp8 else None
            vs = out["v_scale"][r] if fp8 else None
            blocks = torch.from_numpy(ids[starts[r]:starts[r + 1]].astype(np.int64))
            for dst, stream, sc in ((k, 2, ks), (v, 3, vs)):
                x = _store(_normal(seed, stream, r, (Hkv, n, D)), w.kv_dtype, sc)
                padded = fresh((Hkv, nb * bs, D))
                padded[:, :n] = x
                # [Hkv][nb][bs][D] -> [nb][Hkv][bs][D]
                dst[blocks] = padded.view(Hkv, nb, bs, D).transpose(0, 1).contiguous()

    if threads > 1 and R > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(R)))
    else:
        for r in range(R):
            fill(r)
    out["k"], out["v"] = k, v
    return out


def algorithmic_bytes(w: Workload, lens, out_bytes: int = 4, split_tokens: int = 0,
                      with_lse: bool = True, partial_results: int | None = None) -> dict:
    """Bytes one call must move if every needed byte is touched exactly once.

    KV: every attended (token, kv head) is one K row and one V row of D elements, read
    once and shared by the G query heads of its group -- per token and layer that is
    the 2*e*(d/G) of the paper's capacity example (Sec. 2.2.2) for one layer.  The rest
    is the per-call operator I/O of Sec. 3.1 (q in, output out) plus the small index
    arrays, and for split-KV the partial results (one per query head and piece, D + 1
    fp32 each) of every row that is cut, written once and read once: either counted from
    fixed partitions of split_tokens tokens, or given directly as partial_results.
    """
    lens = np.asarray(lens, dtype=np.int64)
    R, Hq, Hkv, D = len(lens), w.num_q_heads, w.num_kv_heads, w.head_dim
    e_kv = 1 if w.kv_dtype == "fp8" else 2
    kv = int(lens.sum()) * Hkv * 2 * D * e_kv
    q = R * Hq * D * 2
    o = R * Hq * D * out_bytes
    lse = R * Hq * 4 if with_lse else 0
    idx = R * 4
    if w.block_size:
        idx += int(((lens + w.block_size - 1) // w.block_size).sum()) * 4
    scales = 2 * R * Hkv * 4 if w.kv_dtype == "fp8" else 0
    partials = 0
    if partial_results is not None:
        partials = 2 * int(partial_results) * (D + 1) * 4
    elif split_tokens > 0:
        parts = (lens + split_tokens - 1) // split_tokens
        partials = 2 * int(parts[parts > 1].sum()) * Hq * (D + 1) * 4
    total = kv + q + o + lse + idx + scales + partials
    return {"kv": kv, "q": q, "out": o, "lse": lse, "index": idx, "scales": scales,
            "partials": partials, "total": total,
            "tokens": int(lens.sum()), "head_tokens": int(lens.sum()) * Hkv}
