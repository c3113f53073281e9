"""Seeded sweep over shapes nobody picked by hand: every case draws its cache type, layout,
group size, number of kv heads, batch, length mix (with empty and one-token requests thrown
in), partitioning, handle capacity and output type from its seed, and is compared with the
fp64 oracle on every row, to the tolerances stated in test_gpu_parity.py."""
import dataclasses

import numpy as np
import pytest

from paper_2405_01814_amd import workloads as W
from test_gpu_parity import check, gpu_of, oracle_of

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(np.random.SeedSequence([20240501, seed]))
    kv = ["bf16", "fp8"][int(rng.integers(2))]
    paged = bool(rng.integers(2))
    G = int(rng.choice([1, 2, 4, 8, 16]))
    hkv = int(rng.choice([1, 2, 3, 8]))
    budget = 6_000_000 // (G * hkv)                       # tokens, so the oracle stays in seconds
    mix = ["lognormal", "uniform", "two_sizes", "short"][int(rng.integers(4))]
    R = int(rng.integers(1, 200 if mix == "short" else 48))
    if mix == "lognormal":
        lens = np.exp(rng.normal(np.log(700.0), 1.2, R))
    elif mix == "uniform":
        lens = rng.uniform(1, 6000, R)
    elif mix == "two_sizes":
        lens = np.where(rng.random(R) < 0.15, rng.uniform(8000, 20000, R), rng.uniform(1, 300, R))
    else:
        lens = rng.uniform(1, 140, R)
    lens = np.clip(np.round(lens), 1, 20000).astype(np.int64)
    lens[rng.random(R) < 0.08] = 0                        # empty requests
    lens[rng.random(R) < 0.05] = 1
    while lens.sum() > budget and lens.max() > 1:         # shrink the longest until it fits
        lens[np.argmax(lens)] //= 2
    splits = int(rng.choice([1, 0, 0, int(rng.integers(2, 70))]))
    slack = int(rng.choice([0, 0, 1, 777]))               # handle capacity beyond what the call uses
    out_dtype = ["f32", "f32", "bf16"][int(rng.integers(3))]
    return dict(kv=kv, paged=paged, G=G, hkv=hkv, lens=lens.astype(np.int32), splits=splits,
                slack=slack, out_dtype=out_dtype, seed=seed)


@pytest.mark.parametrize("seed", range(64))
def test_drawn_shape_matches_the_oracle(seed):
    c = draw_case(seed)
    print({k: (v if k != "lens" else f"{len(v)} requests, {int(v.sum())} tokens, max {int(v.max())}")
           for k, v in c.items()}, flush=True)
    base = W.WORKLOADS["fp8_paged" if c["kv"] == "fp8" else "llama3_8b_ctx4096"]
    w = dataclasses.replace(base, num_q_heads=c["G"] * c["hkv"], num_kv_heads=c["hkv"],
                            block_size=16 if c["paged"] else 0, index=1000 + seed)
    b = W.generate(w, lens=c["lens"])
    cap = max(int(c["lens"].max()), 1) + c["slack"]
    got, info = gpu_of(b, out_dtype=c["out_dtype"], num_splits=c["splits"], max_seq_len=cap,
                       max_batch=len(c["lens"]) + (c["slack"] > 0))
    if c["splits"] > 1:
        assert info[0] == c["splits"]
    kind = "fp8" if c["kv"] == "fp8" else ("bf16_bf16" if c["out_dtype"] == "bf16" else "bf16_f32")
    if kind == "fp8" and c["out_dtype"] == "bf16":
        out, lse = got
        ref_out, ref_lse = oracle_of(b)
        assert (np.abs(out - ref_out) <= 3e-2 + 1e-2 * np.abs(ref_out)).all()
        fin = np.isfinite(ref_lse)
        assert (lse[~fin] == ref_lse[~fin]).all() and np.abs(lse[fin] - ref_lse[fin]).max(initial=0) <= 5e-3
    else:
        check(got, oracle_of(b), kind)
    out, lse = got
    empty = c["lens"] == 0
    assert (out[empty] == 0).all() and np.isneginf(lse[empty]).all()
