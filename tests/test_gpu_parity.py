"""Parity of the HIP library (through its C ABI) with the fp64 CPU oracle, element by
element on the same seeded inputs.  Tolerances (stated with the target of this build):

* bf16 cache, fp32 accumulate, fp32 output: max |gpu - ref| <= 2e-3 over all elements and
  max |gpu - ref| / |ref| <= 1e-2 over elements with |ref| >= 1e-3;
* bf16 output: |gpu - ref| <= 2e-3 + 1e-2 |ref| (half an ulp of bf16 exceeds 2e-3 above 1);
* fp8 cache: max |gpu - ref| <= 3e-2 against the oracle on the same dequantised values;
* lse: 1e-3 absolute (5e-3 for fp8).
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2405_01814_amd import lamina, workloads as W

pytestmark = pytest.mark.gpu
SCALE = 1.0 / math.sqrt(128)


def dev():
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def oracle_of(b, pairs=None):
    w = b["workload"]
    return oracle.decode_attention(
        b["q"], b["k"], b["v"], b["seq_lens"], num_kv_heads=w.num_kv_heads, scale=SCALE,
        block_table=b.get("block_table"), block_size=w.block_size,
        k_scale=b.get("k_scale"), v_scale=b.get("v_scale"), pairs=pairs)


def gpu_of(b, out_dtype="f32", num_splits=None, max_seq_len=None, max_batch=None, reps=1):
    w = b["workload"]
    d = dev()
    R = b["q"].shape[0]
    op = lamina.DecodeAttention(
        w.num_q_heads, w.num_kv_heads, max_batch=max_batch or max(R, 1),
        max_seq_len=max_seq_len or max(b["max_seq_len"], 1), kv_dtype=w.kv_dtype,
        out_dtype=out_dtype, block_size=w.block_size,
        num_splits=w.num_splits if num_splits is None else num_splits)
    t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
    outs = []
    for _ in range(reps):
        out, lse = op(t["q"], t["k"], t["v"], t["seq_lens"], block_table=t.get("block_table"),
                      k_scale=t.get("k_scale"), v_scale=t.get("v_scale"))
        torch.cuda.synchronize()
        outs.append((out.float().cpu().double().numpy(), lse.cpu().double().numpy()))
    info = (op.num_splits, op.split_tokens)
    op.close()
    return outs if reps > 1 else outs[0], info


def check(got, ref, kind, pairs=None):
    out, lse = got
    ref_out, ref_lse = ref
    if pairs is not None:
        pr = np.asarray(pairs)
        out, lse = out[pr[:, 0], pr[:, 1]], lse[pr[:, 0], pr[:, 1]]
    assert np.isfinite(out).all(), "non-finite output (poisoned padding was read?)"
    err = np.abs(out - ref_out)
    fin = np.isfinite(ref_lse)
    assert (lse[~fin] == ref_lse[~fin]).all()
    lerr = np.abs(lse[fin] - ref_lse[fin]).max() if fin.any() else 0.0
    if kind == "bf16_f32":
        big = np.abs(ref_out) >= 1e-3
        rel = (err[big] / np.abs(ref_out[big])).max() if big.any() else 0.0
        assert err.max() <= 2e-3, f"max abs {err.max():.3e}"
        assert rel <= 1e-2, f"max rel {rel:.3e}"
        assert lerr <= 1e-3, f"lse {lerr:.3e}"
    elif kind == "bf16_bf16":
        assert (err <= 2e-3 + 1e-2 * np.abs(ref_out)).all(), f"max abs {err.max():.3e}"
        assert lerr <= 1e-3
    elif kind == "fp8":
        assert err.max() <= 3e-2, f"max abs {err.max():.3e}"
        assert lerr <= 5e-3, f"lse {lerr:.3e}"
    else:
        raise ValueError(kind)
    return float(err.max()), float(lerr)


def sized(name, lens, **over):
    w = W.WORKLOADS[name]
    if over:
        import dataclasses
        w = dataclasses.replace(w, **over)
    return W.generate(w, lens=np.asarray(lens, dtype=np.int32))


# ---- the named workloads at sizes the oracle finishes in seconds ---------------------------

def test_tiny_workload_matches_oracle():
    b = W.generate(W.WORKLOADS["tiny"])
    got, _ = gpu_of(b)
    check(got, oracle_of(b), "bf16_f32")


RAGGED = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000, 4101]


@pytest.mark.parametrize("splits", [1, 0, 3, 40])
def test_ragged_lengths_contiguous_bf16(splits):
    b = sized("llama3_8b_ctx4096", RAGGED)
    got, info = gpu_of(b, num_splits=splits)
    check(got, oracle_of(b), "bf16_f32")
    if splits > 1:
        assert info[0] == splits


def test_bf16_output_type():
    b = sized("llama3_8b_ctx4096", [300, 4096, 77])
    got, _ = gpu_of(b, out_dtype="bf16")
    check(got, oracle_of(b), "bf16_bf16")


@pytest.mark.parametrize("hq,hkv", [(8, 8), (8, 4), (16, 1), (4, 1)])
def test_other_group_sizes(hq, hkv):
    b = sized("llama3_8b_ctx4096", [200, 515, 64], num_q_heads=hq, num_kv_heads=hkv)
    got, _ = gpu_of(b)
    check(got, oracle_of(b), "bf16_f32")


# The library dispatches one kernel per (cache dtype, layout, number of four-head Q row groups):
# twelve variants, each with its own register budget and Q-prefetch schedule.  Every one of
# them runs here in each of the three partitioning modes -- rows (never cut), balanced shares
# (the grid holds more work-groups than the call has units, so every row longer than one unit
# is cut and goes through the merge) and fixed partitions -- on ragged lengths that include an
# empty request, single tokens and tails that end inside a tile and inside a page.
VARIANT_LENS = [0, 1, 17, 4101, 300, 2049, 128, 129]


@pytest.mark.parametrize("splits", [1, 0, 3], ids=["rows", "balanced", "fixed3"])
@pytest.mark.parametrize("G", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("layout", ["contiguous", "paged"])
@pytest.mark.parametrize("kv", ["bf16", "fp8"])
def test_every_kernel_variant_in_every_mode(kv, layout, G, splits):
    name = "fp8_paged" if kv == "fp8" else "llama3_8b_ctx4096"
    b = sized(name, VARIANT_LENS, num_q_heads=2 * G, num_kv_heads=2,
              block_size=16 if layout == "paged" else 0)
    got, info = gpu_of(b, num_splits=splits, max_seq_len=4101)
    assert info[0] == splits
    check(got, oracle_of(b), "fp8" if kv == "fp8" else "bf16_f32")
    out, lse = got
    assert (out[0] == 0).all() and np.isneginf(lse[0]).all()          # the empty request


@pytest.mark.parametrize("layout", ["contiguous", "paged"])
@pytest.mark.parametrize("G", [8, 16])
def test_bf16_output_of_cut_rows_for_the_wide_groups(G, layout):
    # the bf16 store paths of the item end and of the merge, 8 and 16 heads per group
    b = sized("llama3_8b_ctx4096", [4101, 0, 640, 1], num_q_heads=G, num_kv_heads=1,
              block_size=16 if layout == "paged" else 0)
    for splits in (1, 0, 5):
        got, _ = gpu_of(b, out_dtype="bf16", num_splits=splits, max_seq_len=4101)
        check(got, oracle_of(b), "bf16_bf16")


@pytest.mark.parametrize("splits", [1, 0, 5])
def test_paged_bf16_with_shuffled_block_table(splits):
    lens = [1, 16, 17, 100, 128, 2049, 700, 31, 3333, 4096, 513, 15]
    b = sized("llama3_70b_headshare_paged", lens)
    got, _ = gpu_of(b, num_splits=splits)
    check(got, oracle_of(b), "bf16_f32")


@pytest.mark.parametrize("splits", [1, 0, 6])
def test_fp8_paged(splits):
    lens = [1024, 1, 17, 2000, 129, 5000, 64, 3071]
    b = sized("fp8_paged", lens)
    got, _ = gpu_of(b, num_splits=splits)
    check(got, oracle_of(b), "fp8")


def test_fp8_contiguous():
    b = sized("fp8_paged", [33, 700, 1], block_size=0)
    got, _ = gpu_of(b)
    check(got, oracle_of(b), "fp8")


def test_split_kv_64_partitions_including_requests_shorter_than_the_split_count():
    # 64 partitions of 256 tokens over max_seq_len 16384; several requests leave most empty
    lens = [16384, 1, 255, 256, 257, 5000, 64, 16383]
    b = sized("longctx_split64", lens)
    got, info = gpu_of(b)
    assert info == (64, 256)
    check(got, oracle_of(b), "bf16_f32")


def test_empty_context_and_empty_batch():
    b = sized("llama3_8b_ctx4096", [0, 5, 0, 300])
    for splits in (1, 4):
        got, _ = gpu_of(b, num_splits=splits, max_seq_len=512)
        out, lse = got
        assert (out[0] == 0).all() and (out[2] == 0).all()
        assert np.isneginf(lse[0]).all() and np.isneginf(lse[2]).all()
        check(got, oracle_of(b), "bf16_f32")
    # batch == 0 is a no-op that must not touch the GPU buffers
    op = lamina.DecodeAttention(32, 8, max_batch=4, max_seq_len=64)
    p = lamina.lamina_call_params()
    p.batch = 0
    assert lamina.lamina_decode_attention(op.handle, None, None, None, None, None, None, None,
                                          p) == lamina.LAMINA_OK
    op.close()


@pytest.mark.parametrize("name,splits,hkv", [
    ("llama3_8b_ctx4096", 1, 8),                  # rows
    ("llama3_8b_ctx4096", 8, 8),                  # fixed partitions shared by four wavefronts
    ("llama3_8b_ctx4096", 0, 8),                  # balanced shares
    ("llama3_70b_headshare_paged", 0, 1),         # balanced shares, paged, 8 heads per group
    ("fp8_paged", 0, 8),                          # balanced shares, fp8
    ("fp8_paged", 6, 8),                          # fixed partitions, fp8
    ("llama3_8b_ctx4096", 64, 8),                 # fixed partitions owned by single wavefronts
    ("fp8_paged", 64, 8),
])
def test_results_are_bitwise_reproducible_run_to_run(name, splits, hkv):
    # No atomics on data and a fixed order in every reduction: the same call gives the same
    # bits, in every partitioning mode and for both cache types.  (With 64 partitions over
    # sixteen requests of up to 16384 tokens each wavefront owns its partitions.)
    w = W.WORKLOADS[name]
    lens = WAVE_OWNED_LENS if splits == 64 else [4096, 1000, 37, 2222, 0, 4101]
    if splits == 64:
        assert wavefronts_own_their_partitions(lens, hkv)
    b = sized(name, lens, num_q_heads=w.group * hkv, num_kv_heads=hkv)
    runs, info = gpu_of(b, num_splits=splits, max_seq_len=max(lens), reps=3)
    assert info[0] == splits
    assert np.isfinite(runs[0][0]).all()
    for o, l in runs[1:]:
        assert np.array_equal(o, runs[0][0]) and np.array_equal(l, runs[0][1])


def test_larger_capacity_than_the_call_uses():
    # max_batch / max_seq_len above what the call needs: same numbers
    b = sized("llama3_8b_ctx4096", [700, 90])
    got, _ = gpu_of(b, max_batch=64, max_seq_len=4096)
    check(got, oracle_of(b), "bf16_f32")


def test_strided_cache_view():
    b = sized("llama3_8b_ctx4096", [130, 257])
    w = b["workload"]
    d = dev()
    R, Hkv, L, D = b["k"].shape
    bigk = torch.full((R, Hkv, L + 7, 2 * D), float("nan"), dtype=torch.bfloat16)
    bigv = torch.full((R, Hkv, L + 7, 2 * D), float("nan"), dtype=torch.bfloat16)
    bigk[:, :, :L, :D] = b["k"]
    bigv[:, :, :L, :D] = b["v"]
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=R, max_seq_len=L)
    out, lse = op(b["q"].to(d), bigk.to(d)[:, :, :, :D], bigv.to(d)[:, :, :, :D],
                  b["seq_lens"].to(d))
    torch.cuda.synchronize()
    check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b), "bf16_f32")
    op.close()


def test_call_argument_errors_are_reported_not_launched():
    d = dev()
    op = lamina.DecodeAttention(32, 8, max_batch=2, max_seq_len=64)
    q = torch.zeros(2, 32, 128, dtype=torch.bfloat16, device=d)
    k = torch.zeros(2, 8, 64, 128, dtype=torch.bfloat16, device=d)
    lens = torch.ones(2, dtype=torch.int32, device=d)
    out = torch.zeros(2, 32, 128, device=d)

    def call(batch=2, qq=q, kk=k, stride_tok=128, oo=out):
        p = lamina.lamina_call_params()
        p.batch = batch
        p.kv_stride_req, p.kv_stride_head, p.kv_stride_tok = 8 * 64 * 128, 64 * 128, stride_tok
        return lamina.lamina_decode_attention(
            op.handle, qq.data_ptr() if qq is not None else None,
            kk.data_ptr() if kk is not None else None, k.data_ptr(), lens.data_ptr(), None,
            oo.data_ptr() if oo is not None else None, None, p)

    assert call() == lamina.LAMINA_OK
    assert call(batch=3) == lamina.LAMINA_ERR_INVALID_ARG
    assert "max_batch" in lamina.lamina_attn_last_error(op.handle)
    assert call(batch=-1) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(qq=None) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(kk=None) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(oo=None) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(stride_tok=100) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(stride_tok=132) == lamina.LAMINA_ERR_INVALID_ARG        # rows not 16 B aligned
    assert lamina.lamina_decode_attention(op.handle, q.data_ptr(), k.data_ptr(), k.data_ptr(),
                                          lens.data_ptr(), None, out.data_ptr(), None,
                                          None) == lamina.LAMINA_ERR_INVALID_ARG
    op.close()
    # paged without a block table, fp8 without scales
    op = lamina.DecodeAttention(8, 1, max_batch=2, max_seq_len=64, block_size=16)
    p = lamina.lamina_call_params()
    p.batch, p.pool_stride_block, p.pool_stride_head, p.block_table_stride = 2, 2048, 2048, 4
    assert lamina.lamina_decode_attention(op.handle, q.data_ptr(), k.data_ptr(), k.data_ptr(),
                                          lens.data_ptr(), None, out.data_ptr(), None,
                                          p) == lamina.LAMINA_ERR_INVALID_ARG
    op.close()
    op = lamina.DecodeAttention(8, 1, max_batch=2, max_seq_len=64, kv_dtype="fp8")
    p = lamina.lamina_call_params()
    p.batch, p.kv_stride_req, p.kv_stride_head, p.kv_stride_tok = 2, 8192, 8192, 128
    assert lamina.lamina_decode_attention(op.handle, q.data_ptr(), k.data_ptr(), k.data_ptr(),
                                          lens.data_ptr(), None, out.data_ptr(), None,
                                          p) == lamina.LAMINA_ERR_INVALID_ARG
    op.close()
    torch.cuda.synchronize()


def test_non_default_stream():
    b = sized("llama3_8b_ctx4096", [900, 64])
    w = b["workload"]
    d = dev()
    t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=2, max_seq_len=1024,
                                num_splits=4)
    s = torch.cuda.Stream(device=d)
    s.wait_stream(torch.cuda.current_stream(d))
    with torch.cuda.stream(s):
        out, lse = op(t["q"], t["k"], t["v"], t["seq_lens"])
    s.synchronize()
    check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b), "bf16_f32")
    op.close()


# ---- the named workloads at full size, in the launch configuration bench.py times ----------

def sample_pairs(b, n, seed):
    R, Hq = b["q"].shape[:2]
    rng = np.random.default_rng(seed)
    lens = b["seq_lens"].numpy()
    # always include the longest and the shortest request
    picks = {(int(lens.argmax()), 0), (int(lens.argmin()), Hq - 1)}
    while len(picks) < min(n, R * Hq):
        picks.add((int(rng.integers(R)), int(rng.integers(Hq))))
    return sorted(picks)


def test_full_llama3_8b_ctx4096_all_rows():
    print("generating llama3_8b_ctx4096", flush=True)
    b = W.generate(W.WORKLOADS["llama3_8b_ctx4096"], threads=16)
    got, info = gpu_of(b)
    print("partitioning", info, flush=True)
    e = check(got, oracle_of(b), "bf16_f32")
    print("max abs err, lse err", e, flush=True)


def test_full_llama3_8b_ctx4096_bf16_output_all_rows():
    # the configuration bench.py times: bf16 output
    print("generating llama3_8b_ctx4096", flush=True)
    b = W.generate(W.WORKLOADS["llama3_8b_ctx4096"], threads=16)
    got, info = gpu_of(b, out_dtype="bf16")
    print("partitioning", info, flush=True)
    e = check(got, oracle_of(b), "bf16_bf16")
    print("max abs err, lse err", e, flush=True)


def test_full_llama3_70b_headshare_paged_all_rows():
    print("generating llama3_70b_headshare_paged", flush=True)
    b = W.generate(W.WORKLOADS["llama3_70b_headshare_paged"], threads=16)
    got, info = gpu_of(b, max_seq_len=32768)
    print("partitioning", info, flush=True)
    e = check(got, oracle_of(b), "bf16_f32")
    print("max abs err, lse err", e, flush=True)


def test_full_mha_shapes_all_rows():
    # G = 1: the paper's LLaMA-33B / 65B shapes, one attention device's head share
    for name in ("llama_65b_mha_ctx4096", "llama_33b_mha_paged"):
        print("generating", name, flush=True)
        b = W.generate(W.WORKLOADS[name], threads=16)
        got, info = gpu_of(b, max_seq_len=int(b["seq_lens"].max()))
        print("partitioning", info, flush=True)
        e = check(got, oracle_of(b), "bf16_f32")
        print("max abs err, lse err", e, flush=True)


def test_full_longctx_split64_all_rows():
    print("generating longctx_split64 (8 GiB)", flush=True)
    b = W.generate(W.WORKLOADS["longctx_split64"], threads=16)
    got, info = gpu_of(b)
    assert info == (64, 2048)
    print("oracle on all", 16 * 32, "rows", flush=True)
    e = check(got, oracle_of(b), "bf16_f32")
    print("max abs err, lse err", e, flush=True)
    # the same batch with bf16 output (the merge's bf16 store path at full size)
    got, _ = gpu_of(b, out_dtype="bf16")
    check(got, oracle_of(b), "bf16_bf16")


def test_full_fp8_paged_all_rows():
    print("generating fp8_paged", flush=True)
    b = W.generate(W.WORKLOADS["fp8_paged"], threads=16)
    got, info = gpu_of(b, max_seq_len=16384)
    print("partitioning", info, flush=True)
    print("oracle on all", 128 * 64, "rows", flush=True)
    e = check(got, oracle_of(b), "fp8")
    print("max abs err, lse err", e, flush=True)


# ---- the new token's path: append k_n, v_n and fold them into a result over prev -----------

def _append_reference(b, k_new, v_new, positions):
    """Host-side expected cache after the append (bf16: the rows; fp8: oracle-encoded bytes)."""
    w = b["workload"]
    k, v = b["k"].clone(), b["v"].clone()
    R, Hkv = k_new.shape[:2]
    for r in range(R):
        pos = int(positions[r])
        if pos < 0:
            continue
        for g in range(Hkv):
            for dst, src, sc in ((k, k_new, b.get("k_scale")), (v, v_new, b.get("v_scale"))):
                if w.block_size:
                    row = dst[int(b["block_table"][r, pos // 16]), g, pos % 16]
                else:
                    row = dst[r, g, pos]
                if w.kv_dtype == "bf16":
                    row.copy_(src[r, g])
                else:
                    x = (src[r, g].double() / sc[r, g].double()).tolist()
                    row.view(torch.uint8).copy_(torch.tensor(
                        [oracle.e4m3fn_encode(float(np.float32(xi))) for xi in x], dtype=torch.uint8))
    return k, v


@pytest.mark.parametrize("name", ["llama3_8b_ctx4096", "llama3_70b_headshare_paged", "fp8_paged"])
def test_append_then_two_phase_equals_one_phase(name):
    # Caches hold the previous tokens; the new token arrives separately (prev/new split).
    lens_prev = np.array([0, 1, 15, 16, 100, 511, 700], dtype=np.int32)
    w = W.WORKLOADS[name]
    import dataclasses
    b = W.generate(dataclasses.replace(w), lens=lens_prev + 1)      # room for the new token
    R = len(lens_prev)
    d = dev()
    g = torch.Generator().manual_seed(77)
    k_new = torch.randn(R, w.num_kv_heads, 128, generator=g).to(torch.bfloat16)
    v_new = torch.randn(R, w.num_kv_heads, 128, generator=g).to(torch.bfloat16)
    positions = torch.from_numpy(lens_prev.copy())
    positions_skip = positions.clone()
    t = {key: val.to(d) for key, val in b.items() if isinstance(val, torch.Tensor)}
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=R, max_seq_len=1024,
                                kv_dtype=w.kv_dtype, out_dtype="f32", block_size=w.block_size,
                                num_splits=2)
    # phase 1: attention over the previous tokens only (the new row in the cache is stale)
    out_prev, lse_prev = op(t["q"], t["k"], t["v"], positions.to(d), block_table=t.get("block_table"),
                            k_scale=t.get("k_scale"), v_scale=t.get("v_scale"))
    # phase 2: fold the new token in, without touching the cache
    out2, lse2 = op.fold_new_token(t["q"], k_new.to(d), v_new.to(d), out_prev, lse_prev,
                                   k_scale=t.get("k_scale"), v_scale=t.get("v_scale"))
    # the fused call (fold + append in one launch) on a copy of the cache: same bits as the two calls
    k_copy, v_copy = t["k"].clone(), t["v"].clone()
    out3, lse3 = op.fold_new_token_and_append(
        t["q"], k_new.to(d), v_new.to(d), out_prev, lse_prev, k_copy, v_copy, positions.to(d),
        block_table=t.get("block_table"), k_scale=t.get("k_scale"), v_scale=t.get("v_scale"))
    # append, bit-exact against the host reference
    op.append_kv(k_new.to(d), v_new.to(d), t["k"], t["v"], positions.to(d),
                 block_table=t.get("block_table"), k_scale=t.get("k_scale"), v_scale=t.get("v_scale"))
    torch.cuda.synchronize()
    k_ref, v_ref = _append_reference(b, k_new, v_new, positions)
    iv = torch.uint8 if w.kv_dtype == "fp8" else torch.int16
    # compare only bytes that are defined (everything but poisoned padding is identical anyway)
    assert torch.equal(t["k"].cpu().view(iv), k_ref.view(iv))
    assert torch.equal(t["v"].cpu().view(iv), v_ref.view(iv))
    assert torch.equal(k_copy.cpu().view(iv), k_ref.view(iv))
    assert torch.equal(v_copy.cpu().view(iv), v_ref.view(iv))
    assert torch.equal(out3, out2) and torch.equal(lse3, lse2)
    # one phase over the appended cache
    out1, lse1 = op(t["q"], t["k"], t["v"], t["seq_lens"], block_table=t.get("block_table"),
                    k_scale=t.get("k_scale"), v_scale=t.get("v_scale"))
    torch.cuda.synchronize()
    # oracle over the appended host cache
    b2 = dict(b)
    b2["k"], b2["v"] = k_ref, v_ref
    ref = oracle_of(b2)
    kind = "fp8" if w.kv_dtype == "fp8" else "bf16_f32"
    check((out1.cpu().double().numpy(), lse1.cpu().double().numpy()), ref, kind)
    check((out2.cpu().double().numpy(), lse2.cpu().double().numpy()), ref, kind)
    # skipping a request (position -1) leaves its rows alone
    positions_skip[:] = -1
    before = t["k"].clone()
    op.append_kv(v_new.to(d), k_new.to(d), t["k"], t["v"], positions_skip.to(d),
                 block_table=t.get("block_table"), k_scale=t.get("k_scale"), v_scale=t.get("v_scale"))
    torch.cuda.synchronize()
    assert torch.equal(before.view(iv), t["k"].view(iv))
    op.close()


def _oracle_bytes(x_bf16, scale_f32):
    """Bytes an fp8 cache holds for bf16 values x under fp32 scales (broadcast along the last
    axis): the quotient in fp32 (numpy's float32 division is IEEE, correctly rounded), then the
    oracle's nearest-even encoder."""
    quot = x_bf16.float().numpy().astype(np.float32) / scale_f32.numpy().astype(np.float32)[..., None]
    assert quot.dtype == np.float32
    return torch.tensor([oracle.e4m3fn_encode(float(v)) for v in quot.ravel()],
                        dtype=torch.uint8).view(*quot.shape)


def test_fp8_append_quantiser_is_bit_exact_at_cache_scale_and_on_ties():
    # (a) one decode step's worth of new rows of the fp8 workload: 128 requests x 8 kv heads x
    #     128 dims, K and V, scales exp(U(ln 1/32, ln 1/8)) -- none a power of two;
    # (b) every midpoint between neighbouring e4m3fn values (both signs, and beyond +-448)
    #     times scales 1/8, 3 and 3/8: the quotient is exactly the tie, which must go to even.
    #     A multiplication by a rounded reciprocal of 3 would miss these.
    d = dev()
    w = W.WORKLOADS["fp8_paged"]
    rng = np.random.default_rng(2405)
    # (a)
    R, Hkv = 128, 8
    lens_prev = rng.integers(0, 48, size=R).astype(np.int32)
    b = W.generate(w, lens=lens_prev + 1)
    t = {key: val.to(d) for key, val in b.items() if isinstance(val, torch.Tensor)}
    g = torch.Generator().manual_seed(5)
    k_new = torch.randn(R, Hkv, 128, generator=g).to(torch.bfloat16)
    v_new = (8.0 * torch.randn(R, Hkv, 128, generator=g)).to(torch.bfloat16)   # some saturate
    op = lamina.DecodeAttention(w.num_q_heads, Hkv, max_batch=R, max_seq_len=64, kv_dtype="fp8",
                                block_size=16)
    print("append 128 x 8 rows", flush=True)
    op.append_kv(k_new.to(d), v_new.to(d), t["k"], t["v"], torch.from_numpy(lens_prev).to(d),
                 block_table=t["block_table"], k_scale=t["k_scale"], v_scale=t["v_scale"])
    torch.cuda.synchronize()
    want_k, want_v = _oracle_bytes(k_new, b["k_scale"]), _oracle_bytes(v_new, b["v_scale"])
    blk = b["block_table"].numpy()[np.arange(R), lens_prev // 16]
    got_k = t["k"].cpu().view(torch.uint8)[torch.from_numpy(blk).long(), :, torch.from_numpy(lens_prev % 16).long()]
    got_v = t["v"].cpu().view(torch.uint8)[torch.from_numpy(blk).long(), :, torch.from_numpy(lens_prev % 16).long()]
    assert torch.equal(got_k, want_k)
    assert torch.equal(got_v, want_v)
    assert int((want_v == 0x7E).sum()) > 0 and int((want_v == 0xFE).sum()) > 0   # saturation was hit
    op.close()
    # (b)
    grid = sorted(oracle.e4m3fn_decode(c) for c in range(0x7F))                  # 0 .. 448
    mids = [(lo + hi) / 2 for lo, hi in zip(grid[:-1], grid[1:])] + [464.0, 480.0]
    vals = torch.tensor(mids + [-m for m in mids], dtype=torch.float64)
    assert vals.numel() == 256
    scales = [0.125, 3.0, 0.375]
    x = torch.stack([vals * sc for sc in scales]).view(len(scales) * 2, 1, 128)
    xb = x.to(torch.bfloat16)
    assert torch.equal(xb.double(), x)                                           # exactly representable
    ks = torch.tensor(scales, dtype=torch.float32).repeat_interleave(2).view(-1, 1)
    R = xb.shape[0]
    b = sized("fp8_paged", [1] * R, num_q_heads=8, num_kv_heads=1)
    t = {key: val.to(d) for key, val in b.items() if isinstance(val, torch.Tensor)}
    op = lamina.DecodeAttention(8, 1, max_batch=R, max_seq_len=16, kv_dtype="fp8", block_size=16)
    print("append the ties", flush=True)
    op.append_kv(xb.to(d), xb.to(d), t["k"], t["v"], torch.zeros(R, dtype=torch.int32, device=d),
                 block_table=t["block_table"], k_scale=ks.to(d), v_scale=ks.to(d))
    torch.cuda.synchronize()
    want = _oracle_bytes(xb, ks)
    blk = torch.from_numpy(b["block_table"].numpy()[:, 0]).long()
    got = t["k"].cpu().view(torch.uint8)[blk, :, 0]
    assert torch.equal(got, want)
    assert torch.equal(t["v"].cpu().view(torch.uint8)[blk, :, 0], want)
    # ties went to even codes
    assert int((want & 1).sum()) == 0
    op.close()
    # (c) (x, scale) pairs -- found by a search on the CPU -- for which x * (1 / scale) in fp32
    #     lands on the other side of a tie than x / scale does: the division is what counts
    pairs = [(-2.71875, 0.2861842215061188), (0.51171875, 0.0444972850382328),
             (0.259765625, 0.488970547914505), (0.6796875, 0.15992645919322968),
             (-1.359375, 0.01999080739915371), (0.859375, 0.018682066351175308),
             (-0.03515625, 0.016544116660952568), (0.9375, 0.24193549156188965),
             (-2.28125, 0.5887097120285034), (0.828125, 0.3154761791229248),
             (0.67578125, 0.2162499874830246), (1.359375, 0.0251736119389534)]
    R = len(pairs)
    xb = torch.zeros(R, 1, 128, dtype=torch.bfloat16)
    xb[:, 0, 0] = torch.tensor([x for x, _ in pairs]).to(torch.bfloat16)
    ks = torch.tensor([sc for _, sc in pairs], dtype=torch.float32).view(-1, 1)
    recip = (xb.float().numpy() * (np.float32(1.0) / ks.numpy())[..., None]).astype(np.float32)
    want = _oracle_bytes(xb, ks)
    assert all(oracle.e4m3fn_encode(float(recip[i, 0, 0])) != int(want[i, 0, 0]) for i in range(R))
    b = sized("fp8_paged", [1] * R, num_q_heads=8, num_kv_heads=1)
    t = {key: val.to(d) for key, val in b.items() if isinstance(val, torch.Tensor)}
    op = lamina.DecodeAttention(8, 1, max_batch=R, max_seq_len=16, kv_dtype="fp8", block_size=16)
    print("append the division-versus-reciprocal cases", flush=True)
    op.append_kv(xb.to(d), xb.to(d), t["k"], t["v"], torch.zeros(R, dtype=torch.int32, device=d),
                 block_table=t["block_table"], k_scale=ks.to(d), v_scale=ks.to(d))
    torch.cuda.synchronize()
    blk = torch.from_numpy(b["block_table"].numpy()[:, 0]).long()
    assert torch.equal(t["k"].cpu().view(torch.uint8)[blk, :, 0], want)
    op.close()


def brute_force_partials(lens, Hkv, G, unit, nwg, parts=None):
    """Deal the unit stream to work-groups one unit at a time and count the pieces of cut rows.
    Balanced shares: a row is one unit for its fixed cost, then its tokens in blocks of `unit`;
    only the token units make pieces."""
    units = [max(1, -(-int(n) // unit)) for n in lens]
    if parts is not None:
        units = [min(parts, u) for u in units]
    cost = 0 if parts is not None else 1
    owner_of_unit = []
    U = sum(u + cost for u in units) * Hkv
    # Fixed partitions are dealt evenly.  Balanced shares: with at least 48 units per work-group
    # the even-numbered work-groups take 68/64 of an even share and the odd-numbered ones 60/64
    # (the odd dies of the chip stream slower); with 12 to 48 units it is 66/64 and 62/64;
    # below that the dealing is even.  With a skew, work-group j starts at unit
    # floor(U * c(j) / c(nwg)), c(j) = 64 j + skew * (j odd).
    skew = 0 if parts is not None else (4 if U >= 48 * nwg else (2 if U >= 12 * nwg else 0))
    if skew == 0:
        q, rem = divmod(U, nwg)
        begin = [j * q + min(j, rem) for j in range(nwg + 1)]
    else:
        c = lambda j: 64 * j + skew * (j & 1)
        begin = [U * c(j) // c(nwg) for j in range(nwg + 1)]
    for j in range(nwg):
        owner_of_unit += [j] * (begin[j + 1] - begin[j])
    assert len(owner_of_unit) == U
    total, at = 0, 0
    for n in units:
        for _ in range(Hkv):
            at += cost
            pieces = n if parts is not None else len(set(owner_of_unit[at:at + n]))
            at += n
            if pieces > 1:
                total += pieces
    return total * G


def test_balanced_shares_follow_the_batch_and_partials_are_counted():
    d = dev()
    w = W.WORKLOADS["llama3_8b_ctx4096"]
    # balanced shares run one work-group per compute unit (half of what can be resident)
    nwg = (min(1024, 2 * torch.cuda.get_device_properties(0).multi_processor_count) + 1) // 2
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=64, max_seq_len=65536)
    assert (op.num_splits, op.split_tokens) == (0, 128)
    # a skewed batch: one long row is spread over many work-groups, short and empty ones are not cut
    lens = [50000, 3, 0, 700, 129, 4096]
    b = sized("llama3_8b_ctx4096", lens)
    t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
    out, lse = op(t["q"], t["k"], t["v"], t["seq_lens"])
    torch.cuda.synchronize()
    check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b), "bf16_f32")
    n = op.count_partials(lens)
    assert n == brute_force_partials(lens, w.num_kv_heads, 4, 128, nwg) and n > 0
    # a big uniform batch on the same handle: two rows per work-group; the shares differ by
    # work-group parity, so rows are cut where an even work-group's share runs into the next row
    lens = [8192] * 64
    b = sized("llama3_8b_ctx4096", lens)
    t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
    out, lse = op(t["q"], t["k"], t["v"], t["seq_lens"])
    torch.cuda.synchronize()
    pairs = sample_pairs(b, 40, 9)
    check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b, pairs=pairs),
          "bf16_f32", pairs=pairs)
    assert op.count_partials(lens) == brute_force_partials(lens, w.num_kv_heads, 4, 128, nwg)
    op.close()
    # an explicit partition count is kept exactly
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=64, max_seq_len=8192,
                                num_splits=16)
    out, lse = op(t["q"], t["k"], t["v"], t["seq_lens"])
    torch.cuda.synchronize()
    assert (op.num_splits, op.split_tokens) == (16, 512)
    assert op.count_partials(lens) == 64 * w.num_q_heads * 16
    assert op.count_partials([8192, 100, 513]) == brute_force_partials(
        [8192, 100, 513], w.num_kv_heads, 4, 512, nwg, parts=16) == (16 + 2) * w.num_q_heads
    check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b, pairs=pairs),
          "bf16_f32", pairs=pairs)
    op.close()


def test_one_long_row_is_spread_over_every_work_group():
    # a single (request, kv head) row of 300 000 tokens: every work-group takes a piece of it
    # and the merge combines several hundred partial results (more than one wavefront of them)
    w = W.WORKLOADS["llama_65b_mha_ctx4096"]
    b = sized("llama_65b_mha_ctx4096", [300_000], num_q_heads=1, num_kv_heads=1)
    got, info = gpu_of(b)
    assert info == (0, 128)
    check(got, oracle_of(b), "bf16_f32")
    # the same row with a few short neighbours, G = 8
    b = sized("llama3_70b_headshare_paged", [5, 200_000, 129, 1])
    got, info = gpu_of(b)
    assert info == (0, 128)
    check(got, oracle_of(b), "bf16_f32")


def test_the_largest_batch_of_a_handle_that_cuts_rows():
    # 1024 requests (the limit of the in-kernel prefix sum), lengths 0 .. 1500: thousands of
    # short rows, most work-groups hold several whole rows and the tails of two more
    rng = np.random.default_rng(7)
    lens = rng.integers(0, 1501, size=1024).astype(np.int32)
    lens[:4] = [0, 1500, 1, 128]
    b = sized("llama_65b_mha_ctx4096", lens, num_q_heads=4, num_kv_heads=2)
    got, info = gpu_of(b, max_seq_len=100_000)             # a capacity that makes the handle cut rows
    assert info == (0, 128)
    check(got, oracle_of(b), "bf16_f32")


def test_partitioned_handle_limits_are_reported_at_creation():
    dev()
    # handles that never cut rows take any batch; so does the library's own choice, by not cutting
    op = lamina.DecodeAttention(8, 8, max_batch=5000, max_seq_len=2048)
    assert op.num_splits == 1 and op.count_partials([2048] * 5000) == 0
    op.close()
    op = lamina.DecodeAttention(8, 1, max_batch=2000, max_seq_len=100000)
    assert op.num_splits == 1
    op.close()
    # explicit partitions need the batch to fit the prefix sum the kernel keeps in LDS
    with pytest.raises(lamina.LaminaError) as ei:
        lamina.DecodeAttention(8, 1, max_batch=2000, max_seq_len=100000, num_splits=4)
    assert ei.value.code == lamina.LAMINA_ERR_UNSUPPORTED
    with pytest.raises(lamina.LaminaError) as ei:
        lamina.DecodeAttention(64, 64, max_batch=1024, max_seq_len=4_000_000)
    assert ei.value.code == lamina.LAMINA_ERR_UNSUPPORTED
    op = lamina.DecodeAttention(8, 8, max_batch=1024, max_seq_len=32768)
    assert (op.num_splits, op.split_tokens) == (0, 128)
    op.close()


def test_captured_in_a_graph_and_replayed_with_new_lengths():
    # The call enqueues kernels only (no host read of seq_lens, no allocation, no memset), so it
    # can be captured once and replayed while q, seq_lens and the cache change underneath it:
    # the partitioning is redone on the device at every replay.
    d = dev()
    w = W.WORKLOADS["llama3_8b_ctx4096"]
    first = sized("llama3_8b_ctx4096", [9000, 40, 3000, 129])
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=4, max_seq_len=9000)
    assert op.num_splits == 0
    t = {k: v.to(d) for k, v in first.items() if isinstance(v, torch.Tensor)}
    out = torch.empty(4, w.num_q_heads, 128, device=d)
    lse = torch.empty(4, w.num_q_heads, device=d)
    side = torch.cuda.Stream(device=d)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                         # warm-up outside the capture
        op(t["q"], t["k"], t["v"], t["seq_lens"], out=out, lse=lse)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        op(t["q"], t["k"], t["v"], t["seq_lens"], out=out, lse=lse)
    for lens in ([9000, 40, 3000, 129], [1, 8999, 0, 4097], [512, 512, 512, 512]):
        b = sized("llama3_8b_ctx4096", lens)
        # same shapes (the cache is laid out for the handle's capacity), new contents
        k = torch.zeros_like(t["k"]); v = torch.zeros_like(t["v"])
        n = b["k"].shape[2]
        k[:, :, :n] = b["k"].to(d); v[:, :, :n] = b["v"].to(d)
        t["k"].copy_(k); t["v"].copy_(v)
        t["q"].copy_(b["q"].to(d)); t["seq_lens"].copy_(b["seq_lens"].to(d))
        out.fill_(float("nan")); lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b), "bf16_f32")
    op.close()


def test_lengths_beyond_the_capacity_are_clamped_and_bad_append_positions_skipped():
    # A length above max_seq_len (or negative) must not turn into a read outside the cache
    # the call was given: it is treated as max_seq_len (or 0).
    d = dev()
    w = W.WORKLOADS["llama3_8b_ctx4096"]
    lens = [300, 77, 200, 300]
    b = sized("llama3_8b_ctx4096", lens)                  # cache rows 0..299 per request
    for splits in (1, 0, 2):
        op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=4, max_seq_len=300,
                                    num_splits=splits)
        t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
        claimed = torch.tensor([300 + 100_000, 77, -5, 300], dtype=torch.int32, device=d)
        out, lse = op(t["q"], t["k"], t["v"], claimed)
        torch.cuda.synchronize()
        eff = dict(b)
        eff["seq_lens"] = torch.tensor([300, 77, 0, 300], dtype=torch.int32)
        check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(eff), "bf16_f32")
        op.close()
    # append: positions outside [0, max_seq_len) leave the cache untouched
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=4, max_seq_len=300)
    t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
    before_k, before_v = t["k"].clone(), t["v"].clone()
    k_new = torch.ones(4, w.num_kv_heads, 128, dtype=torch.bfloat16, device=d)
    pos = torch.tensor([300, -1, 1 << 30, 299], dtype=torch.int32, device=d)
    op.append_kv(k_new, k_new, t["k"], t["v"], pos)
    torch.cuda.synchronize()
    iv = torch.int16
    assert torch.equal(before_k[:3].view(iv), t["k"][:3].view(iv))
    assert torch.equal(before_v[:3].view(iv), t["v"][:3].view(iv))
    assert bool((t["k"][3, :, 299] == 1).all()) and bool((t["v"][3, :, 299] == 1).all())
    assert torch.equal(before_k[3, :, :299].view(iv), t["k"][3, :, :299].view(iv))
    op.close()


def test_two_handles_on_two_streams_do_not_disturb_each_other():
    # each handle owns its workspace; calls of different handles may overlap on the device
    d = dev()
    w = W.WORKLOADS["llama3_8b_ctx4096"]
    ba = sized("llama3_8b_ctx4096", [6000, 130, 2500])
    bb = sized("llama3_8b_ctx4096", [17, 5000, 5000, 900, 64])
    ops, outs, streams = [], [], [torch.cuda.Stream(device=d), torch.cuda.Stream(device=d)]
    tens = []
    for b in (ba, bb):
        ops.append(lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=8,
                                          max_seq_len=6000))
        tens.append({k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)})
    torch.cuda.synchronize()
    for _ in range(5):                                    # interleave launches of both handles
        outs = []
        for op, t, s in zip(ops, tens, streams):
            outs.append(op(t["q"], t["k"], t["v"], t["seq_lens"], stream=s))
    for s in streams:
        s.synchronize()
    for b, (out, lse) in zip((ba, bb), outs):
        check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b), "bf16_f32")
    for op in ops:
        op.close()


@pytest.mark.parametrize("hq,hkv,block", [(8, 8, 16), (4, 2, 0), (16, 1, 16), (16, 1, 0), (8, 1, 0)])
def test_fp8_group_sizes_and_layouts(hq, hkv, block):
    # the fp8 path splits Q per head; cover 1, 2, 8 and 16 heads per group on both layouts
    b = sized("fp8_paged", [200, 1515, 64, 300], num_q_heads=hq, num_kv_heads=hkv,
              block_size=block)
    got, _ = gpu_of(b, max_seq_len=3000)                  # a capacity that makes the handle cut rows
    check(got, oracle_of(b), "fp8")


def test_fp8_queries_of_extreme_and_mixed_magnitude():
    # With an fp8 cache each query row is rescaled by a power of two and split into two e4m3
    # halves.  Heads whose queries are huge, tiny, zero, or mix magnitudes inside one row must
    # come out as exactly as ordinary ones.
    b = sized("fp8_paged", [900, 130, 257], num_q_heads=16, num_kv_heads=2)
    q = b["q"].float()
    q[:, 0] *= 3.0e4                                      # saturates the softmax on one key
    q[:, 1] *= 1.0e-6                                     # uniform softmax
    q[:, 2] = 0.0
    q[:, 3, :64] *= 2.0 ** -12                            # 4096:1 inside one row
    q[:, 4, ::2] *= 2.0 ** 9
    q[:, 5] *= 40.0
    q[:, 6, 5] = 1.0e3                                    # one dominant component
    b["q"] = q.to(torch.bfloat16)
    got, _ = gpu_of(b, max_seq_len=1000)
    out, lse = got
    ref_out, ref_lse = oracle_of(b)
    assert np.isfinite(out).all()
    assert np.abs(out - ref_out).max() <= 3e-2
    # lse grows with the score scale: compare relative to its magnitude
    assert (np.abs(lse - ref_lse) <= 5e-3 + 2e-3 * np.abs(ref_lse)).all()


def test_bf16_queries_of_extreme_and_mixed_magnitude():
    # saturated, flat and degenerate softmaxes through the online recurrence and the merge
    b = sized("llama3_8b_ctx4096", [5000, 130, 257], num_q_heads=8, num_kv_heads=2)
    q = b["q"].float()
    q[:, 0] *= 3.0e4
    q[:, 1] *= 1.0e-6
    q[:, 2] = 0.0
    q[:, 3, :64] *= 2.0 ** -12
    q[:, 4] *= 40.0
    b["q"] = q.to(torch.bfloat16)
    for splits in (1, 0, 3):
        got, _ = gpu_of(b, num_splits=splits, max_seq_len=5000)
        out, lse = got
        ref_out, ref_lse = oracle_of(b)
        assert np.isfinite(out).all()
        assert np.abs(out - ref_out).max() <= 2e-3
        assert (np.abs(lse - ref_lse) <= 1e-3 + 1e-6 * np.abs(ref_lse)).all()


def test_fp8_scales_over_many_orders_of_magnitude():
    # the K scale folds into the score scale and the V scale into the epilogue; neither may
    # lose accuracy when the scales are far from 1 (the oracle dequantises with the same ones)
    b = sized("fp8_paged", [700, 64, 2000, 129], num_q_heads=8, num_kv_heads=2)
    b["k_scale"] = torch.tensor([[1e-4, 1.0], [0.5, 3e-3], [2e-2, 1e-5], [7.0, 0.125]])
    b["v_scale"] = torch.tensor([[1e3, 1e-4], [1.0, 40.0], [1e-6, 2.0], [0.3, 5e2]])
    got, _ = gpu_of(b, max_seq_len=2000)
    out, lse = got
    ref_out, ref_lse = oracle_of(b)
    assert np.isfinite(out).all()
    vs = b["v_scale"].numpy().repeat(4, axis=1)[:, :, None]          # per (request, query head)
    assert (np.abs(out - ref_out) <= 3e-2 * np.maximum(vs * 8.0, 1e-30)).all()   # error scales with V
    assert (np.abs(lse - ref_lse) <= 5e-3 + 2e-3 * np.abs(ref_lse)).all()


# Sixteen requests of up to 16384 tokens in 64 partitions of 256: enough partitions for every
# wavefront of the grid to own at least two, the condition under which wavefronts work through
# partitions on their own instead of sharing each one four ways.
WAVE_OWNED_LENS = [16384] * 9 + [16000, 1, 0, 9000, 16383, 4097, 12345]


def wavefronts_own_their_partitions(lens, hkv, unit=256, parts=64):
    nwg = min(1024, 2 * torch.cuda.get_device_properties(0).multi_processor_count)
    units = sum(min(parts, max(1, -(-int(n) // unit))) for n in lens) * hkv
    return units >= 2 * 4 * nwg


@pytest.mark.parametrize("name,kind,out_dtype", [("fp8_paged", "fp8", "f32"),
                                                 ("llama3_70b_headshare_paged", "bf16_bf16", "bf16"),
                                                 ("llama3_8b_ctx4096", "bf16_f32", "f32")])
def test_many_fixed_partitions_are_worked_through_by_single_wavefronts(name, kind, out_dtype):
    # each wavefront takes partitions of its own (no combining across wavefronts); ragged ends,
    # one single-token and one empty request included; every row checked
    w = W.WORKLOADS[name]
    hkv = 8
    lens = WAVE_OWNED_LENS
    assert wavefronts_own_their_partitions(lens, hkv)
    b = sized(name, lens, num_q_heads=w.group * hkv, num_kv_heads=hkv)
    got, info = gpu_of(b, out_dtype=out_dtype, num_splits=64, max_seq_len=16384)
    assert info == (64, 256)
    check(got, oracle_of(b), kind)
    out, lse = got
    assert (out[11] == 0).all() and np.isneginf(lse[11]).all()        # the empty request
