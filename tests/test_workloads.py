"""Host-side checks of the seeded generators and of the algorithmic-bytes model.  CPU only."""
import math
import os

import numpy as np
import torch

import oracle
from paper_2405_01814_amd import workloads as W


def read_kv(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, val = line.split()
            out[key] = float(val)
    return out


def test_bytes_model_reproduces_the_papers_capacity_example(golden_dir):
    g = read_kv(os.path.join(golden_dir, "kv_capacity_example.txt"))
    # one attention device holding all L layers' caches of one request at this context:
    # per layer the model is algorithmic_bytes()["kv"] with Hkv*D = d/G elements per token.
    hkv = int(g["d"] / g["G"] / W.HEAD_DIM)
    w = W.Workload("x", 0, 1, hkv * int(g["G"]), hkv, ("fixed", int(g["context"])))
    per_layer = W.algorithmic_bytes(w, [int(g["context"])])["kv"]
    per_request = per_layer * g["L"]
    assert per_request == 2 * g["e"] * (g["d"] / g["G"]) * g["L"] * g["context"]
    assert abs(per_request / 1e9 - 2.68) < 0.01
    fit = g["device_memory_GB"] * 1e9 / per_request
    assert abs(fit - g["requests_about"]) < 1.0          # "about 30 requests"


def test_bytes_model_reproduces_the_papers_operator_io(golden_dir):
    g = read_kv(os.path.join(golden_dir, "operator_io_example.txt"))
    hkv = int(g["d"] / g["G"] / W.HEAD_DIM)
    w = W.Workload("x", 0, 1, hkv * int(g["G"]), hkv, ("fixed", 1))
    b = W.algorithmic_bytes(w, [1], out_bytes=int(g["e"]), with_lse=False)
    # q in + out back + the new token's k and v (which is the whole cache when len = 1)
    assert b["q"] + b["out"] + b["kv"] == g["bytes_per_request_per_layer"]
    assert b["q"] + b["out"] + b["kv"] == (2 + 2 / g["G"]) * g["e"] * g["d"]


def test_named_workloads_have_the_stated_shapes():
    w = W.WORKLOADS
    assert (w["tiny"].batch, w["tiny"].num_q_heads, w["tiny"].num_kv_heads) == (4, 8, 2)
    l1 = W.draw_lens(w["tiny"])
    assert l1.min() >= 16 and l1.max() <= 256
    l2 = W.draw_lens(w["llama3_8b_ctx4096"])
    assert len(l2) == 64 and (l2 == 4096).all()
    b2 = W.algorithmic_bytes(w["llama3_8b_ctx4096"], l2)
    assert b2["kv"] == 1024 * 2 ** 20 and b2["tokens"] == 262144 and b2["head_tokens"] == 2097152
    l3 = W.draw_lens(w["llama3_70b_headshare_paged"])
    assert len(l3) == 256 and l3.min() >= 128 and l3.max() <= 32768
    assert 1200 < np.median(l3) < 3200
    l4 = W.draw_lens(w["longctx_split64"])
    assert len(l4) == 16 and (l4 == 131072).all()
    b4 = W.algorithmic_bytes(w["longctx_split64"], l4, split_tokens=2048)
    assert b4["kv"] == 8192 * 2 ** 20 and b4["partials"] == 2 * 16 * 32 * 64 * 129 * 4
    assert w["llama_65b_mha_ctx4096"].group == 1 and w["llama_33b_mha_paged"].group == 1
    # 64 and 52 heads of 128 (d = 8192 and 6656) over 8 and 4 attention devices
    assert w["llama_65b_mha_ctx4096"].num_q_heads * 8 * 128 == 8192
    assert w["llama_33b_mha_paged"].num_q_heads * 4 * 128 == 6656
    l7 = W.draw_lens(w["llama_33b_mha_paged"])
    assert len(l7) == 256 and l7.min() >= 128 and l7.max() <= 16384
    l5 = W.draw_lens(w["fp8_paged"])
    assert len(l5) == 128 and l5.min() >= 1024 and l5.max() <= 16384


def test_generation_is_reproducible_and_thread_count_independent():
    w = W.WORKLOADS["tiny"]
    a = W.generate(w, threads=1)
    b = W.generate(w, threads=4)
    for key in ("q", "k", "v"):
        assert torch.equal(a[key].view(torch.int16), b[key].view(torch.int16))
    assert torch.equal(a["seq_lens"], b["seq_lens"])


def test_contiguous_padding_is_poisoned_and_valid_rows_are_finite():
    b = W.generate(W.WORKLOADS["tiny"])
    for r, n in enumerate(b["seq_lens"].tolist()):
        assert torch.isfinite(b["k"][r, :, :n].float()).all()
        assert torch.isnan(b["k"][r, :, n:].float()).all()
        assert torch.isnan(b["v"][r, :, n:].float()).all()
    x = b["k"][0, :, :b["seq_lens"][0]].float()
    assert abs(float(x.mean())) < 0.05 and abs(float(x.std()) - 1.0) < 0.05


def test_paged_pool_layout_and_block_table():
    w = W.WORKLOADS["llama3_70b_headshare_paged"]
    lens = np.array([1, 16, 17, 100, 0], dtype=np.int32)
    b = W.generate(w, lens=lens)
    bt, k = b["block_table"], b["k"]
    assert k.shape[1:] == (1, 16, 128)
    used = []
    for r, n in enumerate(lens):
        nb = (n + 15) // 16
        assert (bt[r, :nb] >= 0).all() and (bt[r, nb:] == -1).all()
        used += bt[r, :nb].tolist()
        for i in range(nb):
            rows = min(16, n - 16 * i)
            assert torch.isfinite(k[bt[r, i], :, :rows].float()).all()
            assert torch.isnan(k[bt[r, i], :, rows:].float()).all()
    assert len(set(used)) == len(used) and k.shape[0] > len(used)
    spare = sorted(set(range(k.shape[0])) - set(used))
    assert torch.isnan(k[spare].float()).all()
    # a paged batch holds the same values as the contiguous batch with the same seed
    wc = W.Workload("c", w.index, len(lens), w.num_q_heads, w.num_kv_heads, w.len_recipe)
    c = W.generate(wc, lens=lens)
    r = 3
    flat = torch.cat([k[bt[r, i]] for i in range(7)], dim=1)[:, :100]
    assert torch.equal(flat.view(torch.int16), c["k"][r, :, :100].view(torch.int16))
    # and the oracle sees the same thing through either layout
    o_p, l_p = oracle.decode_attention(b["q"], b["k"], b["v"], b["seq_lens"], num_kv_heads=1,
                                       scale=1 / math.sqrt(128), block_table=bt, block_size=16)
    o_c, l_c = oracle.decode_attention(c["q"], c["k"], c["v"], c["seq_lens"], num_kv_heads=1,
                                       scale=1 / math.sqrt(128))
    assert np.array_equal(o_p, o_c) and np.array_equal(l_p, l_c)


def test_fp8_batch_has_no_nan_codes_in_valid_rows_and_sane_scales():
    w = W.WORKLOADS["fp8_paged"]
    lens = np.array([40, 33], dtype=np.int32)
    b = W.generate(w, lens=lens)
    assert b["k"].dtype == torch.float8_e4m3fn
    assert b["k_scale"].shape == (2, 8) and b["k_scale"].dtype == torch.float32
    assert (b["k_scale"] >= 1 / 32 - 1e-6).all() and (b["k_scale"] <= 1 / 8 + 1e-6).all()
    bt = b["block_table"]
    for r, n in enumerate(lens):
        blk = b["k"][bt[r, 0]].view(torch.uint8)
        assert ((blk & 0x7F) != 0x7F).all()
        deq = b["k"][bt[r, 0]].float() * b["k_scale"][r].view(-1, 1, 1)
        assert abs(float(deq.std()) - 1.0) < 0.1
