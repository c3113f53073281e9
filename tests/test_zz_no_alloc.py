"""lamina_decode_attention_static -- the call that allocates nothing -- against
lamina_decode_attention on a handle made from the same configuration: same kernels, same
partitioning, so the two must agree bit for bit (which is inside every tolerance the parity
tests state), on two calls in a row that share the static scratch area, the second one smaller.
Both go through the C ABI with raw device pointers."""
import numpy as np
import pytest
import torch

from paper_2405_01814_amd import lamina, workloads as W

pytestmark = pytest.mark.gpu


def dev():
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


def both_ways(name, lens, num_splits, max_batch, max_seq_len, out_dtype="f32", **over):
    """Returns ((out, lse) from the handle, (out, lse) from the static call) as numpy arrays."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS[name], **over) if over else W.WORKLOADS[name]
    b = W.generate(w, lens=np.asarray(lens, dtype=np.int32))
    d = dev()
    t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
    R = len(lens)
    op = lamina.DecodeAttention(w.num_q_heads, w.num_kv_heads, max_batch=max_batch,
                                max_seq_len=max_seq_len, kv_dtype=w.kv_dtype, out_dtype=out_dtype,
                                block_size=w.block_size, num_splits=num_splits)
    p = op.params_for(t["q"], t["k"], t.get("block_table"), t.get("k_scale"), t.get("v_scale"))
    odt = torch.float32 if out_dtype == "f32" else torch.bfloat16
    res = []
    for which in ("handle", "static"):
        out = torch.full((R, w.num_q_heads, 128), float("nan"), device=d, dtype=odt)
        lse = torch.full((R, w.num_q_heads), float("nan"), device=d)
        args = (t["q"].data_ptr(), t["k"].data_ptr(), t["v"].data_ptr(), t["seq_lens"].data_ptr(),
                t["block_table"].data_ptr() if "block_table" in t else None,
                out.data_ptr(), lse.data_ptr(), p)
        print(f"{name} {which}: R={R} splits={num_splits} max_seq_len={max_seq_len}", flush=True)
        if which == "handle":
            rc = lamina.lamina_decode_attention(op.handle, *args)
        else:
            rc = lamina.lamina_decode_attention_static(op.cfg, *args)
        assert rc == lamina.LAMINA_OK, lamina.lamina_attn_last_error(
            op.handle if which == "handle" else None)
        torch.cuda.synchronize()
        res.append((out.float().cpu().numpy(), lse.cpu().numpy()))
    cut = op.count_partials(lens)
    op.close()
    return res[0], res[1], cut


def assert_same(a, b):
    assert np.isfinite(a[0]).all()
    assert np.array_equal(a[0], b[0])
    assert np.array_equal(a[1], b[1])                     # -inf == -inf for empty requests


def test_static_call_equals_the_handle_call_on_two_calls_in_a_row():
    # balanced shares, bf16 contiguous: a long row cut over many work-groups, then -- on the
    # scratch area the first call left behind -- a smaller batch with an empty request
    h1, s1, cut1 = both_ways("llama3_8b_ctx4096", [20000, 300, 4097, 129, 1], 0, 8, 20000)
    assert cut1 > 0
    assert_same(h1, s1)
    h2, s2, cut2 = both_ways("llama3_8b_ctx4096", [5000, 0, 77], 0, 8, 20000)
    assert cut2 > 0
    assert_same(h2, s2)


def test_static_call_fixed_partitions_fp8_paged_then_smaller():
    h1, s1, cut1 = both_ways("fp8_paged", [3000, 1, 700, 2049], 6, 4, 3000)
    assert cut1 > 0
    assert_same(h1, s1)
    h2, s2, _ = both_ways("fp8_paged", [513, 64], 6, 4, 3000)
    assert_same(h2, s2)


def test_static_call_without_cut_rows_and_with_bf16_output():
    h, s, cut = both_ways("llama3_70b_headshare_paged", [900, 16, 515], 1, 4, 1024,
                          out_dtype="bf16")
    assert cut == 0
    assert_same(h, s)


def test_static_call_rejects_what_the_scratch_area_cannot_hold():
    dev()
    # 1024 requests x 8 kv heads x 64 partitions x 4 heads x 129 floats = 1 GiB of partials
    cfg = lamina.lamina_attn_config(32, 8, 128, lamina.LAMINA_BF16, lamina.LAMINA_F32, 0,
                                    1024, 131072, 64, 0.0, 0)
    assert lamina.lamina_attn_workspace_bytes(cfg) > lamina.LAMINA_STATIC_SCRATCH_BYTES
    q = torch.zeros(1, 32, 128, dtype=torch.bfloat16, device=dev())
    p = lamina.lamina_call_params()
    p.batch = 1
    p.kv_stride_req, p.kv_stride_head, p.kv_stride_tok = 8 * 128, 128, 128
    rc = lamina.lamina_decode_attention_static(cfg, q.data_ptr(), q.data_ptr(), q.data_ptr(),
                                               q.data_ptr(), None, q.data_ptr(), None, p)
    assert rc == lamina.LAMINA_ERR_WORKSPACE
    assert "static scratch" in lamina.lamina_attn_last_error(None)
    # a bad configuration is reported as lamina_attn_create reports it
    cfg.head_dim = 64
    rc = lamina.lamina_decode_attention_static(cfg, q.data_ptr(), q.data_ptr(), q.data_ptr(),
                                               q.data_ptr(), None, q.data_ptr(), None, p)
    assert rc == lamina.LAMINA_ERR_UNSUPPORTED
    assert lamina.lamina_decode_attention_static(None, None, None, None, None, None, None, None,
                                                 None) == lamina.LAMINA_ERR_INVALID_ARG
