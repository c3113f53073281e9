"""The vector-ALU-only version of the operator (lamina_probe_valu_attention, a measurement aid:
the reference for what the matrix cores buy) against the fp64 oracle, to the product's own
tolerance for bf16 caches with fp32 output; and its argument checks."""
import numpy as np
import pytest
import torch

from paper_2405_01814_amd import lamina
from test_gpu_parity import check, dev, oracle_of, sized

pytestmark = pytest.mark.gpu
LENS = [0, 1, 17, 4101, 300, 2049, 128, 129, 31, 32, 33, 1000]


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_vector_alu_operator_matches_the_oracle(G):
    b = sized("llama3_8b_ctx4096", LENS, num_q_heads=3 * G, num_kv_heads=3)
    t = {k: v.to(dev()) for k, v in b.items() if isinstance(v, torch.Tensor)}
    out, lse = lamina.valu_attention(t["q"], t["k"], t["v"], t["seq_lens"], 3, max(LENS))
    torch.cuda.synchronize()
    got = (out.cpu().double().numpy(), lse.cpu().double().numpy())
    check(got, oracle_of(b), "bf16_f32")
    assert (got[0][0] == 0).all() and np.isneginf(got[1][0]).all()    # the empty request


def test_vector_alu_operator_on_a_strided_view_and_a_small_grid():
    b = sized("llama3_8b_ctx4096", [700, 64, 5, 2500], num_q_heads=8, num_kv_heads=2)
    d = dev()
    t = {k: v.to(d) for k, v in b.items() if isinstance(v, torch.Tensor)}
    R, Hkv, L, D = t["k"].shape
    big_k = torch.full((R, Hkv, L + 9, D + 8), float("nan"), device=d, dtype=torch.bfloat16)
    big_v = torch.full_like(big_k, float("nan"))
    big_k[:, :, :L, :D] = t["k"]
    big_v[:, :, :L, :D] = t["v"]
    out, lse = lamina.valu_attention(t["q"], big_k[:, :, :L, :D], big_v[:, :, :L, :D],
                                     t["seq_lens"], Hkv, L, work_groups=3)
    torch.cuda.synchronize()
    check((out.cpu().double().numpy(), lse.cpu().double().numpy()), oracle_of(b), "bf16_f32")


def test_vector_alu_operator_rejects_what_it_does_not_cover():
    d = dev()
    q = torch.zeros(2, 16, 128, device=d, dtype=torch.bfloat16)
    k = torch.zeros(2, 1, 64, 128, device=d, dtype=torch.bfloat16)
    lens = torch.ones(2, device=d, dtype=torch.int32)
    out = torch.zeros(2, 16, 128, device=d)
    args = lambda **kw: {**dict(q=q.data_ptr(), k=k.data_ptr(), v=k.data_ptr(), lens=lens.data_ptr(),
                                out=out.data_ptr(), lse=None, R=2, Hq=16, Hkv=1, L=64, sr=64 * 128,
                                sh=64 * 128, st=128), **kw}
    call = lambda a: lamina.lamina_probe_valu_attention(
        a["q"], a["k"], a["v"], a["lens"], a["out"], a["lse"], a["R"], a["Hq"], a["Hkv"], a["L"],
        a["sr"], a["sh"], a["st"], 0.0, 0, None)
    assert call(args()) == lamina.LAMINA_ERR_UNSUPPORTED              # group size 16
    assert call(args(Hq=8, q=None)) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(args(Hq=8, st=64)) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(args(Hq=8, st=132)) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(args(Hq=8, L=0)) == lamina.LAMINA_ERR_INVALID_ARG
    assert call(args(Hq=8, R=0)) == lamina.LAMINA_OK                  # empty batch: nothing to do
    torch.cuda.synchronize()
