"""Pins for the CPU oracle: each check fixes the oracle to something other than itself
(closed forms, invariants, brute force with unrelated code, a library routine the oracle
does not link).  CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import naive, splitmerge

D = 128
SCALE = 1.0 / math.sqrt(D)


def rand_batch(seed, R, Hq, Hkv, lens, Dh=D, lmax=None):
    g = torch.Generator().manual_seed(seed)
    lmax = lmax or max(max(lens), 1)
    q = torch.randn(R, Hq, Dh, generator=g).to(torch.bfloat16)
    k = torch.randn(R, Hkv, lmax, Dh, generator=g).to(torch.bfloat16)
    v = torch.randn(R, Hkv, lmax, Dh, generator=g).to(torch.bfloat16)
    return q, k, v, torch.tensor(lens, dtype=torch.int32)


def run(q, k, v, lens, Hkv, scale=SCALE, **kw):
    return oracle.decode_attention(q, k, v, lens, num_kv_heads=Hkv, scale=scale, **kw)


# P1 ------------------------------------------------------------------------------------
def test_softmax_weights_sum_to_one_and_lie_in_unit_interval():
    n = 100
    q, k, v, lens = rand_batch(1, 2, 4, 2, [n, 37])
    # V = ones: out = sum_j w_j / S must be 1.
    ones = torch.ones_like(v)
    out, _ = run(q, k, ones, lens, 2)
    assert np.abs(out - 1.0).max() <= n * 1e-16
    # V rows = unit vectors: out[c] = w_c / S is the c-th softmax weight itself.
    eye = torch.zeros_like(v)
    for j in range(n):
        eye[:, :, j, j] = 1.0
    out, _ = run(q, k, eye, lens, 2)
    assert (out >= 0).all() and (out <= 1).all()
    assert np.abs(out.sum(-1) - 1.0).max() <= n * 1e-16
    assert (out[1, :, 37:] == 0).all()          # request 1 only attends 37 tokens


# P2 ------------------------------------------------------------------------------------
def test_single_token_context_returns_v_exactly():
    q, k, v, lens = rand_batch(2, 3, 8, 2, [1, 1, 1], lmax=5)
    out, lse = run(q, k, v, lens, 2)
    G = 4
    for r in range(3):
        for h in range(8):
            g = h // G
            assert np.array_equal(out[r, h], v[r, g, 0].double().numpy())
            s0 = SCALE * float((q[r, h].double() * k[r, g, 0].double()).sum())
            assert abs(lse[r, h] - s0) <= 1e-14


# P3 ------------------------------------------------------------------------------------
def test_uniform_scores_give_mean_of_v():
    n = 77
    q, k, v, lens = rand_batch(3, 2, 4, 1, [n, n])
    q0 = torch.zeros_like(q)
    out, lse = run(q0, k, v, lens, 1)
    mean = v[:, 0, :n].double().mean(1).numpy()
    assert np.abs(out - mean[:, None, :]).max() <= 1e-14
    assert np.abs(lse - math.log(n)).max() <= 1e-14
    # all K rows equal: every score is the same non-zero number s
    k_same = k[:, :, :1].expand(-1, -1, n, -1).contiguous()
    out, lse = run(q, k_same, v, lens, 1)
    assert np.abs(out - mean[:, None, :]).max() <= 1e-13
    for r in range(2):
        for h in range(4):
            s = SCALE * float((q[r, h].double() * k[r, 0, 0].double()).sum())
            assert abs(lse[r, h] - (s + math.log(n))) <= 1e-13


# P4 ------------------------------------------------------------------------------------
@pytest.mark.parametrize("parts_kind", ["even4", "uneven", "sixtyfour", "prev_new",
                                        "with_empty", "interleaved"])
def test_split_then_merge_equals_unsplit(parts_kind):
    n = 300
    q, k, v, lens = rand_batch(4, 1, 4, 2, [n])
    out, lse = run(q, k, v, lens, 2)
    idx = np.arange(n)
    parts = {
        "even4": np.array_split(idx, 4),
        "uneven": [idx[:7], idx[7:200], idx[200:201], idx[201:]],
        "sixtyfour": np.array_split(idx, 64),
        "prev_new": [idx[:-1], idx[-1:]],
        "with_empty": [idx[:150], idx[:0], idx[150:], idx[:0]],
        "interleaved": [idx[0::3], idx[1::3], idx[2::3]],
    }[parts_kind]
    for h in range(4):
        g = h // 2
        K = k[0, g].double().numpy()
        V = v[0, g].double().numpy()
        pr = [splitmerge.partial(q[0, h].double().numpy(), K, V, SCALE, p) for p in parts]
        for merge in (splitmerge.merge_paper_form, splitmerge.merge_lse_form):
            o, l = merge(pr)
            assert np.abs(o - out[0, h]).max() <= 1e-12
            assert abs(l - lse[0, h]) <= 1e-12


def test_merge_of_only_empty_parts_is_the_empty_result():
    o, l = splitmerge.merge_lse_form([(np.zeros(4), -np.inf), (np.zeros(4), -np.inf)])
    assert (o == 0).all() and l == -np.inf


# P5 ------------------------------------------------------------------------------------
@pytest.mark.parametrize("Dh", [4, 128])
def test_literal_per_element_definition_matches(Dh):
    lens = [8, 3]
    q, k, v, lens_t = rand_batch(5, 2, 4, 2, lens, Dh=Dh)
    sc = 1.0 / math.sqrt(Dh)
    out, lse = run(q, k, v, lens_t, 2, scale=sc)
    nout, nlse = naive.decode_attention(q.double().tolist(), k.double().tolist(),
                                        v.double().tolist(), lens, 2, sc)
    assert np.abs(np.array(nout) - out).max() <= 1e-13
    assert np.abs(np.array(nlse) - lse).max() <= 1e-13


# P6 ------------------------------------------------------------------------------------
def test_gqa_equals_mha_on_repeated_kv_and_group_mapping_is_contiguous():
    lens = [50, 64]
    q, k, v, lens_t = rand_batch(6, 2, 8, 2, lens)
    out, lse = run(q, k, v, lens_t, 2)
    k_rep = k.repeat_interleave(4, dim=1).contiguous()     # head h reads kv head h // 4
    v_rep = v.repeat_interleave(4, dim=1).contiguous()
    out_m, lse_m = run(q, k_rep, v_rep, lens_t, 8)
    assert np.array_equal(out, out_m) and np.array_equal(lse, lse_m)
    # identical queries inside one group give identical outputs
    q_same = q.clone()
    q_same[:, 0:4] = q[:, 0:1]
    o, _ = run(q_same, k, v, lens_t, 2)
    for h in range(1, 4):
        assert np.array_equal(o[:, h], o[:, 0])
    # relabelling heads inside a group permutes the outputs the same way
    perm = [2, 0, 3, 1, 4, 5, 6, 7]
    o_p, l_p = run(q[:, perm].contiguous(), k, v, lens_t, 2)
    assert np.array_equal(o_p, out[:, perm]) and np.array_equal(l_p, lse[:, perm])
    # and a head moved ACROSS groups changes its output (kv head really is h // G)
    swapped = q.clone()
    swapped[:, [0, 4]] = q[:, [4, 0]]
    o_s, _ = run(swapped, k, v, lens_t, 2)
    assert not np.allclose(o_s[:, 0], out[:, 4])


# P7 ------------------------------------------------------------------------------------
def test_two_tokens_is_the_logistic_blend():
    q, k, v, lens = rand_batch(7, 4, 2, 1, [2, 2, 2, 2])
    out, lse = run(q, k, v, lens, 1)
    for r in range(4):
        for h in range(2):
            s = [SCALE * float((q[r, h].double() * k[r, 0, j].double()).sum()) for j in (0, 1)]
            sig = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
            ref = sig * v[r, 0, 0].double().numpy() + (1 - sig) * v[r, 0, 1].double().numpy()
            assert np.abs(out[r, h] - ref).max() <= 1e-14
            assert abs(lse[r, h] - (max(s) + math.log1p(math.exp(-abs(s[0] - s[1]))))) <= 1e-14


# P8 ------------------------------------------------------------------------------------
def test_token_permutation_invariance_and_paged_is_bit_identical():
    lens = [45, 16, 33, 1]
    q, k, v, lens_t = rand_batch(8, 4, 4, 2, lens, lmax=48)
    out, lse = run(q, k, v, lens_t, 2)
    g = torch.Generator().manual_seed(80)
    kp, vp = k.clone(), v.clone()
    for r, n in enumerate(lens):
        p = torch.randperm(n, generator=g)
        kp[r, :, :n] = k[r][:, p]
        vp[r, :, :n] = v[r][:, p]
    o2, l2 = run(q, kp, vp, lens_t, 2)
    assert np.abs(o2 - out).max() <= 1e-13 and np.abs(l2 - lse).max() <= 1e-13
    # paged: scatter 16-token blocks into a shuffled pool, tails and spare blocks = NaN
    bs = 16
    nblk = [(n + bs - 1) // bs for n in lens]
    total = sum(nblk) + 3
    ids = torch.randperm(total, generator=g)[:sum(nblk)].tolist()
    pool_k = torch.full((total, 2, bs, D), float("nan"), dtype=torch.bfloat16)
    pool_v = torch.full((total, 2, bs, D), float("nan"), dtype=torch.bfloat16)
    bt = torch.full((4, max(nblk)), -1, dtype=torch.int32)
    it = iter(ids)
    for r, n in enumerate(lens):
        for b in range(nblk[r]):
            blk = next(it)
            bt[r, b] = blk
            m = min(bs, n - b * bs)
            pool_k[blk, :, :m] = k[r, :, b * bs:b * bs + m]
            pool_v[blk, :, :m] = v[r, :, b * bs:b * bs + m]
    o3, l3 = run(q, pool_k, pool_v, lens_t, 2, block_table=bt, block_size=bs)
    assert np.array_equal(o3, out) and np.array_equal(l3, lse)


# P9 ------------------------------------------------------------------------------------
def test_shifting_every_key_moves_lse_only():
    n = 40
    q, k, v, lens = rand_batch(9, 1, 4, 1, [n])
    # a shift that stays exactly representable: keys and shift on a coarse grid
    k = (k.float() * 4).round().div(4).to(torch.bfloat16)
    u = torch.randint(-3, 4, (D,)).float()
    k_shift = (k.float() + u).to(torch.bfloat16)
    assert torch.equal(k_shift.float(), k.float() + u)
    out, lse = run(q, k, v, lens, 1)
    o2, l2 = run(q, k_shift, v, lens, 1)
    assert np.abs(o2 - out).max() <= 1e-13
    for h in range(4):
        c = SCALE * float((q[0, h].double() * u.double()).sum())
        assert abs((l2[0, h] - lse[0, h]) - c) <= 1e-12


# P10 -----------------------------------------------------------------------------------
def test_convex_hull_and_dominant_key():
    n = 64
    q, k, v, lens = rand_batch(10, 2, 4, 2, [n, n])
    out, _ = run(q, k, v, lens, 2)
    for r in range(2):
        for h in range(4):
            V = v[r, h // 2, :n].double().numpy()
            assert (out[r, h] >= V.min(0) - 1e-15).all() and (out[r, h] <= V.max(0) + 1e-15).all()
    # one key aligned with q so that its score is ~60 above all others (which are 0)
    q1 = q[:1, :1].contiguous()
    kk = torch.zeros(1, 1, n, D, dtype=torch.bfloat16)
    qn2 = float((q1[0, 0].double() ** 2).sum())
    c = 60.0 / (SCALE * qn2)
    kk[0, 0, 17] = (q1[0, 0].float() * c).to(torch.bfloat16)
    s17 = SCALE * float((q1[0, 0].double() * kk[0, 0, 17].double()).sum())
    assert s17 > 50
    o, l = run(q1, kk, v[:1, :1].contiguous(), lens[:1], 1)
    bound = n * math.exp(-s17) * 2 * float(v[0, 0, :n].abs().max())
    assert np.abs(o[0, 0] - v[0, 0, 17].double().numpy()).max() <= bound
    assert abs(l[0, 0] - s17) <= n * math.exp(-s17)
    # scores far beyond exp()'s fp64 range still work thanks to the max shift
    kk[0, 0, 17] = (q1[0, 0].float() * (c * 40)).to(torch.bfloat16)
    o, l = run(q1, kk, v[:1, :1].contiguous(), lens[:1], 1)
    assert np.isfinite(o).all() and np.isfinite(l).all() and l[0, 0] > 1500


# P11 -----------------------------------------------------------------------------------
def test_against_torch_cpu_fp64_softmax_and_logsumexp():
    lens = [68, 63, 229, 78]
    q, k, v, lens_t = rand_batch(11, 4, 8, 2, lens)
    out, lse = run(q, k, v, lens_t, 2)
    for r, n in enumerate(lens):
        K = k[r, :, :n].double().repeat_interleave(4, dim=0)      # [Hq][n][D]
        V = v[r, :, :n].double().repeat_interleave(4, dim=0)
        s = torch.einsum("hd,hnd->hn", q[r].double(), K) * SCALE
        ref = torch.einsum("hn,hnd->hd", torch.softmax(s, dim=-1), V)
        assert np.abs(out[r] - ref.numpy()).max() <= 1e-13
        assert np.abs(lse[r] - torch.logsumexp(s, dim=-1).numpy()).max() <= 1e-13


def test_empty_context_gives_zero_and_minus_inf():
    q, k, v, lens = rand_batch(12, 2, 4, 2, [0, 5], lmax=5)
    out, lse = run(q, k, v, lens, 2)
    assert (out[0] == 0).all() and np.isneginf(lse[0]).all()
    assert np.isfinite(out[1]).all() and np.isfinite(lse[1]).all()


# P12 -----------------------------------------------------------------------------------
def test_e4m3fn_decoder_matches_torch_for_all_bytes():
    b = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = b.view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for i in range(256):
        got = oracle.e4m3fn_decode(i)
        if i in (0x7F, 0xFF):
            assert math.isnan(got) and math.isnan(ref[i])
        else:
            assert got == float(ref[i])
    assert oracle.e4m3fn_decode(0x7E) == 448.0 and oracle.e4m3fn_decode(0x01) == 2.0 ** -9
    assert oracle.e4m3fn_decode(0x38) == 1.0 and oracle.e4m3fn_decode(0xB8) == -1.0


def test_e4m3fn_encoder_is_round_to_nearest_even_and_saturates():
    finite = [c for c in range(256) if c not in (0x7F, 0xFF)]
    for c in finite:
        x = oracle.e4m3fn_decode(c)
        if x == 0:
            continue
        assert oracle.e4m3fn_encode(x) == c
    grid = sorted(oracle.e4m3fn_decode(c) for c in range(0x7F))
    rng = np.random.default_rng(12)
    xs = np.concatenate([rng.uniform(-460, 460, 4000), rng.normal(0, 1, 4000),
                         rng.uniform(-0.02, 0.02, 2000)])
    for x in xs:
        got = abs(oracle.e4m3fn_decode(oracle.e4m3fn_encode(x)))
        best = min(abs(abs(x) - gval) for gval in grid)
        assert abs(abs(x) - got) == best
    # exact midpoints go to the even code
    for c in range(0, 0x7E):
        lo, hi = oracle.e4m3fn_decode(c), oracle.e4m3fn_decode(c + 1)
        mid = (lo + hi) / 2
        assert oracle.e4m3fn_encode(mid) == (c if c % 2 == 0 else c + 1)
    assert oracle.e4m3fn_encode(1e9) == 0x7E and oracle.e4m3fn_encode(-1e9) == 0xFE
    # agrees with torch's own cast on in-range values
    x = torch.from_numpy(rng.uniform(-440, 440, 2000).astype(np.float32))
    ref = x.to(torch.float8_e4m3fn).view(torch.uint8).tolist()
    for xi, ri in zip(x.tolist(), ref):
        assert oracle.e4m3fn_encode(xi) & 0x7F == ri & 0x7F


def test_fp8_path_equals_bf16_path_on_the_dequantised_values():
    lens = [40, 17]
    g = torch.Generator().manual_seed(13)
    q = torch.randn(2, 8, D, generator=g).to(torch.bfloat16)
    bytes_k = torch.randint(0, 0x7F, (2, 2, 40, D), generator=g, dtype=torch.int32).to(torch.uint8)
    bytes_v = torch.randint(0x80, 0xFF, (2, 2, 40, D), generator=g, dtype=torch.int32).to(torch.uint8)
    lens_t = torch.tensor(lens, dtype=torch.int32)
    # power-of-two scales keep decode*scale exactly representable in bf16
    ks = torch.tensor([[0.125, 0.0625], [0.03125, 0.125]])
    vs = torch.tensor([[0.0625, 0.125], [0.125, 0.03125]])
    o8, l8 = run(q, bytes_k.view(torch.float8_e4m3fn), bytes_v.view(torch.float8_e4m3fn),
                 lens_t, 2, k_scale=ks, v_scale=vs)
    kd = (bytes_k.view(torch.float8_e4m3fn).float() * ks[:, :, None, None]).to(torch.bfloat16)
    vd = (bytes_v.view(torch.float8_e4m3fn).float() * vs[:, :, None, None]).to(torch.bfloat16)
    assert torch.equal(kd.float(), bytes_k.view(torch.float8_e4m3fn).float() * ks[:, :, None, None])
    o16, l16 = run(q, kd, vd, lens_t, 2)
    assert np.array_equal(o8, o16) and np.array_equal(l8, l16)
    # general fp32 scales: against torch fp64 on decode(byte) * scale
    ks = torch.rand(2, 2, generator=g) * 0.1 + 0.03
    vs = torch.rand(2, 2, generator=g) * 0.1 + 0.03
    o8, l8 = run(q, bytes_k, bytes_v, lens_t, 2, k_scale=ks, v_scale=vs)
    for r, n in enumerate(lens):
        K = (bytes_k.view(torch.float8_e4m3fn)[r, :, :n].double() * ks[r].double()[:, None, None])
        V = (bytes_v.view(torch.float8_e4m3fn)[r, :, :n].double() * vs[r].double()[:, None, None])
        K, V = K.repeat_interleave(4, 0), V.repeat_interleave(4, 0)
        s = torch.einsum("hd,hnd->hn", q[r].double(), K) * SCALE
        ref = torch.einsum("hn,hnd->hd", torch.softmax(s, -1), V)
        assert np.abs(o8[r] - ref.numpy()).max() <= 1e-13
        assert np.abs(l8[r] - torch.logsumexp(s, -1).numpy()).max() <= 1e-13


# P14 -----------------------------------------------------------------------------------
def test_rows_are_independent_of_what_else_is_in_the_batch():
    lens = [30, 70, 5]
    q, k, v, lens_t = rand_batch(14, 3, 8, 2, lens)
    out, lse = run(q, k, v, lens_t, 2)
    pairs = [[2, 7], [0, 0], [1, 5]]
    o, l = run(q, k, v, lens_t, 2, pairs=pairs)
    for i, (r, h) in enumerate(pairs):
        assert np.array_equal(o[i], out[r, h]) and l[i] == lse[r, h]
    # one request alone, with its own tensors
    o1, l1 = run(q[1:2].contiguous(), k[1:2].contiguous(), v[1:2].contiguous(), lens_t[1:2], 2)
    assert np.array_equal(o1[0], out[1]) and np.array_equal(l1[0], lse[1])
    # one kv head alone (its G query heads)
    o2, l2 = run(q[:, 4:8].contiguous(), k[:, 1:2].contiguous(), v[:, 1:2].contiguous(), lens_t, 1)
    assert np.array_equal(o2, out[:, 4:8]) and np.array_equal(l2, lse[:, 4:8])


def test_strided_cache_views_are_honoured():
    lens = [9, 12]
    q, k, v, lens_t = rand_batch(15, 2, 4, 2, lens, lmax=12)
    out, lse = run(q, k, v, lens_t, 2)
    big_k = torch.full((2, 2, 20, 2 * D), float("nan"), dtype=torch.bfloat16)
    big_v = torch.full((2, 2, 20, 2 * D), float("nan"), dtype=torch.bfloat16)
    big_k[:, :, :12, :D] = k
    big_v[:, :, :12, :D] = v
    o, l = run(q, big_k[:, :, :, :D], big_v[:, :, :, :D], lens_t, 2)
    assert np.array_equal(o, out) and np.array_equal(l, lse)


# prev/new split --------------------------------------------------------------------------
def test_fold_new_token_equals_attention_over_all_tokens():
    n = 57
    q, k, v, lens = rand_batch(21, 2, 4, 2, [n, 1])
    out, lse = run(q, k, v, lens, 2)
    prev = torch.tensor([n - 1, 0], dtype=torch.int32)
    po, pl = run(q, k, v, prev, 2)                        # request 1 has no previous tokens
    assert np.isneginf(pl[1]).all()
    for r, m in enumerate([n, 1]):
        for h in range(4):
            g = h // 2
            for merge_input_lse in (pl[r, h],):
                o, l = splitmerge.fold_new_token(q[r, h].double().numpy(),
                                                 k[r, g, m - 1].double().numpy(),
                                                 v[r, g, m - 1].double().numpy(),
                                                 po[r, h], merge_input_lse, SCALE)
                assert np.abs(o - out[r, h]).max() <= 1e-13
                assert abs(l - lse[r, h]) <= 1e-13
