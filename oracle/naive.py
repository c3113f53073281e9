"""Literal evaluator of the partial-result definitions -- TEST INFRASTRUCTURE ONLY.

Paper Sec. 4.2.2 defines, for a query q and a token index set I,

    S_q(I) = sum_{i in I} exp(q.k_i / sqrt(d))
    A_q(I) = sum_{i in I} softmax(q.k_i / sqrt(d)) v_i        (softmax normalised by S_q(I))

This module evaluates exactly that, one output element at a time, in Python floats
(fp64), with NO max shift and no shared intermediate between output elements: every
element recomputes every score.  It is quadratic-ish and only meant for tiny inputs,
where it pins the C oracle with code that has nothing in common with it.
"""
from __future__ import annotations

import math


def scores(q_row, k_rows, scale):
    """[scale * <q, k_i>] for every row k_i; plain Python floats."""
    return [scale * sum(float(a) * float(b) for a, b in zip(q_row, k)) for k in k_rows]


def S_q(q_row, k_rows, scale):
    """Softmax denominator over the given rows, unshifted."""
    return sum(math.exp(s) for s in scores(q_row, k_rows, scale))


def A_q_element(q_row, k_rows, v_rows, scale, c):
    """Element c of the attention output over the given rows."""
    denom = S_q(q_row, k_rows, scale)
    num = 0.0
    for i, k in enumerate(k_rows):
        s_i = scale * sum(float(a) * float(b) for a, b in zip(q_row, k))
        num += math.exp(s_i) * float(v_rows[i][c])
    return num / denom


def decode_attention(q, k, v, seq_lens, num_kv_heads, scale):
    """q [R][Hq][D], k/v [R][Hkv][L][D] nested sequences (or arrays) of floats.

    Query head h reads kv head h // G with G = Hq // Hkv (Sec. 2.2.2: the G queries of
    a group share one k/v and their outputs are concatenated).  Returns nested lists
    out[R][Hq][D], lse[R][Hq] with lse = ln S_q(I).
    """
    R = len(q)
    Hq = len(q[0])
    D = len(q[0][0])
    G = Hq // num_kv_heads
    out, lse = [], []
    for r in range(R):
        n = int(seq_lens[r])
        out_r, lse_r = [], []
        for h in range(Hq):
            g = h // G
            k_rows = [k[r][g][j] for j in range(n)]
            v_rows = [v[r][g][j] for j in range(n)]
            out_r.append([A_q_element(q[r][h], k_rows, v_rows, scale, c) for c in range(D)])
            lse_r.append(math.log(S_q(q[r][h], k_rows, scale)))
        out.append(out_r)
        lse.append(lse_r)
    return out, lse
