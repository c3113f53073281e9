"""Partial attention results and their combination -- TEST INFRASTRUCTURE ONLY.

Paper Sec. 4.2.2: for disjoint index sets I1, I2 with I = I1 u I2,

    A_q(I) = (A_q(I1) S_q(I1) + A_q(I2) S_q(I2)) / (S_q(I1) + S_q(I2)).

By induction the same holds for any number of parts.  The GPU library stores
ln S_q(I) instead of S_q(I); both forms of the combination are written out here so the
tests can check that they agree with each other and with the unsplit definition.
All arithmetic is numpy fp64 over one (query row, K matrix, V matrix) at a time.
"""
from __future__ import annotations

import numpy as np


def partial(q_row, K, V, scale, idx):
    """(A_q(I), ln S_q(I)) over the token rows listed in idx; empty I -> (0, -inf)."""
    idx = np.asarray(idx, dtype=np.int64)
    D = V.shape[1]
    if idx.size == 0:
        return np.zeros(D), -np.inf
    s = scale * (K[idx].astype(np.float64) @ np.asarray(q_row, dtype=np.float64))
    m = s.max()
    w = np.exp(s - m)
    S = w.sum()
    return (w @ V[idx].astype(np.float64)) / S, m + np.log(S)


def merge_paper_form(parts):
    """sum_p A_p S_p / sum_p S_p with S_p = exp(lse_p) taken unshifted, as printed."""
    num = 0.0
    den = 0.0
    for A, lse in parts:
        S = np.exp(lse)           # exp(-inf) = 0: empty parts drop out
        num = num + A * S
        den = den + S
    return num / den, np.log(den)


def merge_lse_form(parts):
    """lse = ln sum_p e^{lse_p};  out = sum_p e^{lse_p - lse} A_p  (shift-safe)."""
    lses = np.array([lse for _, lse in parts], dtype=np.float64)
    top = lses.max()
    if not np.isfinite(top):
        return np.zeros_like(parts[0][0]), -np.inf
    lse = top + np.log(np.exp(lses - top).sum())
    out = 0.0
    for A, l in parts:
        out = out + np.exp(l - lse) * A
    return out, lse


def fold_new_token(q_row, k_new, v_new, out_prev, lse_prev, scale):
    """The prev/new split of Sec. 4.2.2: I = prev u {new}.  The new token alone has
    A_q({new}) = v_new and ln S_q({new}) = scale * <q, k_new>; combine it with the given
    (A_q(prev), ln S_q(prev)).  Returns (A_q(I), ln S_q(I))."""
    s = scale * float(np.dot(np.asarray(q_row, dtype=np.float64), np.asarray(k_new, dtype=np.float64)))
    return merge_lse_form([(np.asarray(out_prev, dtype=np.float64), float(lse_prev)),
                           (np.asarray(v_new, dtype=np.float64), s)])
