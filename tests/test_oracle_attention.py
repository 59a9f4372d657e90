"""Pins for the oracle's masked attention (Eq. 13 with epsilon -> 0)."""
import math

import numpy as np
import pytest
import torch

from oracle import dynamicrad_oracle as o


def _qkv(N, d, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, d)), rng.standard_normal((N, d)), rng.standard_normal((N, d)))


def _assemble(blocks, N, d, Bs):
    O = np.zeros((N, d))
    for qb, blk in blocks.items():
        O[qb * Bs: qb * Bs + blk.shape[0]] = blk
    return O


def test_full_mask_equals_dense_attention_library():
    N, d, Bs = 45, 8, 16      # ragged tail
    Q, K, V = _qkv(N, d, 0)
    rp, ci = o.full_csr(3)
    got = _assemble(o.masked_attention(Q, K, V, rp, ci, Bs), N, d, Bs)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0].numpy()
    np.testing.assert_allclose(got, want, atol=1e-12)
    np.testing.assert_allclose(got, o.dense_attention_bruteforce(Q, K, V), atol=1e-12)


def test_masked_equals_bruteforce_with_minus_inf_mask():
    N, d, Bs = 40, 6, 8
    Q, K, V = _qkv(N, d, 1)
    rng = np.random.default_rng(5)
    Sb = 5
    dense = rng.random((Sb, Sb)) < 0.5
    dense[np.arange(Sb), np.arange(Sb)] = True
    rowptr = np.zeros(Sb + 1, dtype=np.int64)
    cols = []
    for qb in range(Sb):
        c = np.flatnonzero(dense[qb])
        cols.append(c)
        rowptr[qb + 1] = rowptr[qb] + len(c)
    colidx = np.concatenate(cols)
    got = _assemble(o.masked_attention(Q, K, V, rowptr, colidx, Bs), N, d, Bs)
    M = o.csr_to_token_mask(rowptr, colidx, Bs, N)
    np.testing.assert_allclose(got, o.dense_attention_bruteforce(Q, K, V, M), atol=1e-12)
    # library third opinion with an additive -inf mask
    add = torch.where(torch.from_numpy(M), 0.0, -math.inf).to(torch.float64)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None], attn_mask=add[None])[0]
    np.testing.assert_allclose(got, want.numpy(), atol=1e-12)


def test_constant_value_and_block_order_invariance_and_lse():
    N, d, Bs = 64, 4, 16
    Q, K, V = _qkv(N, d, 2)
    rowptr = np.array([0, 2, 4, 7, 9])
    colidx = np.array([0, 1, 1, 3, 0, 2, 3, 1, 3])
    Vc = np.full((N, d), 0.75)
    for blk in o.masked_attention(Q, K, Vc, rowptr, colidx, Bs).values():
        np.testing.assert_allclose(blk, 0.75, atol=1e-14)       # weights sum to one
    a = o.masked_attention(Q, K, V, rowptr, colidx, Bs)
    perm = np.array([1, 0, 3, 1, 3, 2, 0, 3, 1])                # same sets, other order
    b = o.masked_attention(Q, K, V, rowptr, perm, Bs)
    for qb in a:
        np.testing.assert_allclose(a[qb], b[qb], atol=1e-13)
    out, lse = o.masked_attention(Q, K, V, rowptr, colidx, Bs, return_lse=True)
    keys = np.r_[0:16, 16:32]
    ref = np.log(np.exp(Q[:16] @ K[keys].T / 2.0).sum(axis=1))
    np.testing.assert_allclose(lse[0], ref, atol=1e-12)


def test_scale_and_sign_conventions():
    # one query, two keys: weights softmax([q.k0, q.k1] / sqrt(d)); checks the 1/sqrt(d) scale explicitly
    d = 4
    Q = np.array([[1.0, 0, 0, 0]]); K = np.array([[2.0, 0, 0, 0], [0.0, 0, 0, 0]]); V = np.array([[1.0] * d, [0.0] * d])
    Qp = np.vstack([Q, np.zeros((1, d))])
    rp, ci = np.array([0, 1]), np.array([0])
    out = o.masked_attention(Qp, K, V, rp, ci, 2)[0]
    w = math.exp(1.0) / (math.exp(1.0) + 1.0)                   # logits 2/sqrt(4) = 1 and 0
    np.testing.assert_allclose(out[0], w, atol=1e-15)
    np.testing.assert_allclose(out[1], 0.5, atol=1e-15)


def test_rows_subset_and_empty_row():
    N, d, Bs = 32, 4, 8
    Q, K, V = _qkv(N, d, 3)
    rowptr = np.array([0, 1, 1, 3, 4])
    colidx = np.array([0, 1, 2, 3])
    full = o.masked_attention(Q, K, V, rowptr, colidx, Bs)
    sub = o.masked_attention(Q, K, V, rowptr, colidx, Bs, rows=[2])
    assert list(sub) == [2]
    np.testing.assert_array_equal(sub[2], full[2])
    assert (full[1] == 0).all()
