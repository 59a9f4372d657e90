"""Pins for the proxy-task utilities: the drift generator's statistics and the search objective (App. C, Eq. 22)."""
import math

import numpy as np

from oracle import dynamicrad_oracle as o
from workloads import make_ar1_proxy


def test_ar1_proxy_has_the_closed_form_autocorrelation():
    """Stationary AR(1): E[h_t . h_{t+k}] / D = (1 - delta^2)^(k/2); unit variance at every frame."""
    Nf, Nt, D = 12, 64, 64
    for delta in (0.02, 0.15, 0.40):
        h = make_ar1_proxy(Nf, Nt, D, delta, seed=3).astype(np.float64).reshape(Nf, Nt, D)
        n = Nt * D
        for t in range(Nf):
            assert abs((h[t] ** 2).mean() - 1.0) < 6.0 * math.sqrt(2.0 / n)
        for k in (1, 3, 7):
            want = (1.0 - delta * delta) ** (k / 2.0)
            got = np.mean([(h[t] * h[t + k]).mean() for t in range(Nf - k)])
            assert abs(got - want) < 6.0 / math.sqrt(n), (delta, k, got, want)
    a = make_ar1_proxy(4, 8, 8, 0.15, seed=1)
    assert (a == make_ar1_proxy(4, 8, 8, 0.15, seed=1)).all() and (a != make_ar1_proxy(4, 8, 8, 0.15, seed=2)).any()
    assert a.dtype == np.float32 and a.shape == (32, 8)


def test_attention_matrix_rows_and_mask():
    rng = np.random.default_rng(0)
    N, d, Bs = 12, 4, 4
    Q, K = rng.standard_normal((N, d)), rng.standard_normal((N, d))
    A = o.attention_matrix(Q, K)
    np.testing.assert_allclose(A.sum(axis=1), 1.0, atol=1e-13)
    # same weights as the attention routine: A V = O for any V
    V = rng.standard_normal((N, d))
    rp, ci = o.full_csr(3)
    np.testing.assert_allclose(A @ V, np.concatenate(list(o.masked_attention(Q, K, V, rp, ci, Bs).values())), atol=1e-12)
    # block-diagonal mask plus one empty row block
    rp = np.array([0, 1, 2, 2])
    ci = np.array([0, 1])
    Am = o.attention_matrix(Q, K, rp, ci, Bs)
    assert (Am[8:] == 0).all() and (Am[:4, 4:] == 0).all() and (Am[4:8, :4] == 0).all()
    np.testing.assert_allclose(Am[:8].sum(axis=1), 1.0, atol=1e-13)
    # inside a kept block the weights are the dense ones renormalised
    np.testing.assert_allclose(Am[:4, :4], A[:4, :4] / A[:4, :4].sum(axis=1, keepdims=True), atol=1e-13)


def test_proxy_loss_closed_forms():
    """Two tokens, logits a (self) and b (other): dense rows softmax(a, b) = (p, 1 - p); keeping only the diagonal
    gives the identity.  ||A - I||^2 = 2 * 2 (1-p)^2, ||A||^2 = 2 (p^2 + (1-p)^2)."""
    p = 1.0 / (1.0 + math.exp(-1.5))
    A = np.array([[p, 1 - p], [1 - p, p]])
    loss, nmse = o.proxy_loss(A, np.eye(2), sparsity=0.5)
    want = 2 * (1 - p) ** 2 / (p ** 2 + (1 - p) ** 2)
    assert abs(nmse - want) < 1e-15
    assert abs(loss - (want + 10.0 * 0.3)) < 1e-12          # sparsity 0.5 misses the 0.80 target by 0.3
    assert o.proxy_loss(A, A, sparsity=0.0) == (8.0, 0.0)    # exact reconstruction, no sparsity: pure penalty
    assert o.proxy_loss(A, A, sparsity=0.9) == (0.0, 0.0)    # target met: no penalty
    loss2, _ = o.proxy_loss(A, np.eye(2), sparsity=0.5, target=0.6, alpha=2.0)
    assert abs(loss2 - (want + 0.2)) < 1e-12


def test_sparser_masks_lose_more_and_slow_drift_is_more_temporal():
    """Sanity of the whole proxy chain on the oracle: dropping kept blocks can only move attention mass away, and the
    share of dense attention mass that crosses frames grows as the drift delta shrinks."""
    Nf, Nt, D, Bs = 6, 16, 32, 8
    N = Nf * Nt
    frame = np.arange(N) // Nt
    cross = []
    for delta in (0.40, 0.15, 0.02):
        h = make_ar1_proxy(Nf, Nt, D, delta, seed=5).astype(np.float64)
        A = o.attention_matrix(h, h)
        cross.append(float(A[frame[:, None] != frame[None, :]].sum() / N))
    assert cross[0] < cross[1] < cross[2]
    tab = o.frame_table(Nf, Nt, Bs, 2.0, 1.0)
    cls = o.classify_blocks(N, Nt, Bs, tab, 0.15, 0.60)
    scores = o.block_scores(h[None, None], h[None, None], Bs, 1).astype(np.float32)
    prev = -1.0
    for rho in (1.0, 0.5, 0.1):
        rp, ci = o.build_mask(scores, cls, "static", rho)[0][0]
        _, nmse = o.proxy_loss(A, o.attention_matrix(h, h, rp, ci, Bs), o.effective_sparsity(rp, N // Bs))
        assert nmse >= prev - 1e-12
        prev = nmse
