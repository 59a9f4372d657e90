"""Pins for the oracle's block scores and the two selection modes."""
import math

import numpy as np
import pytest

from oracle import dynamicrad_oracle as o


def test_block_score_is_block_mean_of_token_logits():
    """Eq. 9 averaged over the token pairs of a block pair, by explicit loops."""
    rng = np.random.default_rng(1)
    B, H, N, d, Bs, Hf = 2, 3, 22, 5, 8, 2          # ragged tail: blocks of 8, 8, 6
    Q = rng.standard_normal((B, H, N, d))
    K = rng.standard_normal((B, H, N, d))
    got = o.block_scores(Q, K, Bs, Hf)
    Sb = 3
    assert got.shape == (B, 1, Sb, Sb)
    for b in range(B):
        for qb in range(Sb):
            for kb in range(Sb):
                rows = range(qb * Bs, min(N, qb * Bs + Bs))
                cols = range(kb * Bs, min(N, kb * Bs + Bs))
                acc = 0.0
                for p in rows:
                    for q in cols:
                        s = 0.0
                        for h in range(Hf):
                            s += float(np.dot(Q[b, h, p], K[b, h, q])) / math.sqrt(d)
                        acc += s / Hf
                want = acc / (len(rows) * len(cols))
                assert abs(got[b, 0, qb, kb] - want) < 1e-12
    per_head = o.block_scores(Q, K, Bs, 0)
    assert per_head.shape == (B, H, Sb, Sb)
    np.testing.assert_allclose(per_head[:, :2].mean(axis=1, keepdims=True), got, atol=1e-13)


def test_block_score_special_cases():
    N, d, Bs = 16, 4, 4
    Q = np.ones((1, 2, N, d))
    K = np.full((1, 2, N, d), 2.0)
    s = o.block_scores(Q, K, Bs, 2)
    np.testing.assert_allclose(s, 2.0 * d / math.sqrt(d))
    # block size 1: the score map is the plain logit matrix
    rng = np.random.default_rng(2)
    Q = rng.standard_normal((1, 1, 7, 3))
    K = rng.standard_normal((1, 1, 7, 3))
    np.testing.assert_allclose(o.block_scores(Q, K, 1, 1)[0, 0], Q[0, 0] @ K[0, 0].T / math.sqrt(3), atol=1e-14)
    # transposed operands would break this asymmetry
    Q = np.zeros((1, 1, 8, 2)); K = np.zeros((1, 1, 8, 2))
    Q[0, 0, :4, 0] = 1.0            # query block 0 lights channel 0
    K[0, 0, 4:, 0] = 3.0            # key block 1 lights channel 0
    s = o.block_scores(Q, K, 4, 1)[0, 0]
    assert s[0, 1] == pytest.approx(3.0 / math.sqrt(2)) and s[1, 0] == 0.0


def _row(n_forced=2, n_sel=9, n_none=3, seed=0):
    rng = np.random.default_rng(seed)
    cls = np.array([o.CLASS_FORCED] * n_forced + [o.CLASS_NEAR] * n_sel + [o.CLASS_NONE] * n_none, dtype=np.uint8)
    rng.shuffle(cls)
    s = rng.standard_normal(len(cls)).astype(np.float32)
    return s, cls


def test_static_topk_properties():
    for seed in range(20):
        s, cls = _row(seed=seed, n_sel=5 + seed)
        n = int(((cls == 1) | (cls == 2)).sum())
        for rho in (0.05, 0.2, 0.5, 0.99, 1.0):
            kept = o.select_static(s, cls, rho)
            sel = [k for k in kept if cls[k] != o.CLASS_FORCED]
            assert set(np.flatnonzero(cls == o.CLASS_FORCED)) <= set(kept)
            assert all(cls[k] != o.CLASS_NONE for k in kept)
            assert len(sel) == max(1, math.floor(n * rho))
            unsel = [k for k in np.flatnonzero((cls == 1) | (cls == 2)) if k not in sel]
            if sel and unsel:
                assert min(s[sel]) >= max(s[unsel])
            assert list(kept) == sorted(kept)
            # brute force: full python sort with the documented total order
            order = sorted(np.flatnonzero((cls == 1) | (cls == 2)), key=lambda k: (-float(s[k]), k))
            assert sorted(sel) == sorted(order[:len(sel)])
        # rho = 1 keeps the whole candidate set
        assert list(o.select_static(s, cls, 1.0)) == list(np.flatnonzero(cls > 0))


def test_static_empty_and_ties_and_negative_zero():
    s = np.zeros(6, dtype=np.float32)
    cls = np.array([3, 0, 0, 3, 0, 0], dtype=np.uint8)
    assert list(o.select_static(s, cls, 0.5)) == [0, 3]                 # nothing selectable: forced only
    cls = np.array([1, 1, 1, 1, 1, 1], dtype=np.uint8)
    assert list(o.select_static(s, cls, 0.5)) == [0, 1, 2]              # all equal: lowest indices
    s = np.array([0.0, -0.0, 0.0, -0.0, 1.0, -1.0], dtype=np.float32)
    assert list(o.select_static(s, cls, 0.5)) == [0, 1, 4]              # -0 == +0, index breaks the tie
    assert list(o.select_static(s, cls, 0.01)) == [4]                   # k = max(1, 0)


def test_static_two_ratios_apply_per_class():
    s = np.array([5, 4, 3, 2, 1, 0, 9, 8, 7, 6], dtype=np.float32)
    cls = np.array([1, 1, 1, 1, 2, 2, 2, 2, 2, 3], dtype=np.uint8)
    kept = o.select_static(s, cls, 0.5, 0.4)        # near: floor(4*.5)=2 -> {0,1}; far: floor(5*.4)=2 -> {6,7}
    assert list(kept) == [0, 1, 6, 7, 9]
    assert list(o.select_static(s, cls, 0.5, -1.0)) == [0, 6, 7, 8, 9]   # single ratio: floor(9*.5)=4 of the union


def test_dynamic_prefix_properties():
    for seed in range(20):
        s, cls = _row(seed=100 + seed, n_sel=4 + seed)
        selectable = np.flatnonzero((cls == 1) | (cls == 2))
        order = sorted(selectable, key=lambda k: (-float(s[k]), k))
        m = float(s[order[0]])
        e = np.array([math.exp(float(s[k]) - m) for k in order])
        cum = np.cumsum(e)            # sequential in order
        for tau in (1e-9, 0.3, 0.9, 0.95, 1.0):
            kept = o.select_dynamic(s, cls, tau)
            sel = [k for k in kept if cls[k] != o.CLASS_FORCED]
            k = len(sel)
            assert sorted(sel) == sorted(order[:k])              # a prefix of the total order
            assert k >= 1
            Z = cum[-1]
            assert cum[k - 1] >= tau * Z * (1 - 1e-15)
            if k > 1:
                assert cum[k - 2] < tau * Z * (1 + 1e-15)       # minimal
        assert len([k for k in o.select_dynamic(s, cls, 1.0) if cls[k] != 3]) == len(selectable)
        assert len([k for k in o.select_dynamic(s, cls, 1e-12) if cls[k] != 3]) == 1


def test_dynamic_equal_scores_keep_ceil_tau_n_lowest_indices():
    n = 10
    s = np.full(n, 0.25, dtype=np.float32)
    cls = np.full(n, o.CLASS_FAR, dtype=np.uint8)
    for tau, want in ((0.31, 4), (0.5, 5), (0.05, 1), (0.95, 10), (0.9, 9)):
        kept = o.select_dynamic(s, cls, tau)
        assert list(kept) == list(range(want)), tau


def test_dynamic_closed_form_geometric_scores():
    # scores 0, -ln2, -2ln2, ...: masses 1, 1/2, 1/4, ...; cumulative 2 - 2^-k; Z = 2 - 2^-(n-1)
    n = 12
    s = np.array([-k * math.log(2.0) for k in range(n)], dtype=np.float32)
    cls = np.full(n, o.CLASS_NEAR, dtype=np.uint8)
    kept = o.select_dynamic(s, cls, 0.9)      # need 2 - 2^-(k-1) >= 0.9 * 1.99951 = 1.79956 -> k = 4 (1.875)
    assert list(kept) == [0, 1, 2, 3]
    kept = o.select_dynamic(s[::-1].copy(), cls, 0.9)
    assert list(kept) == [n - 4, n - 3, n - 2, n - 1]


def test_dynamic_no_selectable():
    s = np.zeros(4, dtype=np.float32)
    cls = np.array([3, 3, 0, 0], dtype=np.uint8)
    assert list(o.select_dynamic(s, cls, 0.9)) == [0, 1]


def test_build_mask_csr_and_sparsity():
    rng = np.random.default_rng(3)
    Nf, Nt, Bs = 8, 64, 32
    N = Nf * Nt
    tab = o.frame_table(Nf, Nt, Bs, 1.0, 1.0)
    cm = o.classify_blocks(N, Nt, Bs, tab, 0.15, 0.6)
    Sb = cm.shape[0]
    sc = rng.standard_normal((2, 1, Sb, Sb)).astype(np.float32)
    for mode, par in (("static", 0.3), ("dynamic", 0.8)):
        masks = o.build_mask(sc, cm, mode, par)
        for b in range(2):
            rowptr, colidx = masks[b][0]
            assert rowptr[0] == 0 and len(colidx) == rowptr[-1]
            M = o.csr_to_token_mask(rowptr, colidx, Bs, N)
            # effective sparsity = pruned fraction of block pairs = 1 - mean of the broadcast token mask
            assert o.effective_sparsity(rowptr, Sb) == pytest.approx(1.0 - M.mean(), abs=1e-15)
            for qb in range(Sb):
                row = colidx[rowptr[qb]:rowptr[qb + 1]]
                assert (np.diff(row) > 0).all()
                assert (cm[qb, row] > 0).all()
                assert set(np.flatnonzero(cm[qb] == o.CLASS_FORCED)) <= set(row)
    # rho = 1 / tau = 1 reproduce the candidate set
    for mode in ("static", "dynamic"):
        rowptr, colidx = o.build_mask(sc, cm, mode, 1.0)[0][0]
        assert rowptr[-1] == (cm > 0).sum()


def test_ratio_for_target_sparsity():
    Nf, Nt, Bs = 24, 64, 32
    N = Nf * Nt
    tab = o.frame_table(Nf, Nt, Bs, 1.0, 1.0)
    cm = o.classify_blocks(N, Nt, Bs, tab, 0.15, 0.6)
    Sb = cm.shape[0]
    forced_frac = (cm == 3).sum() / Sb ** 2
    target = 1.0 - forced_frac - 0.03
    rho = o.ratio_for_target_sparsity(cm, target)
    sc = np.random.default_rng(4).standard_normal((1, 1, Sb, Sb)).astype(np.float32)
    rp, _ = o.build_mask(sc, cm, "static", rho)[0][0]
    assert o.effective_sparsity(rp, Sb) >= target
    rp2, _ = o.build_mask(sc, cm, "static", rho + 1e-3)[0][0]
    assert o.effective_sparsity(rp2, Sb) < target or rho + 1e-3 > 1.0
    with pytest.raises(ValueError):
        o.ratio_for_target_sparsity(cm, 1.0 - forced_frac + 0.01)
