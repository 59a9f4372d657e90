"""Pins for the oracle's statement of Algorithm 1 in the paper's own order: token links chosen inside every frame
pair's candidate set by standardised score (Eqs. 7, 9-11), then aggregated to blocks by the density rule."""
import math

import numpy as np
import pytest

from oracle import dynamicrad_oracle as o


def _tab(Nf, Nt, Bs, gamma=1.0, lam=1.0):
    return o.frame_table(Nf, Nt, Bs, gamma, lam)


def _block_keep(csr, Sb):
    rp, ci = csr
    keep = np.zeros((Sb, Sb), dtype=bool)
    for qb in range(Sb):
        keep[qb, ci[rp[qb]:rp[qb + 1]]] = True
    return keep


# ------------------------------------------------------------------ token scores
def test_token_scores_against_explicit_loops_and_block_mean():
    """Eq. 9 pair by pair; and the pooled block score is the mean of the token scores of the block pair."""
    rng = np.random.default_rng(1)
    B, H, N, d, Bs = 2, 3, 24, 8, 8
    Q, K = rng.standard_normal((B, H, N, d)), rng.standard_normal((B, H, N, d))
    for hf in (2, 0):
        S = o.token_scores(Q, K, hf)
        heads = [range(hf)] if hf else [[h] for h in range(H)]
        assert S.shape == (B, len(heads), N, N)
        for b in range(B):
            for m, hs in enumerate(heads):
                for p in (0, 5, 23):
                    for q in (0, 7, 22):
                        want = sum(sum(Q[b, h, p, c] * K[b, h, q, c] for c in range(d)) for h in hs) / len(hs) / math.sqrt(d)
                        assert abs(S[b, m, p, q] - want) < 1e-12
        pooled = o.block_scores(Q, K, Bs, hf)
        means = S.reshape(B, -1, N // Bs, Bs, N // Bs, Bs).mean(axis=(3, 5))
        assert np.abs(pooled - means).max() < 1e-12


# ------------------------------------------------------------------ summation order
def test_summation_order_is_columns_first_one_by_one():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((37, 23)) * 10.0 ** rng.integers(-6, 6, size=(37, 23))).astype(np.float64)
    total = 0.0
    for v in range(x.shape[1]):
        col = 0.0
        for u in range(x.shape[0]):
            col = col + x[u, v]
        total = total + col
    assert o._sum_columns_then_across(x) == total
    rows_first = 0.0
    for u in range(x.shape[0]):
        r = 0.0
        for v in range(x.shape[1]):
            r = r + x[u, v]
        rows_first = rows_first + r
    assert rows_first != total, "the example must be able to tell the two orders apart"


# ------------------------------------------------------------------ links per frame pair
def _links_by_enumeration(S, N, Nt, tab, tau_near, tau_far, eps=1e-6):
    """Second route: the candidate set of a frame pair as an explicit list, numpy's mean / std on it."""
    Nf = N // Nt
    links = np.zeros((N, N), dtype=bool)
    margin = np.inf
    for i in range(Nf):
        for j in range(Nf):
            t = abs(i - j)
            pairs = [(u, v) for u in range(Nt) for v in range(Nt)
                     if o.token_candidate(i * Nt + u, j * Nt + v, Nt, tab)]
            if t <= 1:
                assert len(pairs) == Nt * Nt
                links[i * Nt:(i + 1) * Nt, j * Nt:(j + 1) * Nt] = True
                continue
            if not pairs:
                continue
            vals = np.array([float(S[i * Nt + u, j * Nt + v]) for u, v in pairs])
            z = (vals - vals.mean()) / (vals.std() + eps)
            tau = tau_near if tab["cls"][t] == o.CLASS_NEAR else tau_far
            if np.isfinite(tau):
                margin = min(margin, float(np.abs(z - tau).min()))
            kept = [pr for pr, zz in zip(pairs, z) if zz >= tau]
            if not kept:
                kept = [pairs[int(np.argmax(vals))]]
            for u, v in kept:
                links[i * Nt + u, j * Nt + v] = True
    return links, margin


@pytest.mark.parametrize("Nf,Nt,Bs,gamma,lam", [(6, 12, 4, 1.0, 1.0), (7, 10, 4, 3.0, 0.5), (9, 8, 2, 2.0, 0.3)])
def test_links_match_enumeration_with_library_statistics(Nf, Nt, Bs, gamma, lam):
    tab = _tab(Nf, Nt, Bs, gamma, lam)
    N = Nf * Nt
    rng = np.random.default_rng(Nf * 100 + Nt)
    S = rng.standard_normal((N, N)).astype(np.float32)
    assert tab["retained"][2:].any()
    for tau_near, tau_far in ((0.0, 0.0), (0.7, -0.3), (-1.0, 1.5), (-np.inf, -np.inf), (50.0, 50.0)):
        want, margin = _links_by_enumeration(S, N, Nt, tab, tau_near, tau_far)
        assert margin > 1e-9, "example sits on a threshold"
        got = o.select_token_links(S, N, Nt, tab, tau_near, tau_far)
        assert (got == want).all()


def test_links_hand_example():
    """Three frames of two tokens; the pair (0, 2) holds the scores 1, 2, 3, 4 and the window covers all four:
    mu = 2.5, population sigma = sqrt(1.25), z = -1.342, -0.447, 0.447, 1.342 (Eq. 10; a sample deviation would give
    0.387 for the third)."""
    tab = _tab(3, 2, 1, gamma=4.0, lam=4.0)
    assert tab["retained"][2] and tab["w"][2] >= 1
    S = np.zeros((6, 6), dtype=np.float32)
    S[0:2, 4:6] = [[1, 2], [3, 4]]
    S[4:6, 0:2] = [[4, 1], [2, 3]]
    links = o.select_token_links(S, 6, 2, tab, 0.42, 0.42)
    assert links[0:2, 4:6].tolist() == [[False, False], [True, True]]
    assert links[4:6, 0:2].tolist() == [[True, False], [False, True]]
    assert links[0:4, 0:4].all() and links[2:6, 2:6].all()
    assert o.select_token_links(S, 6, 2, tab, 1.0, 1.0)[0:2, 4:6].tolist() == [[False, False], [False, True]]
    z4 = 1.5 / (math.sqrt(1.25) + 1e-6)
    assert o.select_token_links(S, 6, 2, tab, z4, z4)[0:2, 4:6].sum() == 1        # inclusive boundary
    assert o.select_token_links(S, 6, 2, tab, -0.45, -0.45)[0:2, 4:6].sum() == 3


def test_links_exact_on_integer_scores_and_symmetric():
    """Integer scores make every sum exact, so any summation order gives the same statistics: the links must then
    equal the enumeration bit for bit, and a symmetric score matrix must give a symmetric link matrix."""
    Nf, Nt, Bs = 6, 10, 4
    tab = _tab(Nf, Nt, Bs, 2.0, 1.0)
    N = Nf * Nt
    rng = np.random.default_rng(3)
    A = rng.integers(-8, 9, size=(N, N))
    S = (A + A.T).astype(np.float32)
    for tau in (0.25, 1.0):
        got = o.select_token_links(S, N, Nt, tab, tau, tau)
        want, _ = _links_by_enumeration(S, N, Nt, tab, tau, tau)
        assert (got == want).all()
        assert (got == got.T).all()


def test_constant_scores_and_the_keep_one_fallback():
    """sigma = 0 gives z = 0: tau <= 0 keeps the whole candidate set (Eq. 7), tau > 0 keeps nothing, and the
    safeguard then keeps the first pair of the set, (u, v) = (0, 0)."""
    Nf, Nt, Bs = 6, 12, 4
    tab = _tab(Nf, Nt, Bs)
    N = Nf * Nt
    S = np.full((N, N), 0.375, dtype=np.float32)
    assert (o.select_token_links(S, N, Nt, tab, 0.0, 0.0) == o.candidate_matrix(N, Nt, tab)).all()
    assert (o.select_token_links(S, N, Nt, tab, -3.0, -3.0) == o.candidate_matrix(N, Nt, tab)).all()
    links = o.select_token_links(S, N, Nt, tab, 0.5, 0.5)
    for i in range(Nf):
        for j in range(Nf):
            t = abs(i - j)
            blk = links[i * Nt:(i + 1) * Nt, j * Nt:(j + 1) * Nt]
            if t <= 1:
                assert blk.all()
            elif tab["retained"][t]:
                assert blk.sum() == 1 and blk[0, 0]
            else:
                assert not blk.any()


def test_fallback_keeps_the_highest_score_of_the_set():
    Nf, Nt, Bs = 5, 9, 2
    tab = _tab(Nf, Nt, Bs)
    N = Nf * Nt
    rng = np.random.default_rng(4)
    S = rng.standard_normal((N, N)).astype(np.float32)
    links = o.select_token_links(S, N, Nt, tab, 1e9, 1e9)
    cand = o.candidate_matrix(N, Nt, tab)
    for i in range(Nf):
        for j in range(Nf):
            if abs(i - j) >= 2 and tab["retained"][abs(i - j)]:
                sl = (slice(i * Nt, (i + 1) * Nt), slice(j * Nt, (j + 1) * Nt))
                assert links[sl].sum() == 1
                assert S[sl][links[sl]][0] == S[sl][cand[sl]].max()


def test_planted_stripe_is_what_survives_a_high_threshold():
    """Scores that are large exactly on u == v: with tau = 1 the kept links of every retained frame pair are the
    stripe (its z is about sqrt((n - Nt) / Nt) >> 1, the rest sit below the mean)."""
    Nf, Nt, Bs = 6, 16, 4
    tab = _tab(Nf, Nt, Bs, 2.0, 1.0)
    N = Nf * Nt
    rng = np.random.default_rng(5)
    S = (0.01 * rng.standard_normal((N, N))).astype(np.float32)
    u = np.arange(N) % Nt
    S[u[:, None] == u[None, :]] += 5.0
    links = o.select_token_links(S, N, Nt, tab, 1.0, 1.0)
    frame = np.arange(N) // Nt
    t = np.abs(frame[:, None] - frame[None, :])
    want = (t <= 1) | (tab["retained"][t] & (u[:, None] == u[None, :]))
    assert (links == want).all()


# ------------------------------------------------------------------ aggregation to blocks
def test_aggregation_hand_example_and_strictness():
    """One far block of 4 x 4 (rows 0-3 = frame 0, columns = frame 3).  Column counts 4, 2, 1, 0 of 4 rows:
    ratios 1, .5, .25, 0.  theta_c = .25 -> columns 0, 1 active (strict >) -> 2/4 = .5 active."""
    N, Nt, Bs = 16, 4, 4
    links = np.zeros((N, N), dtype=bool)
    links[0:4, 12] = True
    links[0:2, 13] = True
    links[3, 14] = True
    assert o.aggregate_links(links, N, Nt, Bs, 0.25, 0.49)[0, 3]
    assert not o.aggregate_links(links, N, Nt, Bs, 0.25, 0.5)[0, 3]          # .5 does not exceed .5
    assert o.aggregate_links(links, N, Nt, Bs, 0.24, 0.5)[0, 3]              # column 2 now active: 3/4
    assert not o.aggregate_links(links, N, Nt, Bs, 0.5, 0.25)[0, 3]          # only column 0 active: 1/4 does not exceed
    keep = o.aggregate_links(links, N, Nt, Bs, 0.25, 0.49)
    frame_gap = np.abs(np.arange(4)[:, None] - np.arange(4)[None, :])
    assert (keep == ((frame_gap <= 1) | ((np.arange(4)[:, None] == 0) & (np.arange(4)[None, :] == 3)))).all()


@pytest.mark.parametrize("Nf,Hg,Wg,Bs,gamma,lam", [(8, 8, 8, 32, 1.0, 1.0), (6, 6, 10, 32, 3.0, 1.0),
                                                  (6, 6, 10, 32, 1.0, 0.4), (5, 7, 9, 64, 2.0, 2.0)])
def test_everything_passing_reproduces_the_candidate_geometry(Nf, Hg, Wg, Bs, gamma, lam):
    """tau = -inf keeps all of P(i, j), so the token-level order must give the block classification of the
    candidate geometry (classify_blocks, pinned on its own), straddling and ragged blocks included."""
    Nt = Hg * Wg
    N = Nf * Nt
    tab = _tab(Nf, Nt, Bs, gamma, lam)
    Sb = -(-N // Bs)
    S = np.random.default_rng(6).standard_normal((1, 1, N, N)).astype(np.float32)
    for theta_c, theta_m in ((0.15, 0.60), (0.5, 0.3)):
        cls = o.classify_blocks(N, Nt, Bs, tab, theta_c, theta_m)
        keep = _block_keep(o.build_mask_from_tokens(S, N, Nt, Bs, tab, theta_c, theta_m, -np.inf)[0][0], Sb)
        assert (keep == (cls != o.CLASS_NONE)).all()


def test_block_mask_shrinks_with_the_threshold_and_never_below_the_forced_zone():
    Nf, Hg, Wg, Bs = 8, 8, 8, 32
    Nt, N = Hg * Wg, Nf * Hg * Wg
    tab = _tab(Nf, Nt, Bs, 1.0, 1.0)
    Sb = N // Bs
    S = np.random.default_rng(7).standard_normal((1, 1, N, N)).astype(np.float32)
    cls = o.classify_blocks(N, Nt, Bs, tab, 0.15, 0.60)
    prev = None
    for tau in (-np.inf, -1.0, 0.0, 1.0, 4.0):
        keep = _block_keep(o.build_mask_from_tokens(S, N, Nt, Bs, tab, 0.15, 0.60, tau)[0][0], Sb)
        assert keep[cls == o.CLASS_FORCED].all() and not keep[cls == o.CLASS_NONE].any()
        if prev is not None:
            assert not (keep & ~prev).any()
        prev = keep
    assert (prev == (cls == o.CLASS_FORCED)).all()      # one link per frame pair cannot make a column dense
