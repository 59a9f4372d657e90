"""Pins for the oracle's restatements of the paper's own two selection rules at block level:
the standardised-score thresholds (Eqs. 10-11) and the seeded uniform sample (Eq. 8)."""
import math

import numpy as np
import pytest

from oracle import dynamicrad_oracle as o

F, NEAR, FAR, NONE = o.CLASS_FORCED, o.CLASS_NEAR, o.CLASS_FAR, o.CLASS_NONE


def _row(classes, gaps, sides, scores):
    return (np.asarray(scores, dtype=np.float32), np.asarray(classes, dtype=np.uint8),
            np.asarray(gaps, dtype=np.int64), np.asarray(sides, dtype=np.int64))


# ------------------------------------------------------------------ z-score thresholds
def test_zscore_hand_example_one_candidate_set():
    """Scores 1, 2, 3, 4: mu = 2.5, sigma = sqrt(1.25) = 1.1180, z = -1.342, -0.447, 0.447, 1.342 (Eq. 10)."""
    s, c, g, sd = _row([F, NEAR, NEAR, NEAR, NEAR, NONE], [0, 2, 2, 2, 2, 2], [0, 1, 1, 1, 1, 1], [9, 1, 2, 3, 4, 100])
    assert o.select_zscore(s, c, g, sd, 0.4, 0.4).tolist() == [0, 3, 4]
    assert o.select_zscore(s, c, g, sd, 1.0, 1.0).tolist() == [0, 4]
    assert o.select_zscore(s, c, g, sd, -1.0, -1.0).tolist() == [0, 2, 3, 4]
    assert o.select_zscore(s, c, g, sd, -2.0, -2.0).tolist() == [0, 1, 2, 3, 4]
    # nothing passes: the highest score survives (Eq. 11's safeguard (ii))
    assert o.select_zscore(s, c, g, sd, 2.0, 2.0).tolist() == [0, 4]
    # the boundary is inclusive (Algorithm 1: keep z >= tau): z of the value 4 is 1.5 / (sqrt(1.25) + 1e-6)
    z4 = 1.5 / (math.sqrt(1.25) + 1e-6)
    assert o.select_zscore(s, c, g, sd, z4, z4).tolist() == [0, 4]
    assert o.select_zscore(s, c, g, sd, np.nextafter(z4, 2.0), z4).tolist() == [0, 4]   # fallback keeps it anyway
    assert o.select_zscore(s, c, g, sd, np.nextafter(z4, 2.0), z4).tolist() == o.select_zscore(s, c, g, sd, 9.0, 9.0).tolist()


def test_zscore_is_per_candidate_set_and_affine_invariant():
    """Two sets with very different score levels keep the same pattern; a * s + b (a > 0) changes nothing."""
    classes = [NEAR] * 3 + [F] + [NEAR] * 3
    gaps = [2, 2, 2, 0, 2, 2, 2]
    sides = [-1, -1, -1, 0, 1, 1, 1]
    s, c, g, sd = _row(classes, gaps, sides, [10, 11, 12, 0, -5, -4, -3])
    assert o.select_zscore(s, c, g, sd, 0.0, 0.0).tolist() == [1, 2, 3, 5, 6]
    assert o.select_zscore(s, c, g, sd, 1.0, 1.0).tolist() == [2, 3, 6]
    # same gap on one side only would be ONE set of six: then the low set is dropped entirely
    one = o.select_zscore(s, c, g, np.asarray([1, 1, 1, 0, 1, 1, 1]), 0.0, 0.0).tolist()
    assert one == [0, 1, 2, 3]
    s2 = (s * np.float32(4.0) + np.float32(8.0)).astype(np.float32)       # exact in fp32
    for tau in (-1.0, 0.0, 0.5, 1.0, 3.0):
        assert o.select_zscore(s2, c, g, sd, tau, tau).tolist() == o.select_zscore(s, c, g, sd, tau, tau).tolist()


def test_zscore_near_and_far_thresholds_and_degenerate_sets():
    classes = [NEAR, NEAR, NEAR, NEAR, FAR, FAR, FAR, FAR, FAR]
    gaps = [2, 2, 2, 2, 5, 5, 5, 5, 7]
    sides = [1] * 9
    s, c, g, sd = _row(classes, gaps, sides, [1, 2, 3, 4, 1, 2, 3, 4, -50])
    # tau_1 applies to the NEAR set, tau_2 to the FAR sets (Eq. 11); the singleton set (gap 7) always survives
    assert o.select_zscore(s, c, g, sd, 0.4, 1.0).tolist() == [2, 3, 7, 8]
    assert o.select_zscore(s, c, g, sd, 1.0, 0.4).tolist() == [3, 6, 7, 8]
    # constant scores: sigma = 0, z = 0 for all: kept iff tau <= 0, else the lowest index by the fallback
    s0, c0, g0, sd0 = _row([NEAR] * 4, [3] * 4, [1] * 4, [2.5] * 4)
    assert o.select_zscore(s0, c0, g0, sd0, 0.0, 0.0).tolist() == [0, 1, 2, 3]
    assert o.select_zscore(s0, c0, g0, sd0, 1e-9, 0.0).tolist() == [0]


def test_zscore_against_vectorised_statistics():
    """Independent route: numpy's mean / std per set, compared wherever the decision is not borderline."""
    rng = np.random.default_rng(5)
    for trial in range(40):
        n = 60
        classes = rng.choice([NONE, NEAR, FAR, F], size=n, p=[0.2, 0.35, 0.35, 0.1]).astype(np.uint8)
        gaps = rng.integers(2, 6, size=n)
        sides = rng.choice([-1, 1], size=n)
        scores = rng.standard_normal(n).astype(np.float32)
        t1, t2 = float(rng.uniform(-1, 1.5)), float(rng.uniform(-1, 1.5))
        got = set(o.select_zscore(scores, classes, gaps, sides, t1, t2).tolist())
        want = set(np.flatnonzero(classes == F).tolist())
        borderline = False
        for gp in range(2, 6):
            for sd in (-1, 1):
                mem = np.flatnonzero((gaps == gp) & (sides == sd) & ((classes == NEAR) | (classes == FAR)))
                if len(mem) == 0:
                    continue
                x = scores[mem].astype(np.float64)
                z = (x - x.mean()) / (x.std() + 1e-6)
                tau = np.where(classes[mem] == NEAR, t1, t2)
                borderline |= bool((np.abs(z - tau) < 1e-9).any())
                ok = mem[z >= tau]
                want |= set(ok.tolist()) if len(ok) else {int(mem[np.argmax(x)])}
        if not borderline:
            assert got == want, trial


def test_block_frame_gap_against_token_enumeration():
    for (Nf, Nt, Bs) in [(5, 6, 4), (4, 10, 4), (6, 7, 16), (3, 8, 8)]:
        N = Nf * Nt
        Sb = -(-N // Bs)
        gap, side = o.block_frame_gap(N, Nt, Bs)
        for qb in range(Sb):
            for kb in range(Sb):
                best, signs = None, set()
                for p in range(qb * Bs, min(N, qb * Bs + Bs)):
                    for q in range(kb * Bs, min(N, kb * Bs + Bs)):
                        dlt = q // Nt - p // Nt
                        best = abs(dlt) if best is None else min(best, abs(dlt))
                        signs.add((dlt > 0) - (dlt < 0))
                assert gap[qb, kb] == best
                if best > 0:
                    assert signs == {int(side[qb, kb])}
                else:
                    assert side[qb, kb] == 0
        assert (gap == gap.T).all() and (side == -side.T).all()
        # consistent with the classification: the never-pruned zone is exactly gap <= 1
        tab = o.frame_table(Nf, Nt, Bs, 1.0, 1.0)
        cls = o.classify_blocks(N, Nt, Bs, tab, 0.15, 0.60)
        assert ((cls == F) == (gap <= 1)).all()


# ------------------------------------------------------------------ seeded uniform sample
def test_fmix32_published_vectors_and_bijectivity():
    """MurmurHash3's 32-bit finaliser: 0 is a fixed point, fmix32(1) = 0x514E28B7, fmix32(0xFFFFFFFF) = 0x81F16F39
    (values of the reference implementation); it is a bijection, so no two inputs collide."""
    assert o.fmix32(0) == 0
    assert o.fmix32(1) == 0x514E28B7
    assert o.fmix32(0xFFFFFFFF) == 0x81F16F39
    outs = {o.fmix32(x) for x in range(1 << 16)}
    assert len(outs) == 1 << 16
    assert all(0 <= v < (1 << 32) for v in list(outs)[:100])


def test_uniform_keep_count_determinism_and_score_freedom():
    rng = np.random.default_rng(9)
    classes = rng.choice([NONE, NEAR, FAR, F], size=200, p=[0.3, 0.3, 0.3, 0.1]).astype(np.uint8)
    n_near, n_far, n_f = int((classes == NEAR).sum()), int((classes == FAR).sum()), int((classes == F).sum())
    for rho in (0.001, 0.1, 0.5, 1.0):
        kept = o.select_uniform(7, classes, rho, None, seed=123)
        assert len(kept) == n_f + max(1, math.floor((n_near + n_far) * rho))          # Eq. 8's k rule
        assert set(np.flatnonzero(classes == F)) <= set(kept.tolist())
        assert (classes[kept] != NONE).all() and (np.diff(kept) > 0).all()
        assert kept.tolist() == o.select_uniform(7, classes, rho, None, seed=123).tolist()
    both = o.select_uniform(7, classes, 0.25, 0.05, seed=123)
    assert int((classes[both] == NEAR).sum()) == max(1, math.floor(n_near * 0.25))
    assert int((classes[both] == FAR).sum()) == max(1, math.floor(n_far * 0.05))
    assert o.select_uniform(7, classes, 1.0, None, seed=5).tolist() == np.flatnonzero(classes != NONE).tolist()
    a = o.select_uniform(7, classes, 0.2, None, seed=1).tolist()
    assert a != o.select_uniform(7, classes, 0.2, None, seed=2).tolist()        # the seed matters
    assert a != o.select_uniform(8, classes, 0.2, None, seed=1).tolist()        # rows draw independently
    # nested samples: a larger ratio keeps a superset (the sample is a prefix of one seeded order)
    assert set(a) <= set(o.select_uniform(7, classes, 0.4, None, seed=1).tolist())


def test_uniform_sample_is_uniform():
    """Inclusion frequency of every selectable block over many (row, seed) draws is k / n (chi-square, 99.9 %)."""
    n, k_ratio, draws = 40, 0.25, 4000
    classes = np.full(n, NEAR, dtype=np.uint8)
    hits = np.zeros(n)
    for i in range(draws):
        hits[o.select_uniform(i % 97, classes, k_ratio, None, seed=1000 + i)] += 1
    k = max(1, math.floor(n * k_ratio))
    expect = draws * k / n
    chi2 = float(((hits - expect) ** 2 / (expect * (1 - k / n))).sum())
    assert chi2 < 72.0, chi2            # chi-square(39 dof): 99.9th percentile is 72.05
    assert hits.sum() == draws * k


def test_build_mask_dispatches_the_paper_modes():
    Nf, Nt, Bs = 8, 8, 4
    N = Nf * Nt
    Sb = N // Bs
    tab = o.frame_table(Nf, Nt, Bs, 3.0, 1.0)
    cls = o.classify_blocks(N, Nt, Bs, tab, 0.15, 0.60)
    gs = o.block_frame_gap(N, Nt, Bs)
    rng = np.random.default_rng(2)
    scores = rng.standard_normal((1, 2, Sb, Sb)).astype(np.float32)
    mz = o.build_mask(scores, cls, "zscore", 0.3, gap_side=gs, tau_far=-0.2)
    mu = o.build_mask(scores, cls, "uniform", 0.3, ratio_far=0.1, seed=77)
    for m in range(2):
        rp, ci = mz[0][m]
        for qb in range(Sb):
            want = o.select_zscore(scores[0, m, qb], cls[qb], gs[0][qb], gs[1][qb], 0.3, -0.2)
            assert ci[rp[qb]:rp[qb + 1]].tolist() == want.tolist()
        rp, ci = mu[0][m]
        for qb in range(Sb):
            assert ci[rp[qb]:rp[qb + 1]].tolist() == o.select_uniform(qb, cls[qb], 0.3, 0.1, 77).tolist()
    # the uniform mask does not depend on the head (scores are not read): both masks are equal
    assert mu[0][0][1].tolist() == mu[0][1][1].tolist()
    with pytest.raises(ValueError):
        o.build_mask(scores, cls, "nonsense", 0.3)
