"""Pins for the oracle's geometry: the per-t table, Eq. 7 and the block classes."""
import math
import os

import numpy as np
import pytest

from oracle import dynamicrad_oracle as o
from workloads import CONFIGS

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_tables():
    cases, cur = [], None
    for line in open(os.path.join(GOLD, "frame_tables.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "case":
            cur = {"name": f[1], "Nf": int(f[2]), "Nt": int(f[3]), "Bs": int(f[4]),
                   "gamma": float(f[5]), "lam": float(f[6]), "rows": []}
            cases.append(cur)
        else:
            cur["rows"].append(tuple(int(x) for x in f))
    return cases


@pytest.mark.parametrize("case", _read_tables(), ids=lambda c: c["name"])
def test_frame_table_matches_hand_derivation(case):
    tab = o.frame_table(case["Nf"], case["Nt"], case["Bs"], case["gamma"], case["lam"])
    for t, w, sf, ret in case["rows"]:
        assert int(tab["w"][t]) == w, (t, "w")
        assert int(tab["sf"][t]) == sf, (t, "sf")
        assert bool(tab["retained"][t]) == bool(ret), (t, "retained")
    # t <= 1 rows of Eq. 3 / Eq. 8
    assert int(tab["w"][0]) == case["Nt"] and bool(tab["retained"][0])
    if case["Nf"] > 1:
        assert int(tab["w"][1]) == case["Nt"] and bool(tab["retained"][1])


def test_log_group_is_bit_length_and_L0_power_of_two():
    tab = o.frame_table(70, 1000, 32, 1.0, 1.0)
    assert int(tab["L0"]) == 1024
    for t in range(1, 70):
        assert int(tab["group"][t]) == t.bit_length()
        base = tab["L0"] / 2.0 ** tab["group"][t]
        # Eq. 2's "approximately L0 / t": 2^(B-1) <= t < 2^B, so L0/(2t) <= L0/2^B(t) < L0/t
        assert tab["L0"] / (2.0 * t) <= base < tab["L0"] / t
    assert int(o.frame_table(3, 1024, 32, 1.0, 1.0)["L0"]) == 1024
    assert int(o.frame_table(3, 1025, 32, 1.0, 1.0)["L0"]) == 2048


def test_near_far_class_follows_decay_length():
    tab = o.frame_table(21, 3600, 128, 1.0, 0.5)
    assert [int(c) for c in tab["cls"][:2]] == [o.CLASS_FORCED] * 2
    # L(t) = 1024, 512, 256, 128 are all >= Bs = 128 -> near everywhere
    assert all(int(c) == o.CLASS_NEAR for c in tab["cls"][2:])
    tab = o.frame_table(21, 1560, 128, 1.0, 0.3)
    assert all(int(tab["cls"][t]) == o.CLASS_NEAR for t in range(2, 16))     # L >= 128
    assert all(int(tab["cls"][t]) == o.CLASS_FAR for t in range(16, 21))     # L = 64


def test_token_predicate_scalar_matches_matrix_and_is_symmetric():
    Nf, Nt, Bs = 9, 20, 8
    tab = o.frame_table(Nf, Nt, Bs, 1.7, 0.9)
    N = Nf * Nt
    M = o.candidate_matrix(N, Nt, tab)
    assert (M == M.T).all()
    rng = np.random.default_rng(0)
    for _ in range(2000):
        p, q = (int(x) for x in rng.integers(0, N, 2))
        assert bool(M[p, q]) == o.token_candidate(p, q, Nt, tab)
    # all t <= 1 pairs are candidates (|u - v| < Nt = w)
    fr = np.arange(N) // Nt
    assert M[np.abs(fr[:, None] - fr[None, :]) <= 1].all()
    # a dropped frame distance has no candidate at all
    for t in range(2, Nf):
        if not tab["retained"][t]:
            assert not M[np.abs(fr[:, None] - fr[None, :]) == t].any()


def test_token_predicate_window_edges():
    # Nt = 64, Bs = 8, gamma = 1: L0 = 64; t = 2: L = 16 -> w = 16
    tab = o.frame_table(4, 64, 8, 1.0, 8.0)
    assert int(tab["w"][2]) == 16 and bool(tab["retained"][2])
    assert o.token_candidate(0 * 64 + 10, 2 * 64 + 26, 64, tab)          # |u - v| = 16
    assert not o.token_candidate(0 * 64 + 10, 2 * 64 + 27, 64, tab)      # 17
    assert o.token_candidate(2 * 64 + 26, 0 * 64 + 10, 64, tab)


GEOMS = [
    # Nf, Hg*Wg, Bs, gamma, lam, theta_c, theta_m
    (8, 64, 32, 1.0, 1.0, 0.15, 0.60),
    (6, 60, 32, 1.0, 1.0, 0.15, 0.60),       # blocks straddle frames, ragged tail (360 = 11.25 blocks)
    (7, 50, 32, 2.5, 0.4, 0.30, 0.50),
    (5, 100, 64, 1.3, 0.7, 0.10, 0.90),
    (12, 24, 32, 3.0, 0.1, 0.50, 0.25),      # blocks longer than a frame
    (9, 37, 32, 1.0, 2.0, 0.0, 0.0),
    (4, 64, 64, 1.0, 0.5, 0.15, 0.60),       # cfg1
    (10, 130, 128, 1.0, 1.0, 0.15, 0.60),
]


@pytest.mark.parametrize("g", GEOMS)
def test_interval_classification_equals_token_level_definition(g):
    Nf, Nt, Bs, gamma, lam, tc, tm = g
    tab = o.frame_table(Nf, Nt, Bs, gamma, lam)
    N = Nf * Nt
    a = o.classify_blocks_literal(N, Nt, Bs, tab, tc, tm)
    b = o.classify_blocks(N, Nt, Bs, tab, tc, tm)
    assert (a == b).all()


def test_classification_by_explicit_loops_tiny():
    """Third opinion: pure-Python loops over token pairs, no numpy broadcasting."""
    Nf, Nt, Bs, tc, tm = 6, 10, 4, 0.3, 0.4
    tab = o.frame_table(Nf, Nt, Bs, 1.0, 4.0)
    N = Nf * Nt
    Sb = -(-N // Bs)
    got = o.classify_blocks(N, Nt, Bs, tab, tc, tm)
    for qb in range(Sb):
        rows = range(qb * Bs, min(N, qb * Bs + Bs))
        for kb in range(Sb):
            cols = range(kb * Bs, min(N, kb * Bs + Bs))
            tmin = min(abs(p // Nt - q // Nt) for p in rows for q in cols)
            if tmin <= 1:
                want = o.CLASS_FORCED
            else:
                act = 0
                for q in cols:
                    cnt = sum(1 for p in rows if o.token_candidate(p, q, Nt, tab))
                    if cnt / len(rows) > tc:
                        act += 1
                want = int(tab["cls"][tmin]) if act / len(cols) > tm else o.CLASS_NONE
            assert got[qb, kb] == want, (qb, kb)


def test_candidate_set_grows_with_gamma_and_forced_zone_is_invariant():
    Nf, Nt, Bs = 10, 96, 32
    N = Nf * Nt
    prev = None
    for gamma in (1.0, 1.5, 2.0, 3.0):
        tab = o.frame_table(Nf, Nt, Bs, gamma, 1.0)
        cm = o.classify_blocks(N, Nt, Bs, tab, 0.15, 0.6)
        cand = cm > 0
        if prev is not None:
            assert (cand | ~prev).all()          # superset
        prev = cand
        fr_lo = (np.arange(cm.shape[0]) * Bs) // Nt
        fr_hi = (np.minimum(N, np.arange(cm.shape[0]) * Bs + Bs) - 1) // Nt
        gap = np.maximum(0, np.maximum(fr_lo[None, :] - fr_hi[:, None], fr_lo[:, None] - fr_hi[None, :]))
        assert ((cm == o.CLASS_FORCED) == (gap <= 1)).all()


def test_cfg1_is_forced_tridiagonal():
    wl = CONFIGS["cfg1"]
    tab = o.frame_table(wl.Nf, wl.Nt, wl.Bs, 1.0, wl.lam)
    cm = o.classify_blocks(wl.N, wl.Nt, wl.Bs, tab, 0.15, 0.60)
    want = np.zeros((4, 4), dtype=np.uint8)
    for i in range(4):
        for j in range(4):
            if abs(i - j) <= 1:
                want[i, j] = o.CLASS_FORCED
    assert (cm == want).all()


def test_block_class_counts_second_opinion():
    for line in open(os.path.join(GOLD, "block_class_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, forced, cand, smin, smax = line.split()
        wl = CONFIGS[name]
        tab = o.frame_table(wl.Nf, wl.Nt, wl.Bs, 1.0, wl.lam)
        cm = o.classify_blocks(wl.N, wl.Nt, wl.Bs, tab, 0.15, 0.60)
        sel = ((cm == o.CLASS_NEAR) | (cm == o.CLASS_FAR)).sum(axis=1)
        assert int((cm == o.CLASS_FORCED).sum()) == int(forced)
        assert int((cm > 0).sum()) == int(cand)
        assert (int(sel.min()), int(sel.max())) == (int(smin), int(smax))


def test_mean_window_tracks_complexity_estimate():
    """App. A: attended tokens per query ~ sum over t of w(t); loose 2x sanity bound when sf == 1."""
    Nf, Nt, Bs = 21, 3600, 128
    tab = o.frame_table(Nf, Nt, Bs, 1.0, 0.5)
    assert (tab["sf"] == 1).all()
    est = float(tab["L0"]) * sum(1.0 / t for t in range(2, Nf))
    # token-level candidate row length for t >= 2 of a query in the middle frame, middle of the frame
    i, u = Nf // 2, Nt // 2
    length = 0
    for j in range(Nf):
        t = abs(i - j)
        if t >= 2:
            w = int(tab["w"][t])
            length += min(Nt - 1, u + w) - max(0, u - w) + 1
    assert 0.5 * est <= length <= 2.0 * est * 2   # both window sides are counted in `length`
