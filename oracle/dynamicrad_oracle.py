"""CPU fp64 oracle for the DynamicRad attention hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the GPU library must compute.
It is imported by the tests, by the smoke check and by the benchmark's
``cpu_baseline`` leg and by nothing else; the GPU library never calls it and
shares no code, tables or constants with it.

Stages, in the order of the method (paper sections in brackets):

  block_scores      pooled proxy score per (query block, key block)
                    [Two-Mode Selection, the proxy-score equation (Eq. 9), and
                    the head-fusion proxy of App. B (Eq. 19)]
  frame_table       per temporal distance t: log group, decay length, window,
                    split stride, retained flag, near/far class
                    [Dynamic Neighborhood Partitioning, Eqs. 1-6; Eq. 8 classes]
  token_candidate   the candidate predicate on one token pair   [Eq. 7]
  classify_blocks   density aggregation (theta_c, theta_m) of the candidate
                    geometry to blocks, plus the never-pruned t<=1 zone
                    ["Density control within blocks"; Eq. 3 / Eq. 8 t<=1 rows]
  select_row        static-ratio top-k or dynamic cumulative-mass prefix on
                    one query-block row  [Eq. 8 with k = max(1, floor(n rho));
                    Eq. 11's keep-one fallback]
  select_zscore     the paper's own dynamic-threshold rule restated per row:
                    scores standardised inside each candidate set, thresholds
                    tau_1 / tau_2 by decay state, keep-one fallback
                    [score normalisation (Eq. 10), threshold selector (Eq. 11)]
  select_uniform    the paper's own static-ratio rule restated per row: a
                    seeded, score-free uniform sample of k blocks
                    [Eq. 8 with k = max(1, floor(n rho)), "deterministic seed"]
  build_mask        all rows -> CSR (rowptr, colidx)  [Algorithm 1's output M_b]
  token_scores / select_token_links / aggregate_links / build_mask_from_tokens
                    Algorithm 1 in its own order, for small N: the proxy score
                    of every token pair, z-score thresholds inside each frame
                    pair's candidate set, then the density aggregation of the
                    kept links to blocks  [Eqs. 7, 9-11; "Density control
                    within blocks"; Algorithm 1]
  masked_attention  softmax over exactly the keys of the kept blocks
                    [Eqs. 12-13 with epsilon -> 0]
  attention_matrix / proxy_loss   the row-normalised attention matrix under a
                    block mask and the offline-search objective built on it:
                    normalised squared error against the dense matrix plus the
                    sparsity penalty  [App. C: proxy attention, Eq. 22]

Readings taken where the text leaves a choice (each is a deliberate
interpretation, listed again in the design notes):

  * epsilon of Eq. 5 is 1e-6 and the quotient is evaluated in fp64.
  * the rounding in Eq. 3 is round-half-up, floor(x + 0.5).
  * u, v of Eq. 7 are the row-major flattened in-frame token indices.
  * blocks are cut on the global token index (the padding S' is global).
  * "exceeds" in the density rule is a strict >, with the counts divided by
    the number of *valid* rows / columns of the block.
  * selection is done at block granularity, per query-block row, over the
    candidate blocks whose every token pair has t > 1; blocks containing any
    token pair with t <= 1 are always kept ("forced").
  * static-ratio mode keeps the top k blocks by pooled score (not a uniform
    sample); dynamic mode keeps the shortest score-descending prefix whose
    softmax mass reaches tau of the total mass of the selectable blocks.
  * order of equal scores: lower key-block index first; -0.0 equals +0.0.
  * z-score mode: the candidate set P(i, j) of a frame pair becomes, for a
    query-block row, the selectable blocks that share the smallest frame
    distance to the row AND lie on the same side of it (before / after): the
    block-level image of "frame j = i - t" and "frame j = i + t".  Mean and
    standard deviation are the population ones (divide by n), epsilon of
    Eq. 10 is 1e-6, and a block is kept when z >= tau (Algorithm 1 writes >=).
    All of it in fp64, sums taken one by one in ascending key-block order.
  * token-level order (build_mask_from_tokens): statistics of a frame pair
    are taken over its whole candidate set P(i, j) as Eq. 10 says; the sums
    run column by column (u ascending inside a column, then the column sums
    over v ascending), one by one in fp64; the aggregation is applied to the
    merged link matrix block by block, and blocks touching the t <= 1 zone
    are kept as in the block-level path.
  * uniform mode: every selectable block of a row gets the 32-bit key
    fmix32(fmix32(seed ^ fmix32(qb)) + kb) (fmix32 = the finaliser of
    MurmurHash3); the k blocks with the smallest keys are kept, equal keys by
    lower index.  With two ratios NEAR and FAR blocks are sampled separately.

Pins: tests/test_oracle_*.py check every function here against brute force,
closed forms, hand-derived tables (tests/golden/) and invariants.  The paper's
reported sparsities, latencies and quality scores depend on real model
activations and are not reproducible here: for those, parity unpinned.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

CLASS_NONE = 0      # not a candidate
CLASS_NEAR = 1      # selectable, decay length >= block size at the block's smallest t
CLASS_FAR = 2       # selectable, decay length < block size
CLASS_FORCED = 3    # contains a token pair with t <= 1: never pruned

SPLIT_EPS = 1e-6    # epsilon of the split-stride equation


# --------------------------------------------------------------------------- #
# stage (a): pooled block scores
# --------------------------------------------------------------------------- #
def block_means(X: np.ndarray, Bs: int) -> np.ndarray:
    """Mean over the valid tokens of each block.  X [N, d] -> [Sb, d] (fp64)."""
    X = np.asarray(X, dtype=np.float64)
    N = X.shape[0]
    Sb = -(-N // Bs)
    out = np.empty((Sb, X.shape[1]), dtype=np.float64)
    for blk in range(Sb):
        lo, hi = blk * Bs, min(N, (blk + 1) * Bs)
        out[blk] = X[lo:hi].sum(axis=0) / float(hi - lo)
    return out


def block_scores(Q: np.ndarray, K: np.ndarray, Bs: int, head_fuse: int) -> np.ndarray:
    """Proxy score of Eq. 9 averaged over each (query block, key block).

    Q, K: [B, H, N, d].  head_fuse = Hf > 0: mean over heads 0..Hf-1, output
    [B, 1, Sb, Sb]; head_fuse = 0: one score map per head, [B, H, Sb, Sb].
    The block mean of the logit equals the logit of the block means (the dot
    product is bilinear), which is what is evaluated here.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    B, H, N, d = Q.shape
    Sb = -(-N // Bs)
    heads_per_mask = [list(range(head_fuse))] if head_fuse > 0 else [[h] for h in range(H)]
    out = np.zeros((B, len(heads_per_mask), Sb, Sb), dtype=np.float64)
    for b in range(B):
        for m, hs in enumerate(heads_per_mask):
            for h in hs:
                qm = block_means(Q[b, h], Bs)
                km = block_means(K[b, h], Bs)
                out[b, m] += (qm @ km.T) / math.sqrt(d)
            out[b, m] /= float(len(hs))
    return out


# --------------------------------------------------------------------------- #
# stage (b1): per temporal distance table
# --------------------------------------------------------------------------- #
def frame_table(Nf: int, Nt: int, Bs: int, gamma: float, lam: float) -> Dict[str, np.ndarray]:
    """Quantities of Eqs. 1-6 for t = 0 .. Nf-1.

    group    B(t) = floor(log2 t) + 1 for t >= 1              (Eq. 1)
    L0       smallest power of two >= Nt                       (Eq. 1)
    decay    L(t) = L0 / 2^B(t) * gamma                        (Eq. 2)
    w        Nt for t <= 1, else max(Bs, round(L(t)))          (Eq. 3)
    lsplit   L0 / 2^B(t) * lambda                              (Eq. 4)
    sf       max(1, floor(Bs / (lsplit + eps)))                (Eq. 5)
    retained t mod sf == 0                                     (Eq. 6)
    cls      FORCED for t <= 1; NEAR if L(t) >= Bs else FAR    (Eq. 8 cases)
    """
    L0 = 1
    while L0 < Nt:
        L0 *= 2
    group = np.zeros(Nf, dtype=np.int64)
    decay = np.zeros(Nf, dtype=np.float64)
    lsplit = np.zeros(Nf, dtype=np.float64)
    w = np.zeros(Nf, dtype=np.int64)
    sf = np.ones(Nf, dtype=np.int64)
    retained = np.zeros(Nf, dtype=bool)
    cls = np.zeros(Nf, dtype=np.int64)
    for t in range(Nf):
        if t <= 1:
            w[t] = Nt
            retained[t] = True
            cls[t] = CLASS_FORCED
            if t == 1:
                group[t] = 1
                decay[t] = L0 / 2.0 * gamma
                lsplit[t] = L0 / 2.0 * lam
            continue
        g = int(math.floor(math.log2(t))) + 1
        assert (1 << (g - 1)) <= t < (1 << g)
        group[t] = g
        decay[t] = (L0 / float(1 << g)) * gamma
        lsplit[t] = (L0 / float(1 << g)) * lam
        w[t] = max(Bs, int(math.floor(decay[t] + 0.5)))
        sf[t] = max(1, int(math.floor(Bs / (lsplit[t] + SPLIT_EPS))))
        retained[t] = (t % sf[t]) == 0
        cls[t] = CLASS_NEAR if decay[t] >= Bs else CLASS_FAR
    return {"L0": np.int64(L0), "group": group, "decay": decay, "lsplit": lsplit,
            "w": w, "sf": sf, "retained": retained, "cls": cls}


def token_candidate(p: int, q: int, Nt: int, tab: Dict[str, np.ndarray]) -> bool:
    """Eq. 7 on global token indices p (query) and q (key)."""
    i, u = divmod(p, Nt)
    j, v = divmod(q, Nt)
    t = abs(i - j)
    return bool(tab["retained"][t]) and abs(u - v) <= int(tab["w"][t])


def candidate_matrix(N: int, Nt: int, tab: Dict[str, np.ndarray]) -> np.ndarray:
    """Token-level candidate mask [N, N], Eq. 7 evaluated for every pair (small N only)."""
    p = np.arange(N)
    i, u = p // Nt, p % Nt
    t = np.abs(i[:, None] - i[None, :])
    return tab["retained"][t] & (np.abs(u[:, None] - u[None, :]) <= tab["w"][t])


# --------------------------------------------------------------------------- #
# stage (b2): block classification
# --------------------------------------------------------------------------- #
def _block_range(blk: int, Bs: int, N: int) -> Tuple[int, int]:
    return blk * Bs, min(N, (blk + 1) * Bs)


def classify_blocks_literal(N: int, Nt: int, Bs: int, tab: Dict[str, np.ndarray],
                            theta_c: float, theta_m: float) -> np.ndarray:
    """Block classes from the full token-level matrix (definition; small N only)."""
    cand = candidate_matrix(N, Nt, tab)
    Sb = -(-N // Bs)
    frame = np.arange(N) // Nt
    out = np.zeros((Sb, Sb), dtype=np.uint8)
    for qb in range(Sb):
        r0, r1 = _block_range(qb, Bs, N)
        for kb in range(Sb):
            c0, c1 = _block_range(kb, Bs, N)
            sub = cand[r0:r1, c0:c1]
            tt = np.abs(frame[r0:r1, None] - frame[None, c0:c1])
            tmin = int(tt.min())
            if tmin <= 1:
                out[qb, kb] = CLASS_FORCED
                continue
            col_ratio = sub.sum(axis=0) / float(r1 - r0)
            active = col_ratio > theta_c
            if active.sum() / float(c1 - c0) > theta_m:
                out[qb, kb] = tab["cls"][tmin]
    return out


def classify_blocks(N: int, Nt: int, Bs: int, tab: Dict[str, np.ndarray],
                    theta_c: float, theta_m: float) -> np.ndarray:
    """Same result as classify_blocks_literal, without materialising [N, N].

    For one query block the rows form one run of in-frame indices [u_lo, u_hi]
    per frame they touch.  For a key token (frame j, index v) and a row run in
    frame i, the number of rows with |u - v| <= w(t) is the size of
    [u_lo, u_hi] intersected with [v - w, v + w]; summed over the runs this is
    the column's retained-row count.
    """
    Sb = -(-N // Bs)
    q = np.arange(N)
    jf, v = q // Nt, q % Nt
    out = np.zeros((Sb, Sb), dtype=np.uint8)
    w, retained, cls = tab["w"], tab["retained"], tab["cls"]
    starts = np.arange(Sb) * Bs
    n_c = np.minimum(N, starts + Bs) - starts
    f_lo_blk = starts // Nt
    f_hi_blk = (np.minimum(N, starts + Bs) - 1) // Nt
    for qb in range(Sb):
        r0, r1 = _block_range(qb, Bs, N)
        count = np.zeros(N, dtype=np.int64)
        i0, i1 = r0 // Nt, (r1 - 1) // Nt
        for i in range(i0, i1 + 1):
            u_lo = max(r0, i * Nt) - i * Nt
            u_hi = min(r1, (i + 1) * Nt) - 1 - i * Nt
            t = np.abs(jf - i)
            lo = np.maximum(u_lo, v - w[t])
            hi = np.minimum(u_hi, v + w[t])
            count += np.where(retained[t], np.maximum(0, hi - lo + 1), 0)
        active = (count / float(r1 - r0)) > theta_c
        n_active = np.add.reduceat(active.astype(np.int64), starts)
        is_cand = (n_active / n_c.astype(np.float64)) > theta_m
        # smallest |i - j| over the frames touched by the row block and by each key block
        gap = np.maximum(0, np.maximum(f_lo_blk - i1, i0 - f_hi_blk))
        row = np.where(is_cand, cls[gap], CLASS_NONE)
        row = np.where(gap <= 1, CLASS_FORCED, row)
        out[qb] = row.astype(np.uint8)
    return out


# --------------------------------------------------------------------------- #
# stage (b3): selection on one row
# --------------------------------------------------------------------------- #
def _ordered(scores_f32: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """idx sorted by score descending, ties by index ascending, -0 == +0."""
    s = scores_f32[idx].astype(np.float32) + np.float32(0.0)   # -0.0 + 0.0 = +0.0
    if np.isnan(s).any():
        raise ValueError("NaN block score")
    order = np.lexsort((idx, -s.astype(np.float64)))
    return idx[order]


def static_keep_count(n: int, ratio: float) -> int:
    """k = max(1, floor(n * rho)) of Eq. 8, 0 for an empty set."""
    return 0 if n == 0 else max(1, int(math.floor(float(n) * float(ratio))))


def select_static(scores_f32: np.ndarray, cls_row: np.ndarray, ratio: float,
                  ratio_far: Optional[float] = None) -> np.ndarray:
    """Kept key blocks of one row, static-ratio mode.  Returns ascending indices."""
    forced = np.flatnonzero(cls_row == CLASS_FORCED)
    if ratio_far is None or ratio_far < 0:
        groups = [(np.flatnonzero((cls_row == CLASS_NEAR) | (cls_row == CLASS_FAR)), ratio)]
    else:
        groups = [(np.flatnonzero(cls_row == CLASS_NEAR), ratio),
                  (np.flatnonzero(cls_row == CLASS_FAR), ratio_far)]
    kept = [forced]
    for idx, rho in groups:
        k = static_keep_count(len(idx), rho)
        kept.append(_ordered(scores_f32, idx)[:k])
    return np.sort(np.concatenate(kept)).astype(np.int64)


def select_dynamic(scores_f32: np.ndarray, cls_row: np.ndarray, tau: float,
                   return_margin: bool = False):
    """Kept key blocks of one row, dynamic cumulative-mass mode.

    e_j = exp(s_j - max s) in fp64 over the selectable blocks; walk them in the
    total order adding e_j one at a time; Z is the final sum; keep the shortest
    prefix with running sum >= tau * Z, never fewer than one.
    """
    forced = np.flatnonzero(cls_row == CLASS_FORCED)
    idx = np.flatnonzero((cls_row == CLASS_NEAR) | (cls_row == CLASS_FAR))
    margin = math.inf
    if len(idx) == 0:
        sel = idx
    else:
        order = _ordered(scores_f32, idx)
        s = scores_f32[order].astype(np.float64)
        m = float(s[0])
        e = [math.exp(float(x) - m) for x in s]
        cums = []
        cum = 0.0
        for x in e:
            cum = cum + x
            cums.append(cum)
        Z = cum
        target = float(tau) * Z
        k = len(order)
        for n, c in enumerate(cums):
            if c >= target:
                k = n + 1
                break
        k = max(1, k)
        margin = min(abs(c - target) for c in cums) / Z
        sel = order[:k]
    kept = np.sort(np.concatenate([forced, sel])).astype(np.int64)
    return (kept, margin) if return_margin else kept


def block_frame_gap(N: int, Nt: int, Bs: int) -> Tuple[np.ndarray, np.ndarray]:
    """Smallest frame distance between the tokens of each (query block, key block) and the side of the key block.

    gap[qb, kb] = min |i - j| over frames i touched by qb and j touched by kb; side = +1 if the key block's
    frames all come after the query block's, -1 if before, 0 if they overlap (gap 0).
    """
    Sb = -(-N // Bs)
    starts = np.arange(Sb) * Bs
    ends = np.minimum(N, starts + Bs)
    f_lo, f_hi = starts // Nt, (ends - 1) // Nt
    after = f_lo[None, :] - f_hi[:, None]        # key's first frame - query's last frame
    before = f_lo[:, None] - f_hi[None, :]       # query's first frame - key's last frame
    gap = np.maximum(0, np.maximum(after, before))
    side = np.where(after > 0, 1, np.where(before > 0, -1, 0))
    return gap.astype(np.int64), side.astype(np.int64)


def select_zscore(scores_f32: np.ndarray, cls_row: np.ndarray, gap_row: np.ndarray, side_row: np.ndarray,
                  tau_near: float, tau_far: float, eps: float = 1e-6) -> np.ndarray:
    """Kept key blocks of one row under the paper's dynamic-threshold rule (Eqs. 10-11).

    The selectable blocks of the row are split into candidate sets by (frame gap, side).  Inside a set:
    mu = mean, sigma = population std, z = (s - mu) / (sigma + eps); keep z >= tau, with tau = tau_near for NEAR
    blocks (decay length >= block size) and tau_far for FAR blocks; if nothing passes, keep the highest score
    (lower index on ties).  Forced blocks (threshold -inf in Eq. 11) are always kept.
    """
    kept = list(np.flatnonzero(cls_row == CLASS_FORCED))
    sel = np.flatnonzero((cls_row == CLASS_NEAR) | (cls_row == CLASS_FAR))
    groups: Dict[Tuple[int, int], List[int]] = {}
    for kb in sel:                                  # ascending key-block order
        groups.setdefault((int(gap_row[kb]), int(side_row[kb])), []).append(int(kb))
    for members in groups.values():
        vals = [float(scores_f32[kb]) for kb in members]
        n = len(vals)
        total = 0.0
        for x in vals:
            total = total + x
        mu = total / n
        ssq = 0.0
        for x in vals:
            dlt = x - mu
            ssq = ssq + dlt * dlt
        sigma = math.sqrt(ssq / n)
        passed = []
        best = None
        for kb, x in zip(members, vals):
            tau = tau_near if cls_row[kb] == CLASS_NEAR else tau_far
            if (x - mu) / (sigma + eps) >= tau:
                passed.append(kb)
            if best is None or x > best[0]:
                best = (x, kb)
        kept.extend(passed if passed else [best[1]])
    return np.sort(np.asarray(kept, dtype=np.int64))


def fmix32(x: int) -> int:
    """Finaliser of MurmurHash3 (32-bit): a bijective integer mixer."""
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x85EBCA6B) & 0xFFFFFFFF
    x ^= x >> 13
    x = (x * 0xC2B2AE35) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def sample_key(seed: int, qb: int, kb: int) -> int:
    """Counter-based 32-bit key of block pair (qb, kb) under `seed`."""
    return fmix32((fmix32((seed & 0xFFFFFFFF) ^ fmix32(qb)) + kb) & 0xFFFFFFFF)


def select_uniform(qb: int, cls_row: np.ndarray, ratio: float, ratio_far: Optional[float], seed: int) -> np.ndarray:
    """Kept key blocks of row qb under the paper's static-ratio rule: a seeded uniform sample of
    k = max(1, floor(n rho)) selectable blocks (Eq. 8), scores not consulted."""
    forced = np.flatnonzero(cls_row == CLASS_FORCED)
    if ratio_far is None or ratio_far < 0:
        groups = [(np.flatnonzero((cls_row == CLASS_NEAR) | (cls_row == CLASS_FAR)), ratio)]
    else:
        groups = [(np.flatnonzero(cls_row == CLASS_NEAR), ratio),
                  (np.flatnonzero(cls_row == CLASS_FAR), ratio_far)]
    kept = [forced]
    for idx, rho in groups:
        k = static_keep_count(len(idx), rho)
        order = sorted(idx.tolist(), key=lambda kb: (sample_key(seed, qb, kb), kb))
        kept.append(np.asarray(order[:k], dtype=np.int64))
    return np.sort(np.concatenate(kept)).astype(np.int64)


# --------------------------------------------------------------------------- #
# stage (b4): whole mask as CSR
# --------------------------------------------------------------------------- #
def build_mask(scores_f32: np.ndarray, cls_map: np.ndarray, mode: str, ratio_or_tau: float,
               ratio_far: Optional[float] = None, gap_side: Optional[Tuple[np.ndarray, np.ndarray]] = None,
               tau_far: Optional[float] = None, seed: int = 0) -> List[List[Tuple[np.ndarray, np.ndarray]]]:
    """CSR (rowptr, colidx) per (batch, mask head).  scores_f32: [B, Hm, Sb, Sb] float32.

    mode "static" / "dynamic": the pooled-score top-k and cumulative-mass rules; "zscore": select_zscore with
    tau_near = ratio_or_tau and tau_far (default: the same), needs gap_side = block_frame_gap(...);
    "uniform": select_uniform with `seed` (scores are only used for their shape).
    """
    scores_f32 = np.asarray(scores_f32)
    assert scores_f32.dtype == np.float32
    B, Hm, Sb, _ = scores_f32.shape
    out = []
    for b in range(B):
        per_b = []
        for m in range(Hm):
            rowptr = np.zeros(Sb + 1, dtype=np.int64)
            cols = []
            for qb in range(Sb):
                if mode == "static":
                    kept = select_static(scores_f32[b, m, qb], cls_map[qb], ratio_or_tau, ratio_far)
                elif mode == "dynamic":
                    kept = select_dynamic(scores_f32[b, m, qb], cls_map[qb], ratio_or_tau)
                elif mode == "zscore":
                    kept = select_zscore(scores_f32[b, m, qb], cls_map[qb], gap_side[0][qb], gap_side[1][qb],
                                         ratio_or_tau, ratio_or_tau if tau_far is None else tau_far)
                elif mode == "uniform":
                    kept = select_uniform(qb, cls_map[qb], ratio_or_tau, ratio_far, seed)
                else:
                    raise ValueError(mode)
                cols.append(kept)
                rowptr[qb + 1] = rowptr[qb] + len(kept)
            per_b.append((rowptr, np.concatenate(cols) if cols else np.zeros(0, np.int64)))
        out.append(per_b)
    return out


# --------------------------------------------------------------------------- #
# Algorithm 1 in its own order: token-pair selection per frame pair, then
# aggregation of the kept links to blocks (small N only)
# --------------------------------------------------------------------------- #
def token_scores(Q: np.ndarray, K: np.ndarray, head_fuse: int) -> np.ndarray:
    """Proxy score of every token pair, Eq. 9: s(p, q) = mean over the head set of Q_p . K_q / sqrt(d).

    Q, K: [B, H, N, d].  head_fuse = Hf > 0: heads 0..Hf-1 averaged, one matrix per batch element;
    0: one matrix per head.  Returns [B, masks, N, N] float64.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    B, H, N, d = Q.shape
    logits = np.einsum("bhpc,bhqc->bhpq", Q, K) / math.sqrt(d)
    if head_fuse > 0:
        return logits[:, :head_fuse].mean(axis=1, keepdims=True)
    return logits


def _sum_columns_then_across(x: np.ndarray) -> float:
    """Sum of a matrix in the order both sides use: every column v is added up over u ascending, then the column
    sums are added up over v ascending, all one by one in fp64.  (Entries outside the window are passed in as +0,
    which leaves every partial sum as it is.)"""
    col = np.add.accumulate(x, axis=0)[-1]          # accumulate is a strictly sequential running sum
    return float(np.add.accumulate(col)[-1])


def select_token_links(scores_f32: np.ndarray, N: int, Nt: int, tab: Dict[str, np.ndarray],
                       tau_near: float, tau_far: float, eps: float = 1e-6) -> np.ndarray:
    """Kept token links [N, N] (bool) under the dynamic-threshold rule, frame pair by frame pair (Algorithm 1).

    For the ordered frame pair (i, j), t = |i - j|:
      t <= 1                     every token pair is kept (w = Nt in Eq. 3, tau = -inf in Eq. 11);
      t mod sf(t) != 0           nothing is kept (Eq. 6);
      otherwise                  P(i, j) = {(u, v): |u - v| <= w(t)} (Eq. 7); mu and sigma are the mean and the
                                 population standard deviation of the scores in P(i, j) (Eq. 10), z = (s - mu) /
                                 (sigma + eps), and a pair is kept when z >= tau, tau = tau_near if the decay length
                                 L(t) >= Bs else tau_far (Eq. 11); if no pair passes, the highest score of the set
                                 is kept (first in row-major (u, v) order on ties).
    scores_f32: [N, N] float32 (token_scores rounded once, or the GPU's own).
    """
    s_all = np.asarray(scores_f32)
    assert s_all.dtype == np.float32 and s_all.shape == (N, N)
    Nf = N // Nt
    assert Nf * Nt == N
    links = np.zeros((N, N), dtype=bool)
    u = np.arange(Nt)
    dist = np.abs(u[:, None] - u[None, :])
    for i in range(Nf):
        for j in range(Nf):
            t = abs(i - j)
            blk = (slice(i * Nt, (i + 1) * Nt), slice(j * Nt, (j + 1) * Nt))
            if t <= 1:
                links[blk] = True
                continue
            if not tab["retained"][t]:
                continue
            inside = dist <= int(tab["w"][t])
            s = s_all[blk].astype(np.float64)
            n = int(inside.sum())
            mu = _sum_columns_then_across(np.where(inside, s, 0.0)) / n
            dev = s - mu
            sigma = math.sqrt(_sum_columns_then_across(np.where(inside, dev * dev, 0.0)) / n)
            tau = tau_near if tab["cls"][t] == CLASS_NEAR else tau_far
            keep = inside & (dev / (sigma + eps) >= tau)
            if not keep.any():
                best = int(np.argmax(np.where(inside, s, -np.inf)))      # first maximum in row-major order
                keep = np.zeros_like(inside)
                keep[best // Nt, best % Nt] = True
            links[blk] = keep
    return links


def aggregate_links(links: np.ndarray, N: int, Nt: int, Bs: int, theta_c: float, theta_m: float) -> np.ndarray:
    """Block mask [Sb, Sb] (bool) from token links ("Density control within blocks"; the last step of Algorithm 1).

    Column c of block (qb, kb) is active when (#kept rows of the column) / (#valid rows) > theta_c; the block is
    kept when (#active columns) / (#valid columns) > theta_m.  A block holding any token pair with t <= 1 is kept
    whatever its density (the never-pruned zone, as in classify_blocks).
    """
    Sb = -(-N // Bs)
    frame = np.arange(N) // Nt
    out = np.zeros((Sb, Sb), dtype=bool)
    for qb in range(Sb):
        r0, r1 = _block_range(qb, Bs, N)
        for kb in range(Sb):
            c0, c1 = _block_range(kb, Bs, N)
            if int(np.abs(frame[r0:r1, None] - frame[None, c0:c1]).min()) <= 1:
                out[qb, kb] = True
                continue
            active = links[r0:r1, c0:c1].sum(axis=0) / float(r1 - r0) > theta_c
            out[qb, kb] = active.sum() / float(c1 - c0) > theta_m
    return out


def build_mask_from_tokens(scores_f32: np.ndarray, N: int, Nt: int, Bs: int, tab: Dict[str, np.ndarray],
                           theta_c: float, theta_m: float, tau_near: float, tau_far: Optional[float] = None
                           ) -> List[List[Tuple[np.ndarray, np.ndarray]]]:
    """Algorithm 1 in the paper's own order, dynamic-threshold mode: token links per frame pair
    (select_token_links), then block aggregation (aggregate_links); CSR per (batch, mask head).
    scores_f32: [B, masks, N, N] float32."""
    scores_f32 = np.asarray(scores_f32)
    assert scores_f32.dtype == np.float32
    B, Hm = scores_f32.shape[:2]
    Sb = -(-N // Bs)
    out = []
    for b in range(B):
        per_b = []
        for m in range(Hm):
            links = select_token_links(scores_f32[b, m], N, Nt, tab, tau_near, tau_near if tau_far is None else tau_far)
            keep = aggregate_links(links, N, Nt, Bs, theta_c, theta_m)
            rowptr = np.zeros(Sb + 1, dtype=np.int64)
            rowptr[1:] = np.cumsum(keep.sum(axis=1))
            per_b.append((rowptr, np.nonzero(keep)[1].astype(np.int64)))
        out.append(per_b)
    return out


def effective_sparsity(rowptr: np.ndarray, Sb: int) -> float:
    """Pruned fraction of block pairs, 1 - nnz / Sb^2."""
    return 1.0 - float(rowptr[-1]) / float(Sb * Sb)


def ratio_for_target_sparsity(cls_map: np.ndarray, target: float, grid: float = 1e-3) -> float:
    """Largest rho on a 1e-3 grid whose static mask reaches the target sparsity.

    The kept count of a static-ratio row depends on the geometry only
    (forced + max(1, floor(n rho))), so rho can be fixed before any score exists.
    """
    Sb = cls_map.shape[0]
    forced = int((cls_map == CLASS_FORCED).sum())
    n_row = ((cls_map == CLASS_NEAR) | (cls_map == CLASS_FAR)).sum(axis=1)
    best = None
    steps = int(round(1.0 / grid))
    for i in range(1, steps + 1):
        rho = i * grid
        kept = forced + sum(static_keep_count(int(n), rho) for n in n_row)
        if 1.0 - kept / float(Sb * Sb) >= target:
            best = rho
    if best is None:
        raise ValueError("target sparsity unreachable for this geometry")
    return best


# --------------------------------------------------------------------------- #
# stage (c): masked attention
# --------------------------------------------------------------------------- #
def masked_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, rowptr: np.ndarray,
                     colidx: np.ndarray, Bs: int, rows: Optional[Sequence[int]] = None,
                     return_lse: bool = False):
    """Eq. 13 with epsilon -> 0 for one (batch, head): Q, K, V [N, d].

    For every valid query token of query block qb: logits a = Q_p . K_q / sqrt(d)
    over the valid key tokens q of the kept key blocks, P = softmax(a),
    O_p = sum_q P_q V_q.  ``rows`` restricts the computation to some query
    blocks; the result is a dict {qb: O_block [n_qb, d]} (and the natural-log
    sum-exp per row if asked).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    N, d = Q.shape
    Sb = -(-N // Bs)
    rows = range(Sb) if rows is None else rows
    out, lse = {}, {}
    for qb in rows:
        r0, r1 = _block_range(qb, Bs, N)
        kbs = colidx[rowptr[qb]:rowptr[qb + 1]]
        if len(kbs) == 0:
            out[qb] = np.zeros((r1 - r0, d))
            lse[qb] = np.full(r1 - r0, -np.inf)
            continue
        keys = np.concatenate([np.arange(*_block_range(int(kb), Bs, N)) for kb in kbs])
        a = (Q[r0:r1] @ K[keys].T) / math.sqrt(d)
        m = a.max(axis=1, keepdims=True)
        e = np.exp(a - m)
        z = e.sum(axis=1, keepdims=True)
        out[qb] = (e / z) @ V[keys]
        lse[qb] = (m + np.log(z))[:, 0]
    return (out, lse) if return_lse else out


def dense_attention_bruteforce(Q: np.ndarray, K: np.ndarray, V: np.ndarray,
                               token_mask: Optional[np.ndarray] = None) -> np.ndarray:
    """Textbook softmax(QK^T/sqrt(d) + log mask) V with explicit Python loops (tiny inputs)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    N, d = Q.shape
    O = np.zeros((N, V.shape[1]))
    for p in range(N):
        logits = []
        for q in range(K.shape[0]):
            if token_mask is not None and not token_mask[p, q]:
                logits.append(-math.inf)
            else:
                logits.append(sum(Q[p, c] * K[q, c] for c in range(d)) / math.sqrt(d))
        m = max(logits)
        if m == -math.inf:
            continue
        ws = [math.exp(x - m) for x in logits]
        z = sum(ws)
        for q, wq in enumerate(ws):
            if wq != 0.0:
                O[p] += (wq / z) * V[q]
    return O


def full_csr(Sb: int) -> Tuple[np.ndarray, np.ndarray]:
    """CSR of the all-ones block mask."""
    return np.arange(Sb + 1, dtype=np.int64) * Sb, np.tile(np.arange(Sb, dtype=np.int64), Sb)


def csr_to_token_mask(rowptr: np.ndarray, colidx: np.ndarray, Bs: int, N: int) -> np.ndarray:
    """Broadcast a block CSR to the token-level mask of Eq. 13 (valid tokens only)."""
    Sb = -(-N // Bs)
    M = np.zeros((N, N), dtype=bool)
    for qb in range(Sb):
        r0, r1 = _block_range(qb, Bs, N)
        for kb in colidx[rowptr[qb]:rowptr[qb + 1]]:
            c0, c1 = _block_range(int(kb), Bs, N)
            M[r0:r1, c0:c1] = True
    return M


# --------------------------------------------------------------------------- #
# evaluation utility: the proxy-task objective of the offline search
# --------------------------------------------------------------------------- #
def attention_matrix(Q: np.ndarray, K: np.ndarray, rowptr: Optional[np.ndarray] = None,
                     colidx: Optional[np.ndarray] = None, Bs: int = 0) -> np.ndarray:
    """Row-normalised attention matrix A[p, q] proportional to exp(Q_p . K_q / sqrt(d)) over the keys the block CSR
    keeps for p's query block (all keys if no CSR is given); rows with no key are zero.  Q, K: [N, d]."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    N, d = Q.shape
    S = (Q @ K.T) / math.sqrt(d)
    if rowptr is not None:
        M = csr_to_token_mask(np.asarray(rowptr), np.asarray(colidx), Bs, N)
        S = np.where(M, S, -np.inf)
    A = np.zeros((N, N))
    for p in range(N):
        row = S[p]
        m = row.max()
        if np.isfinite(m):
            e = np.exp(row - m)
            A[p] = e / e.sum()
    return A


def proxy_loss(A_dense: np.ndarray, A_sparse: np.ndarray, sparsity: float, target: float = 0.80,
               alpha: float = 10.0) -> Tuple[float, float]:
    """Objective of the offline search: ||A_dense - A_sparse||_F^2 / ||A_dense||_F^2 + alpha * max(0, target - sparsity).
    Returns (loss, normalised squared error)."""
    num = float(((A_dense - A_sparse) ** 2).sum())
    den = float((A_dense ** 2).sum())
    nmse = num / den
    return nmse + alpha * max(0.0, target - sparsity), nmse
