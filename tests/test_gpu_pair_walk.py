"""Block sizes 128 and 64, bf16, d = 128: the attention kernel in which 256 queries (two or four adjacent query blocks)
walk the merged list of their rows, against the oracle on hand-made CSR lists that reach its corner cases (ownership
patterns of the merged list, the sequence's last key block in its shapes, a last group that is not full, empty rows,
lists longer than one register window), and the kernels it replaced kept under test through DR_ATTN_PAIRS=0.  Every
row is compared."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2604_20470_amd as dr
from oracle import dynamicrad_oracle as o
from workloads import tiny_case

from helpers import GpuRun, to_f64

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _case(frames, hg, wg, H=2, seed_index=41, bs=128):
    """bf16, d = 128; N = frames * hg * wg."""
    return dataclasses.replace(tiny_case("ragged128"), Nf=frames, Hg=hg, Wg=wg, H=H, index=seed_index, Bs=bs)


def _csr(rows, Sb):
    rp = np.zeros(Sb + 1, dtype=np.int64)
    ci = []
    for qb in range(Sb):
        ci.extend(rows[qb])
        rp[qb + 1] = len(ci)
    return rp, np.asarray(ci if ci else [0], dtype=np.int64)


def _check(run, rp, ci, lse_too=True):
    wl = run.wl
    rowptr = torch.from_numpy(rp.astype(np.int32)).view(1, 1, -1).contiguous().cuda()
    colidx = torch.from_numpy(ci.astype(np.int32)).view(1, 1, -1).contiguous().cuda()
    O, lse = run.attention(rowptr, colidx, colidx.shape[2], want_lse=True)
    worst = 0.0
    for h in range(len(run.heads)):
        want, want_lse = o.masked_attention(to_f64(run.Qc[0, h]), to_f64(run.Kc[0, h]), to_f64(run.Vc[0, h]), rp, ci, wl.Bs,
                                            return_lse=True)
        for qb, blk in want.items():
            got = to_f64(O[0, h, qb * wl.Bs: qb * wl.Bs + blk.shape[0]])
            worst = max(worst, float(np.abs(got - blk).max()))
            if lse_too:
                g = lse[0, h, qb * wl.Bs: qb * wl.Bs + blk.shape[0]].cpu().numpy().astype(np.float64)
                w = want_lse[qb]
                both_inf = np.isinf(g) & np.isinf(w) & (g < 0) & (w < 0)
                with np.errstate(invalid="ignore"):
                    close = np.abs(g - w) <= 5e-2
                assert (both_inf | close).all(), (qb, g[:4], w[:4])
    assert worst <= TOL, worst
    return worst


def _rows(Sb, rng, density, force_last=None):
    rows = []
    for qb in range(Sb):
        keep = sorted(set(np.nonzero(rng.random(Sb) < density)[0].tolist()))
        if force_last is True and Sb - 1 not in keep:
            keep.append(Sb - 1)
        if force_last is False:
            keep = [k for k in keep if k != Sb - 1]
        rows.append(sorted(keep))
    return rows


@pytest.mark.parametrize("pairs", ["1", "0"])
@pytest.mark.parametrize("bs", [128, 64, 32])
@pytest.mark.parametrize("frames,hg,wg,what", [
    (7, 9, 21, "last key block of 43 keys: a partial first chunk only"),        # N = 1323 = 10 * 128 + 43
    (8, 10, 17, "last key block of 80 (16) keys: one full chunk and a partial one"),  # N = 1360 = 10 * 128 + 80
    (10, 8, 16, "last key block full"),                                           # N = 1280
    (3, 8, 24, "last key block of exactly 64 keys"),                              # N = 576 = 4 * 128 + 64
])
def test_random_lists_against_the_oracle(frames, hg, wg, what, bs, pairs, monkeypatch):
    monkeypatch.setenv("DR_ATTN_PAIRS", pairs)
    run = GpuRun(_case(frames, hg, wg, bs=bs))
    Sb = run.wl.Sb
    rng = np.random.default_rng(frames * 100 + hg)
    rows = _rows(Sb, rng, 0.45)
    rows[0] = []                                            # an empty row inside a pair
    if Sb > 3:
        rows[2], rows[3] = [], []                           # a pair with nothing to do
    rows[1] = list(range(Sb))                               # a full row beside an empty one
    rp, ci = _csr(rows, Sb)
    _check(run, rp, ci)


def test_ownership_patterns_of_four_rows_at_block_size_64(monkeypatch):
    """Four query blocks per workgroup: every wave owns its own subset of the merged list (disjoint rows, one row that
    lists everything beside three that list nothing, identical rows, the partial last key block listed by one wave
    only), and the last group holds a single query block."""
    monkeypatch.setenv("DR_ATTN_PAIRS", "1")
    run = GpuRun(_case(8, 10, 17, bs=64))
    Sb = run.wl.Sb                                           # 22: N = 1360 = 21 * 64 + 16; groups of four: 5 full + 2 blocks
    assert Sb == 22
    rows = [[] for _ in range(Sb)]
    rows[0], rows[1], rows[2], rows[3] = [0, 4, 8, 12], [1, 5, 9, 21], [2, 6, 10], [3, 7, 11]      # disjoint
    rows[4] = list(range(Sb))                                                                      # rows 5..7 empty
    rows[8], rows[9], rows[10], rows[11] = [3, 20, 21], [3, 20, 21], [3, 20, 21], [3, 20, 21]      # identical
    rows[12], rows[13], rows[14], rows[15] = [21], [0], [], [0, 21]                                # the partial block, owners vary
    rows[16], rows[17], rows[18], rows[19] = [5, 6, 7, 8], [6, 7], [7], [4, 5, 6, 7, 8, 9]        # nested
    rows[20], rows[21] = [0, 1, 21], [20]                                                          # the last group: two blocks
    rp, ci = _csr(rows, Sb)
    _check(run, rp, ci)


def test_ownership_patterns_of_eight_rows_at_block_size_32(monkeypatch):
    """Eight query blocks per workgroup, two per wave, a chunk = two entries of the merged list: the four 32 x 32 tiles
    of a wave's chunk each have their own owner bit.  Rows that list disjoint key blocks (every tile pattern with one
    owner), one row that lists everything beside seven empty ones, identical rows, an odd number of entries, the
    partial last key block (11 keys) listed by one query block of a wave only, by both, and by another wave; a last
    group of one query block."""
    monkeypatch.setenv("DR_ATTN_PAIRS", "1")
    run = GpuRun(_case(7, 9, 21, bs=32))
    Sb = run.wl.Sb                                           # 42: N = 1323 = 41 * 32 + 11; groups of eight: 5 full + 2 blocks
    assert Sb == 42
    rows = [[] for _ in range(Sb)]
    for r in range(8):
        rows[r] = [r, r + 8, r + 17, 41 - r]                 # disjoint (row 0 lists the partial block): 32 entries
    rows[8] = list(range(Sb))                                # rows 9..15 empty
    for r in range(16, 24):
        rows[r] = [3, 20, 40]                                # identical, odd count
    rows[24], rows[25], rows[26], rows[27] = [41], [0], [0, 41], [41]       # the partial block: one half of wave 0, both of wave 1
    rows[28], rows[29], rows[30], rows[31] = [5, 6, 7, 8], [6, 7], [], [4, 5, 6, 7, 8, 9, 41]
    rows[32], rows[33], rows[34] = [0, 1, 2], [1, 2, 3], [2]                # rows 35..39 empty: waves 2, 3 sit every chunk out
    rows[40], rows[41] = [0, 1, 41], [40]                    # the last group: two blocks, one wave
    rp, ci = _csr(rows, Sb)
    _check(run, rp, ci)


def test_ownership_patterns_of_the_merged_list(monkeypatch):
    """Disjoint rows (every chunk skipped by one half of the workgroup), a row that is a strict subset of its
    neighbour, identical rows, and a pair whose merged list starts with a block that only the second row lists (the
    exponent reference of the first row then comes from a key block it does not attend to)."""
    monkeypatch.setenv("DR_ATTN_PAIRS", "1")
    run = GpuRun(_case(8, 10, 17))
    Sb = run.wl.Sb                                           # 11
    rows = [[] for _ in range(Sb)]
    rows[0], rows[1] = [0, 2, 4, 6, 8, 10], [1, 3, 5, 7, 9]            # disjoint; row 0 lists the partial last block
    rows[2], rows[3] = [1, 2, 3, 4, 5, 6], [3, 4]                        # subset
    rows[4], rows[5] = [0, 5, 10], [0, 5, 10]                            # identical, with the last block
    rows[6], rows[7] = [4, 9], [0, 9]                                    # merged list starts with a block of row 7 only
    rows[8], rows[9] = [10], [10]                                        # only the partial last block
    rows[10] = [0, 1]                                                    # the odd block at the end: a pair of one
    rp, ci = _csr(rows, Sb)
    _check(run, rp, ci)


@pytest.mark.parametrize("bs", [128, 32])
def test_lists_longer_than_one_register_window_and_per_head_masks(bs, monkeypatch):
    """More than 64 key blocks in a merged list (the walk reloads its window), with one mask per head."""
    monkeypatch.setenv("DR_ATTN_PAIRS", "1")
    wl = _case(10, 30, 32, H=2, bs=bs)                       # N = 9600: 75 key blocks of 128, 300 of 32
    run = GpuRun(wl)
    Sb = wl.Sb
    rng = np.random.default_rng(9600)
    per_head = []
    for h in range(2):
        rows = [[] for _ in range(Sb)]
        for qb in (0, 1, 36, 37, Sb - 1):
            rows[qb] = sorted(set(np.nonzero(rng.random(Sb) < 0.93)[0].tolist()))
        per_head.append(_csr(rows, Sb))
    cap = max(len(ci) for _, ci in per_head)
    rowptr = torch.zeros((1, 2, Sb + 1), dtype=torch.int32)
    colidx = torch.zeros((1, 2, cap), dtype=torch.int32)
    for h, (rp, ci) in enumerate(per_head):
        rowptr[0, h] = torch.from_numpy(rp.astype(np.int32))
        colidx[0, h, :len(ci)] = torch.from_numpy(ci.astype(np.int32))
    O = torch.full_like(run.Q, float("nan"))
    dr.dr_sparse_attn_fwd(run.ctx, run.shape, run.Q, run.K, run.V, rowptr.cuda(), colidx.cuda(), 2, cap, O, None)
    torch.cuda.synchronize()
    worst = 0.0
    for h, (rp, ci) in enumerate(per_head):
        want = o.masked_attention(to_f64(run.Qc[0, h]), to_f64(run.Kc[0, h]), to_f64(run.Vc[0, h]), rp, ci, wl.Bs,
                                  rows=[0, 1, 36, 37, Sb - 1])
        for qb, blk in want.items():
            worst = max(worst, float(np.abs(to_f64(O[0, h, qb * wl.Bs: qb * wl.Bs + blk.shape[0]]) - blk).max()))
        for qb in (2, 35, 38):
            assert (O[0, h, qb * wl.Bs:(qb + 1) * wl.Bs] == 0).all()
    assert worst <= TOL, worst


def test_rows_the_pair_walk_hands_to_the_second_pass(monkeypatch):
    """Logits that rise far above those of the merged list's first chunk (a per-block constant channel): the pair walk
    keeps its exponent reference, so the normaliser leaves the range it checks, the rows are flagged and the second pass
    (moving reference, fp32 scaling) recomputes them."""
    monkeypatch.setenv("DR_ATTN_PAIRS", "1")
    run = GpuRun(_case(8, 10, 17))
    wl = run.wl
    Sb, Bs = wl.Sb, wl.Bs
    Qc, Kc = run.Qc.clone(), run.Kc.clone()
    Qc[..., 0] = 8.0
    for j in range(Sb):
        Kc[:, :, j * Bs:(j + 1) * Bs, 0] = 24.0 * j                     # +17 nats per key block
    run.Qc, run.Kc = Qc, Kc
    run.Q, run.K = Qc.cuda(), Kc.cuda()
    rp, ci = o.full_csr(Sb)
    _check(run, rp, ci, lse_too=False)
