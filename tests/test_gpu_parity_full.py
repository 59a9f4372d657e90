"""GPU parity at the benchmark configurations (full sizes, the launch configuration bench.py times).

Scores and masks are compared in full.  The oracle's attention at these sizes would take
minutes per head, so attention is compared on a seeded sample of (head, query block) rows --
rows are independent, each sampled row is checked element by element: the first and last
block (ragged tail), blocks straddling a frame boundary, and random ones.
"""
import numpy as np
import pytest
import torch

import paper_2604_20470_amd as dr
from oracle import dynamicrad_oracle as o
from workloads import CONFIGS

from helpers import GpuRun, assert_masks_equal, oracle_class_map, oracle_masks_from, score_error, to_f64
from test_gpu_parity import ATTN_TOL, SCORE_TOL, _attention_check

pytestmark = pytest.mark.gpu


def _mode_par(wl, cls):
    if wl.mode == "dynamic":
        return "dynamic", wl.tau
    if wl.ratio is not None:
        return "static", wl.ratio
    return "static", o.ratio_for_target_sparsity(cls, wl.target_sparsity)


def _sample_rows(wl, rng, n_random):
    Sb, Bs, Nt = wl.Sb, wl.Bs, wl.Nt
    straddle = [qb for qb in range(Sb) if (qb * Bs) // Nt != (min(wl.N, qb * Bs + Bs) - 1) // Nt]
    rows = {0, Sb - 1}
    rows.update(rng.choice(straddle, size=min(2, len(straddle)), replace=False).tolist() if straddle else [])
    rows.update(rng.integers(0, Sb, n_random).tolist())
    return sorted(rows)


@pytest.mark.parametrize("name,heads,n_heads_attn,n_rows", [
    ("cfg2", None, 3, 6),
    ("cfg3", [0, 1, 7, 39], 2, 4),
    ("cfg4", [0, 1, 22], 2, 3),
    ("cfg5", [0, 1, 13], 2, 3),
])
def test_config_pipeline(name, heads, n_heads_attn, n_rows):
    wl = CONFIGS[name]
    rng = np.random.default_rng(1000 + wl.index)
    run = GpuRun(wl, heads=heads)
    print(f"[{name}] N={wl.N} Sb={wl.Sb} heads={run.heads}", flush=True)
    cls = oracle_class_map(wl)
    assert (run.class_map().cpu().numpy() == cls).all()
    # (a) fused-head scores (heads 0, 1 of the workload are generated first in every subset)
    scores = run.block_scores()
    want = o.block_scores(to_f64(run.Qc[:, :2]), to_f64(run.Kc[:, :2]), wl.Bs, 2)
    err = score_error(scores, want)
    print(f"[{name}] score err {err:.2e}", flush=True)
    assert err <= SCORE_TOL
    # (b) mask from the GPU's fp32 scores, bit-exact
    mode, par = _mode_par(wl, cls)
    rowptr, colidx, nnz, cap = run.build_mask(scores, mode, par)
    masks = oracle_masks_from(scores, cls, mode, par)
    assert_masks_equal(rowptr, colidx, nnz, masks)
    sparsity = o.effective_sparsity(masks[0][0][0], wl.Sb)
    print(f"[{name}] {mode} par={par} nnz={int(nnz[0, 0])} sparsity={sparsity:.4f}", flush=True)
    if wl.target_sparsity:
        assert sparsity >= wl.target_sparsity
    # (c) attention on sampled rows
    hs = rng.choice(len(run.heads), size=n_heads_attn, replace=False).tolist()
    sample = [(0, hi, _sample_rows(wl, rng, n_rows)) for hi in hs]
    worst = _attention_check(run, rowptr, colidx, cap, sample, ATTN_TOL[wl.dtype])
    print(f"[{name}] attention max-abs err {worst:.3e} on {sample}", flush=True)


def test_cfg4_with_all_heads_as_the_benchmark_launches_it():
    """The launch bench.py times: all 40 heads of cfg4 in one call.  The work-item order of the attention kernel depends
    on Sb * H (each XCD walks one contiguous eighth of the items), so a subset of heads takes a different mapping: here
    the rows of the first head, of the head where the last XCD's run starts and of the last head are compared with the
    oracle, the last rows of the last head among them."""
    wl = CONFIGS["cfg4"]
    rng = np.random.default_rng(4040)
    run = GpuRun(wl, threads=12)
    assert len(run.heads) == 40
    cls = oracle_class_map(wl)
    scores = run.block_scores()
    par, achieved = dr.dr_static_ratio_for_sparsity(run.ctx, run.shape, wl.lam, run.params, wl.target_sparsity)
    assert par == o.ratio_for_target_sparsity(cls, wl.target_sparsity)          # the ratio bench.py derives
    rowptr, colidx, nnz, cap = run.build_mask(scores, "static", par)
    masks = oracle_masks_from(scores, cls, "static", par)
    assert_masks_equal(rowptr, colidx, nnz, masks)
    assert abs(achieved - o.effective_sparsity(masks[0][0][0], wl.Sb)) < 1e-12
    Sb = wl.Sb
    sample = [(0, 0, [0, 1, Sb - 1]),
              (0, 35, [0, 1] + rng.integers(0, Sb, 2).tolist()),                  # 7/8 of the items: the last XCD's first
              (0, 39, sorted({Sb - 1, Sb - 2, Sb - 3, *rng.integers(0, Sb, 3).tolist()}))]
    worst = _attention_check(run, rowptr, colidx, cap, sample, ATTN_TOL[wl.dtype])
    print(f"[cfg4 x 40 heads] attention max-abs err {worst:.3e}", flush=True)


@pytest.mark.parametrize("name", ["cfg2", "cfg3"])
def test_per_head_masks_full(name):
    """head_fuse = 0: one mask per head, both modes, selection bit-exact on every head generated."""
    wl = CONFIGS[name]
    heads = None if name == "cfg2" else [0, 5, 17]
    run = GpuRun(wl, heads=heads, params=dr.MaskParams(head_fuse=0))
    scores = run.block_scores()
    want = o.block_scores(to_f64(run.Qc), to_f64(run.Kc), wl.Bs, 0)
    assert score_error(scores, want) <= SCORE_TOL
    cls = oracle_class_map(wl)
    for mode, par in (("static", 0.2), ("dynamic", 0.9)):
        rowptr, colidx, nnz, cap = run.build_mask(scores, mode, par)
        assert_masks_equal(rowptr, colidx, nnz, oracle_masks_from(scores, cls, mode, par))


@pytest.mark.parametrize("name,heads", [("cfg3", [0, 1]), ("cfg4", [0, 1]), ("cfg5", [0, 1])])
def test_paper_selection_rules_full(name, heads):
    """The paper's own rules (z-score thresholds of Eqs. 10-11, seeded uniform sample of Eq. 8) at the full geometries:
    masks bit-exact against the oracle selecting from the GPU's fp32 scores."""
    wl = CONFIGS[name]
    cls = oracle_class_map(wl)
    gs = o.block_frame_gap(wl.N, wl.Nt, wl.Bs)
    run = GpuRun(wl, heads=heads, params=dr.MaskParams(tau_far=0.8, ratio_far=0.02, seed=wl.index))
    scores = run.block_scores()
    s_host = scores.cpu().numpy()
    rowptr, colidx, nnz, cap = run.build_mask(scores, "zscore", 0.3)
    assert_masks_equal(rowptr, colidx, nnz, o.build_mask(s_host, cls, "zscore", 0.3, gap_side=gs, tau_far=0.8))
    print(f"[{name}] zscore nnz={int(nnz[0, 0])} sparsity={1 - int(nnz[0, 0]) / wl.Sb ** 2:.4f}", flush=True)
    rowptr, colidx, nnz, cap = run.build_mask(None, "uniform", 0.05)
    assert_masks_equal(rowptr, colidx, nnz, o.build_mask(s_host, cls, "uniform", 0.05, ratio_far=0.02, seed=wl.index))
    print(f"[{name}] uniform nnz={int(nnz[0, 0])} sparsity={1 - int(nnz[0, 0]) / wl.Sb ** 2:.4f}", flush=True)


@pytest.mark.parametrize("name,bs", [("cfg3", 64), ("cfg3", 32), ("cfg4", 64), ("cfg4", 32), ("micro264k", 32)])
def test_small_block_sizes_full(name, bs):
    """The benchmark geometries at Bs = 64 / 32 (MFMA path that walks the union of several CSR rows): scores, masks in
    full, attention on sampled query blocks."""
    import dataclasses
    wl = dataclasses.replace(CONFIGS[name], Bs=bs)
    rng = np.random.default_rng(2000 + wl.index + bs)
    run = GpuRun(wl, heads=[0, 1, 9])
    cls = oracle_class_map(wl)
    assert (run.class_map().cpu().numpy() == cls).all()
    scores = run.block_scores()
    want = o.block_scores(to_f64(run.Qc[:, :2]), to_f64(run.Kc[:, :2]), wl.Bs, 2)
    assert score_error(scores, want) <= SCORE_TOL
    rowptr, colidx, nnz, cap = run.build_mask(scores, "static", 0.08)
    assert_masks_equal(rowptr, colidx, nnz, oracle_masks_from(scores, cls, "static", 0.08))
    print(f"[{name} Bs={bs}] Sb={wl.Sb} nnz={int(nnz[0, 0])} sparsity={1 - int(nnz[0, 0]) / wl.Sb ** 2:.4f}", flush=True)
    sample = [(0, hi, _sample_rows(wl, rng, 4)) for hi in (0, 2)]
    worst = _attention_check(run, rowptr, colidx, cap, sample, ATTN_TOL[wl.dtype])
    print(f"[{name} Bs={bs}] attention max-abs err {worst:.3e} on {sample}", flush=True)


def test_micro_benchmark_shape_every_rule_on_sampled_rows():
    """264 000 tokens at block size 32 (8250 key blocks per row, up to several thousand selectable ones): the long-row
    code paths of the selection kernels (large sort, radix selection over long rows, the full-width z-score tile).
    Scores in full; the five rules on 150 sampled rows, bit for bit, the oracle selecting from the GPU's scores."""
    wl = CONFIGS["micro264k"]
    rng = np.random.default_rng(264)
    run = GpuRun(wl, heads=[0, 1], params=dr.MaskParams(tau_far=0.8, ratio_far=0.02, seed=7))
    cls = oracle_class_map(wl)
    gs = o.block_frame_gap(wl.N, wl.Nt, wl.Bs)
    scores = run.block_scores()
    want = o.block_scores(to_f64(run.Qc[:, :2]), to_f64(run.Kc[:, :2]), wl.Bs, 2)
    assert score_error(scores, want) <= SCORE_TOL
    s_host = scores[0, 0].cpu().numpy()
    rows = sorted(set(_sample_rows(wl, rng, 140)) | {wl.Sb // 2, 249, 250, 251})
    n_sel = ((cls == 1) | (cls == 2)).sum(axis=1)
    print(f"[micro264k] selectable per row: max {int(n_sel.max())}, sampled max {int(n_sel[rows].max())}", flush=True)

    def check(mode, par, pick):
        rowptr, colidx, nnz, cap = run.build_mask(None if mode == "uniform" else scores, mode, par)
        rp = rowptr[0, 0].cpu().numpy().astype(np.int64)
        ci = colidx[0, 0].cpu().numpy()
        assert rp[-1] == int(nnz[0, 0]) <= cap
        for qb in rows:
            got = ci[rp[qb]:rp[qb + 1]]
            assert np.array_equal(got, pick(qb)), (mode, qb)
        print(f"[micro264k] {mode}: nnz={rp[-1]} sparsity={1 - rp[-1] / wl.Sb ** 2:.4f}", flush=True)

    check("static", 0.1, lambda qb: o.select_static(s_host[qb], cls[qb], 0.1, 0.02))
    check("dynamic", 0.9, lambda qb: o.select_dynamic(s_host[qb], cls[qb], 0.9))
    check("zscore", 0.3, lambda qb: o.select_zscore(s_host[qb], cls[qb], gs[0][qb], gs[1][qb], 0.3, 0.8))
    check("uniform", 0.1, lambda qb: o.select_uniform(qb, cls[qb], 0.1, 0.02, 7))
    run.params = dr.MaskParams(seed=7)                      # one ratio for NEAR and FAR together
    check("static", 0.35, lambda qb: o.select_static(s_host[qb], cls[qb], 0.35, None))
    # gamma = 3 widens the windows: rows of several thousand selectable blocks (sort area beyond 64 KB of LDS)
    run.params = dr.MaskParams(gamma=3.0, seed=7)
    cls = oracle_class_map(wl, gamma=3.0)
    n_sel = ((cls == 1) | (cls == 2)).sum(axis=1)
    rows = sorted({0, wl.Sb - 1, int(np.argmax(n_sel))} | set(rng.integers(0, wl.Sb, 12).tolist()))
    print(f"[micro264k gamma=3] selectable per row: max {int(n_sel.max())}", flush=True)
    assert int(n_sel.max()) > 4096
    check("dynamic", 0.9, lambda qb: o.select_dynamic(s_host[qb], cls[qb], 0.9))
    check("static", 0.2, lambda qb: o.select_static(s_host[qb], cls[qb], 0.2, None))
    check("zscore", 0.3, lambda qb: o.select_zscore(s_host[qb], cls[qb], gs[0][qb], gs[1][qb], 0.3, 0.3))


def test_zscore_masks_in_full_at_24_frames_block_32():
    """24 frames of 40 x 80 tokens at block size 32 (2400 key blocks per row, candidate sets of up to 101 blocks): the
    z-score rule's masks in full, bit for bit, fused and per head."""
    from workloads import Workload
    wl = Workload("f24b32", 41, 1, 2, 128, 24, 40, 80, 32, "bf16", "field", "dynamic", 0.5, 0.9, 0.7)
    cls = oracle_class_map(wl, gamma=2.0)
    gs = o.block_frame_gap(wl.N, wl.Nt, wl.Bs)
    for head_fuse, tau, tau_far in ((2, 0.3, 0.8), (0, -0.5, None)):
        run = GpuRun(wl, params=dr.MaskParams(gamma=2.0, head_fuse=head_fuse, tau_far=tau_far))
        scores = run.block_scores()
        rowptr, colidx, nnz, cap = run.build_mask(scores, "zscore", tau)
        want = o.build_mask(scores.cpu().numpy(), cls, "zscore", tau, gap_side=gs, tau_far=tau_far)
        assert_masks_equal(rowptr, colidx, nnz, want)
        print(f"[24 frames Bs=32, head_fuse={head_fuse}] nnz={int(nnz[0, 0])} of {int((cls != 0).sum())} candidates", flush=True)
