"""dr_sparse_attn_fwd_static (the entry point for callers that cannot allocate) against dr_sparse_attn_fwd, through the C
ABI: two calls in a row, the second on a smaller input, on every attention path that uses scratch; results must be
identical bit for bit (same kernels, only the scratch lives elsewhere).  Collected last (file name), so that a failure
here hides no other test."""
from __future__ import annotations

import dataclasses

import numpy as np
import pytest
import torch

import paper_2604_20470_amd as dr
from oracle import dynamicrad_oracle as o
from workloads import tiny_case

from helpers import GpuRun, oracle_class_map, oracle_masks_from

pytestmark = pytest.mark.gpu


def _both(run: GpuRun, rowptr, colidx, cap):
    """(O, lse) of the allocating entry point and of the static one on the same inputs."""
    out = []
    for fn in (dr.dr_sparse_attn_fwd, dr.dr_sparse_attn_fwd_static):
        O = torch.full_like(run.Q, float("nan"))
        lse = torch.full((run.wl.B, len(run.heads), run.wl.N), float("nan"), dtype=torch.float32, device="cuda")
        fn(run.ctx, run.shape, run.Q, run.K, run.V, rowptr, colidx, rowptr.shape[1], cap, O, lse)
        torch.cuda.synchronize()
        out.append((O, lse))
    return out


def _masked_run(frames: int, bs: int):
    wl = dataclasses.replace(tiny_case("ragged128"), Bs=bs, Nf=frames)
    run = GpuRun(wl)
    scores = run.block_scores()
    rowptr, colidx, nnz, cap = run.build_mask(scores, wl.mode, wl.ratio if wl.mode == "static" else wl.tau)
    return run, rowptr, colidx, cap


@pytest.mark.parametrize("bs", [128, 64, 32])
def test_static_scratch_entry_matches_the_allocating_one_twice_in_a_row(bs):
    big, small = _masked_run(7, bs), _masked_run(4, bs)
    assert small[0].wl.N < big[0].wl.N
    for run, rowptr, colidx, cap in (big, small):        # the second call is the smaller one
        (O_a, lse_a), (O_s, lse_s) = _both(run, rowptr, colidx, cap)
        assert torch.isfinite(O_a.float()).all()
        assert torch.equal(O_a.view(torch.int16), O_s.view(torch.int16))
        assert torch.equal(lse_a.view(torch.int32), lse_s.view(torch.int32))
    # and against the oracle once, so that "identical" is not "identically wrong"
    run, rowptr, colidx, cap = small
    wl = run.wl
    rp = rowptr[0, 0].cpu().numpy().astype(np.int64)
    ci = colidx[0, 0].cpu().numpy().astype(np.int64)
    O = torch.full_like(run.Q, float("nan"))
    dr.dr_sparse_attn_fwd_static(run.ctx, run.shape, run.Q, run.K, run.V, rowptr, colidx, rowptr.shape[1], cap, O, None)
    torch.cuda.synchronize()
    f64 = lambda t: t.to(torch.float64).cpu().numpy()
    want = o.masked_attention(f64(run.Qc[0, 0]), f64(run.Kc[0, 0]), f64(run.Vc[0, 0]), rp, ci, wl.Bs)
    worst = max(float(np.abs(f64(O[0, 0, qb * wl.Bs: qb * wl.Bs + blk.shape[0]]) - blk).max()) for qb, blk in want.items())
    assert worst <= 2e-2, worst


def test_static_scratch_entry_refuses_what_does_not_fit():
    """A mask capacity whose merged lists alone exceed the 16 MiB area: refused on the host, nothing launched."""
    run, rowptr, colidx, cap = _masked_run(7, 128)
    huge = 5_000_000                                           # entries: 20 MB of merged lists
    colidx_big = torch.zeros((1, 1, huge), dtype=torch.int32, device="cuda")
    colidx_big[0, 0, :colidx.shape[2]] = colidx[0, 0]
    O = torch.full_like(run.Q, float("nan"))
    with pytest.raises(dr.DRError) as e:
        dr.dr_sparse_attn_fwd_static(run.ctx, run.shape, run.Q, run.K, run.V, rowptr, colidx_big, 1, huge, O, None)
    assert "static area" in str(e.value) and "16777216" in str(e.value)
    dr.dr_sparse_attn_fwd(run.ctx, run.shape, run.Q, run.K, run.V, rowptr, colidx_big, 1, huge, O, None)   # the other one takes it
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all()
