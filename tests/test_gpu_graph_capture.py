"""After one eager call (which sizes the context's scratch and caches the geometry) the three stages only enqueue
kernels, so the sequence can be captured in a HIP graph and replayed on new input values."""
import pytest
import torch

import paper_2604_20470_amd as dr
from workloads import CONFIGS, tiny_case

from helpers import GpuRun

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wl,mode,par", [(CONFIGS["cfg2"], dr.MODE_STATIC, 0.2), (tiny_case("ragged128", Bs=32), dr.MODE_ZSCORE, 0.3),
                                         (tiny_case("tiny8"), dr.MODE_DYNAMIC, 0.9)],
                         ids=["cfg2-static", "ragged-bs32-zscore", "tiny8-f32-dynamic"])
def test_three_stage_call_replays_from_a_graph(wl, mode, par):
    run = GpuRun(wl)
    ctx, shape, params = run.ctx, run.shape, run.params
    Sb = wl.Sb
    cap, _ = dr.dr_mask_capacity(ctx, shape, wl.lam, params)
    scores = torch.empty((wl.B, 1, Sb, Sb), dtype=torch.float32, device="cuda")
    rowptr = torch.empty((wl.B, 1, Sb + 1), dtype=torch.int32, device="cuda")
    colidx = torch.zeros((wl.B, 1, cap), dtype=torch.int32, device="cuda")
    nnz = torch.empty((wl.B, 1), dtype=torch.int64, device="cuda")
    Q, K, V = run.Q.clone(), run.K.clone(), run.V.clone()
    O = torch.empty_like(Q)

    def call():
        dr.dr_block_scores(ctx, shape, Q, K, params.head_fuse, scores)
        dr.dr_build_mask(ctx, shape, mode, par, wl.lam, params, scores, rowptr, colidx, cap, nnz)
        dr.dr_sparse_attn_fwd(ctx, shape, Q, K, V, rowptr, colidx, 1, cap, O)

    call()                                   # eager: allocations and the one synchronising geometry build happen here
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call()                               # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(5)
    for rep in range(3):
        # new values in the captured buffers, eager work and synchronisations between the replays
        for t in (Q, K, V):
            t.copy_((t.float() * 0.5 + 0.5 * torch.randn(t.shape, generator=gen, device="cuda")).to(t.dtype))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (O.clone(), rowptr.clone(), colidx.clone(), nnz.clone(), scores.clone())
        O.fill_(float("nan")); rowptr.zero_(); nnz.zero_(); scores.zero_(); colidx.zero_()
        call()
        torch.cuda.synchronize()
        assert torch.equal(got[4], scores) and torch.equal(got[1], rowptr) and torch.equal(got[3], nnz), rep
        n = int(nnz[0, 0])
        assert torch.equal(got[2][0, 0, :n], colidx[0, 0, :n])
        assert torch.equal(got[0], O), rep
