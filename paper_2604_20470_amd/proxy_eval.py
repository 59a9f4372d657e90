"""Evaluation utility on the GPU path: the objective of the paper's offline parameter search on its proxy task
(App. C: drift-proxy features, proxy attention matrix, Eq. 22), computed with the library's own three stages.

The attention *matrix* is not an output of the hot path, so it is read off the attention kernel column block by
column block: with V set to the 128 one-hot columns of a key range, O = A V is that column range of A.  fp32 tensors
keep the read-out exact to fp32 rounding (they run the fp32 attention kernel).  Meant for the small N of the proxy
task (N x N floats are materialised); the Frobenius norms and the penalty are reduced on the device by dr_proxy_loss.
"""
from __future__ import annotations

from typing import Tuple

from . import binding as dr

MODE_TOKENS = -1     # proxy_loss: build the mask with Algorithm 1 in its own order (token links, then aggregation)


def attention_matrix(ctx: dr.Context, shape: dr.Shape, Q, K, rowptr, colidx, mask_heads: int, capacity: int):
    """A[b, h, p, q] under the block CSR, float32 torch tensor on Q's device.  Q, K: [B, H, N, d] float32."""
    import torch
    B, H, N, d = Q.shape
    assert Q.dtype == torch.float32 and K.dtype == torch.float32, "the read-out uses the fp32 attention path"
    A = torch.zeros((B, H, N, N), dtype=torch.float32, device=Q.device)
    V = torch.zeros_like(Q)
    O = torch.empty_like(Q)
    for c0 in range(0, N, d):
        w = min(d, N - c0)
        V.zero_()
        idx = torch.arange(w, device=Q.device)
        V[:, :, c0 + idx, idx] = 1.0                      # key c0 + j carries the unit vector e_j
        dr.dr_sparse_attn_fwd(ctx, shape, Q, K, V, rowptr, colidx, mask_heads, capacity, O)
        A[:, :, :, c0:c0 + w] = O[:, :, :, :w]
    torch.cuda.synchronize()
    return A


def proxy_loss(ctx: dr.Context, Q, K, Nf: int, Hg: int, Wg: int, Bs: int, mode: int, ratio_or_tau: float, lam: float,
               params: dr.MaskParams, target: float = 0.80, alpha: float = 10.0) -> Tuple[float, float, float]:
    """(loss, normalised squared error, effective sparsity) of one configuration on given features, averaged over
    (batch, head); `mode` is one of the library's selection rules or MODE_TOKENS: ||A_dense - A_sparse||_F^2 / ||A_dense||_F^2 + alpha * max(0, target - sparsity)."""
    import torch
    B, H, N, d = Q.shape
    shape = dr.shape_of(Q, Nf, Hg, Wg, Bs)
    Sb = shape.Sb
    masks = 1 if params.head_fuse > 0 else H
    cap, _ = dr.dr_mask_capacity(ctx, shape, lam, params)
    scores = torch.empty((B, masks, Sb, Sb), dtype=torch.float32, device=Q.device)
    rowptr = torch.empty((B, masks, Sb + 1), dtype=torch.int32, device=Q.device)
    colidx = torch.empty((B, masks, cap), dtype=torch.int32, device=Q.device)
    nnz = torch.empty((B, masks), dtype=torch.int64, device=Q.device)
    if mode == MODE_TOKENS:          # ratio_or_tau is tau_1; tau_2 comes from params
        tscores = torch.empty((B, masks, N, N), dtype=torch.float32, device=Q.device)
        dr.dr_token_scores(ctx, shape, Q, K, params.head_fuse, tscores)
        dr.dr_build_mask_tokens(ctx, shape, ratio_or_tau, lam, params, tscores, rowptr, colidx, cap, nnz)
    else:
        dr.dr_block_scores(ctx, shape, Q, K, params.head_fuse, scores)
        dr.dr_build_mask(ctx, shape, mode, ratio_or_tau, lam, params, scores, rowptr, colidx, cap, nnz)
    A_sparse = attention_matrix(ctx, shape, Q, K, rowptr, colidx, masks, cap)
    # dense reference through the same kernel: the all-ones block mask
    full_rp = (torch.arange(Sb + 1, dtype=torch.int32, device=Q.device) * Sb).view(1, 1, -1).repeat(B, 1, 1).contiguous()
    full_ci = torch.arange(Sb, dtype=torch.int32, device=Q.device).repeat(Sb).view(1, 1, -1).repeat(B, 1, 1).contiguous()
    A_dense = attention_matrix(ctx, shape, Q, K, full_rp, full_ci, 1, Sb * Sb)
    assert A_dense.is_contiguous() and A_sparse.is_contiguous() and nnz.is_contiguous()
    out = torch.empty(3, dtype=torch.float64, device=Q.device)
    dr.dr_proxy_loss(ctx, A_dense, A_sparse, nnz, Sb, target, alpha, out)
    loss, nmse, sparsity = out.tolist()
    return loss, nmse, sparsity
