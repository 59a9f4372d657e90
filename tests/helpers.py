"""Shared plumbing for the GPU parity tests: run the library stages on a workload and
compute the oracle's answer for the same bits."""
from __future__ import annotations

import numpy as np
import torch

import paper_2604_20470_amd as dr
from oracle import dynamicrad_oracle as o
from workloads import Workload, make_qkv
from workloads.generate import make_head, round_to_dtype

DEFAULT = dict(gamma=1.0, theta_c=0.15, theta_m=0.60)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_class_map(wl: Workload, gamma=1.0, theta_c=0.15, theta_m=0.60, lam=None):
    tab = o.frame_table(wl.Nf, wl.Nt, wl.Bs, gamma, wl.lam if lam is None else lam)
    return o.classify_blocks(wl.N, wl.Nt, wl.Bs, tab, theta_c, theta_m)


def make_qkv_threaded(wl: Workload, heads, workers: int = 12):
    """make_qkv with the heads generated on host threads (bit-identical: every head has its own random stream)."""
    from concurrent.futures import ThreadPoolExecutor
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    out = [torch.empty((wl.B, len(heads), wl.N, wl.d), dtype=tdt) for _ in range(3)]

    def one(job):
        b, i = job
        return b, i, [round_to_dtype(x, wl.dtype) for x in make_head(wl, b, heads[i])]

    with ThreadPoolExecutor(max_workers=workers) as ex:
        for b, i, tensors in ex.map(one, [(b, i) for b in range(wl.B) for i in range(len(heads))]):
            for dst, src in zip(out, tensors):
                dst[b, i].copy_(src)
    return out


class GpuRun:
    """Device tensors + library handles for one workload."""

    def __init__(self, wl: Workload, heads=None, device="cuda:0", params: dr.MaskParams = None, threads: int = 0):
        self.wl = wl
        self.heads = list(range(wl.H)) if heads is None else list(heads)
        gen = (lambda: make_qkv_threaded(wl, self.heads, threads)) if threads else (lambda: make_qkv(wl, self.heads))
        self.Qc, self.Kc, self.Vc = gen()                                  # CPU, run dtype
        self.Q, self.K, self.V = (t.to(device) for t in (self.Qc, self.Kc, self.Vc))
        self.ctx = dr.Context(0)
        self.shape = dr.shape_of(self.Q, wl.Nf, wl.Hg, wl.Wg, wl.Bs)
        self.params = params if params is not None else dr.MaskParams(head_fuse=wl.head_fuse)
        self.device = device
        self.Sb = wl.Sb

    @property
    def masks(self) -> int:
        return 1 if self.params.head_fuse > 0 else len(self.heads)

    def block_scores(self) -> torch.Tensor:
        s = torch.full((self.wl.B, self.masks, self.Sb, self.Sb), float("nan"), dtype=torch.float32, device=self.device)
        dr.dr_block_scores(self.ctx, self.shape, self.Q, self.K, self.params.head_fuse, s)
        torch.cuda.synchronize()
        return s

    def class_map(self, lam=None) -> torch.Tensor:
        cm = torch.full((self.Sb, self.Sb), 255, dtype=torch.uint8, device=self.device)
        dr.dr_class_map(self.ctx, self.shape, self.wl.lam if lam is None else lam, self.params, cm)
        torch.cuda.synchronize()
        return cm

    def build_mask(self, scores: torch.Tensor, mode: str, par: float, capacity: int = None, lam=None):
        lam = self.wl.lam if lam is None else lam
        if capacity is None:
            capacity, _ = dr.dr_mask_capacity(self.ctx, self.shape, lam, self.params)
        B, M = self.wl.B, self.masks
        guard = 64
        rowptr = torch.full((B, M, self.Sb + 1), -7, dtype=torch.int32, device=self.device)
        colidx = torch.full((B * M * capacity + guard,), -7, dtype=torch.int32, device=self.device)
        nnz = torch.full((B, M), -7, dtype=torch.int64, device=self.device)
        code = {"static": dr.MODE_STATIC, "dynamic": dr.MODE_DYNAMIC, "zscore": dr.MODE_ZSCORE,
                "uniform": dr.MODE_UNIFORM}[mode]
        dr.dr_build_mask(self.ctx, self.shape, code, par, lam, self.params, scores, rowptr, colidx, capacity, nnz)
        torch.cuda.synchronize()
        assert (colidx[B * M * capacity:] == -7).all(), "colidx guard overwritten"
        return rowptr, colidx[:B * M * capacity].view(B, M, capacity), nnz, capacity

    def attention(self, rowptr, colidx, capacity, want_lse=False):
        O = torch.full_like(self.Q, float("nan"))
        lse = torch.full((self.wl.B, len(self.heads), self.wl.N), float("nan"), dtype=torch.float32,
                         device=self.device) if want_lse else None
        dr.dr_sparse_attn_fwd(self.ctx, self.shape, self.Q, self.K, self.V, rowptr, colidx, rowptr.shape[1], capacity,
                              O, lse)
        torch.cuda.synchronize()
        return (O, lse) if want_lse else O


def oracle_masks_from(scores_gpu: torch.Tensor, cls_map: np.ndarray, mode: str, par: float, ratio_far=None):
    return o.build_mask(scores_gpu.cpu().numpy(), cls_map, mode, par, ratio_far)


def assert_masks_equal(rowptr, colidx, nnz, masks_oracle):
    rp = rowptr.cpu().numpy()
    ci = colidx.cpu().numpy()
    nz = nnz.cpu().numpy()
    B, M = rp.shape[:2]
    for b in range(B):
        for m in range(M):
            orp, oci = masks_oracle[b][m]
            assert nz[b, m] == orp[-1], (b, m, nz[b, m], orp[-1])
            assert (rp[b, m] == orp).all(), (b, m)
            assert (ci[b, m, :orp[-1]] == oci).all(), (b, m)


def score_error(got: torch.Tensor, want: np.ndarray) -> float:
    """max |g - o| / max(|o|, rms(o over the (b, mask) slice)): the 1e-5 'relative' bar."""
    g = got.cpu().numpy().astype(np.float64)
    rms = np.sqrt((want ** 2).mean(axis=(2, 3), keepdims=True))
    return float((np.abs(g - want) / np.maximum(np.abs(want), rms)).max())
