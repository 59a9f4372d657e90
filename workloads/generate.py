"""Seeded input generators for the five benchmark shapes plus tiny test cases.

Every tensor is produced per (batch, head) from its own numpy Philox stream, so
a test that needs only a few heads of a 40-head workload can generate just
those, bit-identically to a full generation.

Value recipes (synthetic stand-ins for DiT activations, which are not
available offline):

* ``iid``    Q, K, V ~ N(0, 1) independently per element.
* ``field``  Q = F + 0.3 xi_Q, K = F + 0.3 xi_K with F a random-Fourier-feature
             field over the (t, y, x) token grid:
             F[p, c] = sqrt(2) cos(2 pi (ft_c t/Nf + fy_c y/Hg + fx_c x/Wg) + phi_c),
             real-valued frequencies (ft, fy, fx) ~ N(0, sigma_f^2 I) with
             sigma_f = 1 cycle per extent and phi ~ U[0, 2 pi) drawn once per
             (head, channel).  E[Q_p . K_q]/sqrt(d) then decays monotonically
             with spatio-temporal distance (a Gaussian kernel), which is the
             energy-decay structure the method's locality prior assumes.
             V ~ N(0, 1).
* ``blob``   ``field`` plus g(p) * b_c added to both Q and K, where g is a
             Gaussian bump of amplitude 1.5 moving linearly across the grid
             over the frames and b a fixed N(0,1) vector per head: tokens on
             the moving object correlate across distant frames.

Values are computed in float64/float32 on the host and rounded once to the run
dtype (float32, or bfloat16 via torch); consumers on both sides read the
rounded values.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 20470
SIGMA_F = 1.0        # cycles per extent
NOISE = 0.3          # iid noise amplitude added to the field
BLOB_AMP = 1.5


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int            # seeds the streams
    B: int
    H: int
    d: int
    Nf: int
    Hg: int
    Wg: int
    Bs: int
    dtype: str            # "f32" | "bf16"
    recipe: str           # "iid" | "field" | "blob"
    mode: str             # "static" | "dynamic"
    ratio: Optional[float]    # static keep ratio (None: derive from target sparsity)
    tau: Optional[float]      # dynamic cumulative-mass threshold
    lam: float
    target_sparsity: Optional[float] = None
    head_fuse: int = 2

    @property
    def Nt(self) -> int:
        return self.Hg * self.Wg

    @property
    def N(self) -> int:
        return self.Nf * self.Nt

    @property
    def Sb(self) -> int:
        return -(-self.N // self.Bs)


CONFIGS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", 1, 1, 2, 64, 4, 8, 8, 64, "f32", "iid", "static", 0.5, None, 0.5),
    "cfg2": Workload("cfg2", 2, 1, 8, 128, 8, 24, 32, 128, "bf16", "field", "static", 0.2, None, 0.5),
    "cfg3": Workload("cfg3", 3, 1, 40, 128, 21, 30, 52, 128, "bf16", "field", "dynamic", None, 0.9, 0.3),
    "cfg4": Workload("cfg4", 4, 1, 40, 128, 21, 45, 80, 128, "bf16", "field", "static", None, None, 0.5,
                     target_sparsity=0.85),
    "cfg5": Workload("cfg5", 5, 1, 24, 128, 33, 45, 80, 128, "bf16", "blob", "dynamic", None, 0.95, 0.7),
    # the shape of the paper's layer micro-benchmark (selector overhead appendix): ~264K tokens, block size 32
    "micro264k": Workload("micro264k", 6, 1, 24, 128, 33, 80, 100, 32, "bf16", "field", "static", None, None, 0.5,
                          target_sparsity=0.85),
}


def get_workload(name: str) -> Workload:
    return CONFIGS[name]


def tiny_case(name: str = "tiny8", **over) -> Workload:
    """Small shapes that, unlike cfg1, leave a non-empty selectable set.

    tiny8:  8 frames x 8x8 tokens, block 32, d=64, lambda=1.0
    ragged: 6 frames x 6x10 tokens (Nt=60, not a multiple of the block), block 32
    """
    base = {
        "tiny8": Workload("tiny8", 11, 1, 4, 64, 8, 8, 8, 32, "f32", "field", "static", 0.5, 0.9, 1.0),
        "ragged": Workload("ragged", 12, 2, 3, 64, 6, 6, 10, 32, "f32", "field", "dynamic", 0.4, 0.8, 1.0),
        "ragged128": Workload("ragged128", 13, 1, 3, 128, 7, 9, 21, 128, "bf16", "blob", "static", 0.3, 0.9, 0.7),
    }[name]
    return dataclasses.replace(base, **over)


def _rng(wl: Workload, kind: int, b: int, h: int) -> np.random.Generator:
    ss = np.random.SeedSequence([BASE_SEED, wl.index, kind, b, h])
    return np.random.Generator(np.random.Philox(ss))


def _grid(wl: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    p = np.arange(wl.N, dtype=np.int64)
    t = p // wl.Nt
    r = p % wl.Nt
    return t.astype(np.float64), (r // wl.Wg).astype(np.float64), (r % wl.Wg).astype(np.float64)


def make_head(wl: Workload, b: int, h: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Q, K, V of one (batch, head) as float32 arrays [N, d] (before dtype rounding)."""
    N, d = wl.N, wl.d
    if wl.recipe == "iid":
        q = _rng(wl, 0, b, h).standard_normal((N, d), dtype=np.float32)
        k = _rng(wl, 1, b, h).standard_normal((N, d), dtype=np.float32)
        v = _rng(wl, 2, b, h).standard_normal((N, d), dtype=np.float32)
        return q, k, v
    g = _rng(wl, 3, b, h)
    freq = g.standard_normal((3, d)) * SIGMA_F
    phi = g.uniform(0.0, 2.0 * math.pi, size=d)
    bvec = g.standard_normal(d)
    t, y, x = _grid(wl)
    phase = (t[:, None] / wl.Nf) * freq[0][None, :]
    phase += (y[:, None] / wl.Hg) * freq[1][None, :]
    phase += (x[:, None] / wl.Wg) * freq[2][None, :]
    phase *= 2.0 * math.pi
    phase += phi[None, :]
    field = np.cos(phase, out=phase)
    field *= math.sqrt(2.0)
    if wl.recipe == "blob":
        sig = wl.Hg / 6.0
        x0, y0 = 0.15 * wl.Wg, 0.2 * wl.Hg
        vx = 0.7 * wl.Wg / max(1, wl.Nf - 1)
        vy = 0.6 * wl.Hg / max(1, wl.Nf - 1)
        bump = BLOB_AMP * np.exp(-((y - y0 - vy * t) ** 2 + (x - x0 - vx * t) ** 2) / (2.0 * sig * sig))
        field += bump[:, None] * bvec[None, :]
    f32 = field.astype(np.float32)
    q = f32 + NOISE * _rng(wl, 0, b, h).standard_normal((N, d), dtype=np.float32)
    k = f32 + NOISE * _rng(wl, 1, b, h).standard_normal((N, d), dtype=np.float32)
    v = _rng(wl, 2, b, h).standard_normal((N, d), dtype=np.float32)
    return q, k, v


def round_to_dtype(x: np.ndarray, dtype: str):
    """Round a float32 array once to the run dtype; returns a torch CPU tensor."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        return t.to(torch.bfloat16)
    if dtype == "f32":
        return t
    raise ValueError(dtype)


def make_qkv(wl: Workload, heads=None, device: str = "cpu"):
    """Q, K, V as torch tensors [B, len(heads), N, d] in the run dtype.

    ``heads`` selects a subset (default: all); head ``h`` is generated from its
    own stream, so subsets agree bit-for-bit with a full generation.
    """
    import torch
    heads = list(range(wl.H)) if heads is None else list(heads)
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    out = [torch.empty((wl.B, len(heads), wl.N, wl.d), dtype=tdt, device=device) for _ in range(3)]
    for b in range(wl.B):
        for i, h in enumerate(heads):
            for dst, src in zip(out, make_head(wl, b, h)):
                dst[b, i].copy_(round_to_dtype(src, wl.dtype))
    return out


def make_ar1_proxy(Nf: int, Nt: int, D: int, delta: float, seed: int) -> np.ndarray:
    """Hidden states of the drift proxy: h[t] = sqrt(1 - delta^2) h[t-1] + delta eps[t], eps ~ N(0, I), per token
    position, h[0] ~ N(0, I).  Returns float32 [Nf * Nt, D], frame-major like the video token order.
    (Input synthesis only: the three motion regimes of the proxy task use delta = 0.02, 0.15, 0.40.)"""
    g = np.random.Generator(np.random.Philox(np.random.SeedSequence([BASE_SEED, 7, seed])))
    h = np.empty((Nf, Nt, D), dtype=np.float64)
    h[0] = g.standard_normal((Nt, D))
    keep = math.sqrt(1.0 - delta * delta)
    for t in range(1, Nf):
        h[t] = keep * h[t - 1] + delta * g.standard_normal((Nt, D))
    return h.reshape(Nf * Nt, D).astype(np.float32)
