"""ctypes binding with the same names as the C entry points (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libdynamicrad.so"

MODE_STATIC, MODE_DYNAMIC, MODE_ZSCORE, MODE_UNIFORM = 0, 1, 2, 3
CLASS_NONE, CLASS_NEAR, CLASS_FAR, CLASS_FORCED = 0, 1, 2, 3
_STATUS = {0: "DR_OK", 1: "DR_ERR_INVALID_ARG", 2: "DR_ERR_UNSUPPORTED", 3: "DR_ERR_CAPACITY", 4: "DR_ERR_HIP",
           5: "DR_ERR_NOMEM"}


class DRError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{_STATUS.get(status, status)}: {text}")
        self.status = status
        self.status_name = _STATUS.get(status, str(status))


class Shape(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("N", C.c_int32), ("d", C.c_int32),
                ("Nf", C.c_int32), ("Hg", C.c_int32), ("Wg", C.c_int32), ("Bs", C.c_int32),
                ("dtype", C.c_int32), ("reserved0", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_n", C.c_int64)]

    @property
    def Sb(self) -> int:
        return -(-self.N // self.Bs)


class MaskParams(C.Structure):
    _fields_ = [("gamma", C.c_double), ("theta_c", C.c_double), ("theta_m", C.c_double),
                ("ratio_far", C.c_double), ("head_fuse", C.c_int32), ("has_tau_far", C.c_int32),
                ("tau_far", C.c_double), ("seed", C.c_uint32), ("reserved", C.c_int32 * 3)]

    def __init__(self, gamma=1.0, theta_c=0.15, theta_m=0.60, ratio_far=-1.0, head_fuse=2, tau_far=None, seed=0):
        super().__init__(gamma, theta_c, theta_m, ratio_far, head_fuse, 0 if tau_far is None else 1,
                         0.0 if tau_far is None else tau_far, seed)


def lib_path() -> str:
    return os.path.join(HERE, _LIB_NAME)


_lib = None


def load_library():
    """Load the built library; raises with the build command if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or `python paper_2604_20470_amd/build.py`) first; there is no CPU fallback")
    lib = C.CDLL(path)
    vp, i32, i64, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_double
    shp, mpp = C.POINTER(Shape), C.POINTER(MaskParams)
    lib.dr_version.restype = C.c_char_p
    lib.dr_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.dr_destroy.argtypes = [vp]
    lib.dr_destroy.restype = None
    lib.dr_last_error.argtypes = [vp]
    lib.dr_last_error.restype = C.c_char_p
    lib.dr_class_map.argtypes = [vp, shp, f64, mpp, vp, vp]
    lib.dr_mask_capacity.argtypes = [vp, shp, f64, mpp, C.POINTER(i64), C.POINTER(i32)]
    lib.dr_static_ratio_for_sparsity.argtypes = [vp, shp, f64, mpp, f64, C.POINTER(f64), C.POINTER(f64)]
    lib.dr_block_scores.argtypes = [vp, shp, vp, vp, i32, vp, vp]
    lib.dr_build_mask.argtypes = [vp, shp, i32, f64, f64, mpp, vp, vp, vp, i64, vp, vp]
    lib.dr_sparse_attn_fwd.argtypes = [vp, shp, vp, vp, vp, vp, vp, i32, i64, vp, vp, vp]
    lib.dr_sparse_attn_fwd_static.argtypes = [vp, shp, vp, vp, vp, vp, vp, i32, i64, vp, vp, vp]
    lib.dr_token_scores.argtypes = [vp, shp, vp, vp, i32, vp, vp]
    lib.dr_build_mask_tokens.argtypes = [vp, shp, f64, f64, mpp, vp, vp, vp, i64, vp, vp, vp]
    lib.dr_proxy_loss.argtypes = [vp, vp, vp, i32, i32, i32, vp, i32, i32, f64, f64, vp, vp]
    lib.dr_clock_probe.argtypes = [vp, C.c_uint64, vp, vp]
    lib.dr_mfma_probe.argtypes = [vp, i32, i32, i32, i32, vp, C.POINTER(f64), vp]
    lib.dr_mfma_mix_probe.argtypes = [vp, i32, i32, vp, C.POINTER(f64), vp]
    for name in ("dr_token_scores", "dr_build_mask_tokens", "dr_proxy_loss", "dr_static_ratio_for_sparsity", "dr_clock_probe", "dr_mfma_probe", "dr_mfma_mix_probe", "dr_create", "dr_class_map", "dr_mask_capacity", "dr_block_scores", "dr_build_mask",
                 "dr_sparse_attn_fwd", "dr_sparse_attn_fwd_static"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def version() -> str:
    return load_library().dr_version().decode()


class Context:
    """Owns a dr_ctx (scratch + cached candidate geometry) on one device."""

    def __init__(self, device: int = 0):
        self._lib = load_library()
        self._h = C.c_void_p()
        st = self._lib.dr_create(C.byref(self._h), int(device))
        if st != 0:
            raise DRError(st, f"dr_create(device={device}) failed")
        self.device = device

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            self._lib.dr_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, st: int):
        if st != 0:
            raise DRError(st, self._lib.dr_last_error(self._h).decode())


def shape_of(t, Nf: int, Hg: int, Wg: int, Bs: int) -> Shape:
    """Shape descriptor of a [B, H, N, d] torch tensor (Q; K, V, O must share its strides)."""
    import torch
    assert t.dim() == 4 and t.stride(3) == 1, "expected [B, H, N, d] with contiguous d"
    dt = {torch.float32: 0, torch.bfloat16: 1}[t.dtype]
    B, H, N, d = t.shape
    return Shape(B, H, N, d, Nf, Hg, Wg, Bs, dt, 0, t.stride(0), t.stride(1), t.stride(2))


def _ptr(t) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


def _pp(params: Optional[MaskParams]):
    return C.byref(params) if params is not None else None


def dr_class_map(ctx: Context, shape: Shape, lam: float, params: Optional[MaskParams], class_map, stream=None):
    ctx.check(ctx._lib.dr_class_map(ctx._h, C.byref(shape), float(lam), _pp(params), _ptr(class_map), _stream(stream)))


def dr_mask_capacity(ctx: Context, shape: Shape, lam: float, params: Optional[MaskParams] = None) -> Tuple[int, int]:
    cand, msel = C.c_int64(0), C.c_int32(0)
    ctx.check(ctx._lib.dr_mask_capacity(ctx._h, C.byref(shape), float(lam), _pp(params), C.byref(cand), C.byref(msel)))
    return cand.value, msel.value


def dr_static_ratio_for_sparsity(ctx: Context, shape: Shape, lam: float, params: Optional[MaskParams],
                                 target: float) -> Tuple[float, float]:
    """(rho, achieved effective sparsity): the largest static ratio on a 1e-3 grid whose mask reaches `target`."""
    rho, got = C.c_double(0.0), C.c_double(0.0)
    ctx.check(ctx._lib.dr_static_ratio_for_sparsity(ctx._h, C.byref(shape), float(lam), _pp(params), float(target),
                                                    C.byref(rho), C.byref(got)))
    return rho.value, got.value


def dr_block_scores(ctx: Context, shape: Shape, Q, K, head_fuse: int, scores, stream=None):
    ctx.check(ctx._lib.dr_block_scores(ctx._h, C.byref(shape), _ptr(Q), _ptr(K), int(head_fuse), _ptr(scores),
                                       _stream(stream)))


def dr_build_mask(ctx: Context, shape: Shape, mode: int, ratio_or_tau: float, lam: float,
                  params: Optional[MaskParams], scores, rowptr, colidx, colidx_capacity: int, nnz, stream=None):
    ctx.check(ctx._lib.dr_build_mask(ctx._h, C.byref(shape), int(mode), float(ratio_or_tau), float(lam), _pp(params),
                                     _ptr(scores), _ptr(rowptr), _ptr(colidx), int(colidx_capacity), _ptr(nnz),
                                     _stream(stream)))


def dr_sparse_attn_fwd(ctx: Context, shape: Shape, Q, K, V, rowptr, colidx, mask_heads: int, colidx_stride: int,
                       O, lse=None, stream=None):
    ctx.check(ctx._lib.dr_sparse_attn_fwd(ctx._h, C.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(rowptr),
                                          _ptr(colidx), int(mask_heads), int(colidx_stride), _ptr(O), _ptr(lse),
                                          _stream(stream)))


def dr_sparse_attn_fwd_static(ctx: Context, shape: Shape, Q, K, V, rowptr, colidx, mask_heads: int, colidx_stride: int,
                              O, lse=None, stream=None):
    ctx.check(ctx._lib.dr_sparse_attn_fwd_static(ctx._h, C.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(rowptr),
                                                 _ptr(colidx), int(mask_heads), int(colidx_stride), _ptr(O), _ptr(lse),
                                                 _stream(stream)))


def dr_token_scores(ctx: Context, shape: Shape, Q, K, head_fuse: int, scores, stream=None):
    ctx.check(ctx._lib.dr_token_scores(ctx._h, C.byref(shape), _ptr(Q), _ptr(K), int(head_fuse), _ptr(scores),
                                       _stream(stream)))


def dr_build_mask_tokens(ctx: Context, shape: Shape, tau_near: float, lam: float, params: Optional[MaskParams],
                         token_scores, rowptr, colidx, colidx_capacity: int, nnz, links=None, stream=None):
    ctx.check(ctx._lib.dr_build_mask_tokens(ctx._h, C.byref(shape), float(tau_near), float(lam), _pp(params),
                                            _ptr(token_scores), _ptr(rowptr), _ptr(colidx), int(colidx_capacity),
                                            _ptr(nnz), _ptr(links), _stream(stream)))


def dr_proxy_loss(ctx: Context, A_dense, A_sparse, nnz, Sb: int, target: float, alpha: float, out, stream=None):
    """Enqueue the proxy objective: A_dense, A_sparse float32 [B, H, N, N]; nnz int64 [B, masks]; out float64 [3]."""
    B, H, N, _ = A_dense.shape
    ctx.check(ctx._lib.dr_proxy_loss(ctx._h, _ptr(A_dense), _ptr(A_sparse), int(B), int(H), int(N), _ptr(nnz),
                                     int(nnz.shape[1]), int(Sb), float(target), float(alpha), _ptr(out), _stream(stream)))


def dr_clock_probe(ctx: Context, window_us: int, out, stream=None):
    """Enqueue the clock probe: `out` is a device int64 tensor of two entries (shader ticks, 100 MHz ticks)."""
    ctx.check(ctx._lib.dr_clock_probe(ctx._h, int(window_us), _ptr(out), _stream(stream)))


def dr_mfma_probe(ctx: Context, shape: int, workgroups: int, iters: int, random_operands: bool, sink,
                  stream=None) -> float:
    """Enqueue the MFMA-only loop (shape 32: 32x32x16, 16: 16x16x32); returns the flop count of the launch."""
    flop = C.c_double(0.0)
    ctx.check(ctx._lib.dr_mfma_probe(ctx._h, int(shape), int(workgroups), int(iters), 1 if random_operands else 0,
                                     _ptr(sink), C.byref(flop), _stream(stream)))
    return flop.value


def dr_mfma_mix_probe(ctx: Context, workgroups: int, iters: int, sink, stream=None) -> float:
    """Enqueue the loop of one 32x32x16 matrix instruction + one exponential + two fp32 instructions per slot."""
    flop = C.c_double(0.0)
    ctx.check(ctx._lib.dr_mfma_mix_probe(ctx._h, int(workgroups), int(iters), _ptr(sink), C.byref(flop), _stream(stream)))
    return flop.value
