"""Thin ctypes binding of librfsf_ts (argument marshalling only).

Every step of the hot path runs in the HIP kernels behind the C ABI declared in
include/rfsf_ts.h. PyTorch is used here for device memory and streams, nothing
else. There is no CPU fallback: if the library is missing or fails to load, the
calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librfsf_ts.so")
_lib = None


class RfsfTsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"librfsf_ts error {code}: {text}")
        self.code = code


class _Shape(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("L", ctypes.c_int64),
                ("d", ctypes.c_int32), ("M", ctypes.c_int32), ("F", ctypes.c_int32), ("D", ctypes.c_int32),
                ("ld_out", ctypes.c_int64), ("rff_bf16", ctypes.c_int32), ("order", ctypes.c_int32)]


class _Profile(ctypes.Structure):
    _fields_ = [("ms_rff_increments", ctypes.c_double), ("launches_rff_increments", ctypes.c_int64),
                ("ms_sketch_fft_scan", ctypes.c_double), ("launches_sketch_fft_scan", ctypes.c_int64),
                ("ms_gram", ctypes.c_double), ("launches_gram", ctypes.c_int64),
                ("ms_normalize", ctypes.c_double), ("launches_normalize", ctypes.c_int64),
                ("ms_dp1d", ctypes.c_double), ("launches_dp1d", ctypes.c_int64),
                ("ms_trp_project", ctypes.c_double), ("launches_trp_project", ctypes.c_int64),
                ("ms_trp_scan", ctypes.c_double), ("launches_trp_scan", ctypes.c_int64)]


class _Peaks(ctypes.Structure):
    _fields_ = [("read_gbs", ctypes.c_double), ("write_gbs", ctypes.c_double), ("write_nt_gbs", ctypes.c_double),
                ("copy_gbs", ctypes.c_double), ("mfma_f32_tflops", ctypes.c_double), ("valu_f32_tflops", ctypes.c_double)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load librfsf_ts.so; build it first only if it has never been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build_library
        build_library()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.rfsf_ts_strerror.restype = ctypes.c_char_p
    lib.rfsf_ts_strerror.argtypes = [ctypes.c_int]
    lib.rfsf_ts_time_cut.restype = ctypes.c_int
    lib.rfsf_ts_time_cut.argtypes = [ctypes.POINTER(_Shape), ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)]
    lib.rfsf_ts_workspace_bytes.restype = ctypes.c_int
    lib.rfsf_ts_workspace_bytes.argtypes = [ctypes.POINTER(_Shape), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.rfsf_ts_features.restype = ctypes.c_int
    lib.rfsf_ts_features.argtypes = [ctypes.POINTER(_Shape), vp, vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.rfsf_ts_features_ragged.restype = ctypes.c_int
    lib.rfsf_ts_features_ragged.argtypes = [ctypes.POINTER(_Shape), vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.rfsf_ts_features_static.restype = ctypes.c_int
    lib.rfsf_ts_features_static.argtypes = [ctypes.POINTER(_Shape), vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.rfsf_ts_validate_tables.restype = ctypes.c_int
    lib.rfsf_ts_validate_tables.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.rfsf_ts_gram.restype = ctypes.c_int
    lib.rfsf_ts_gram.argtypes = [vp, i64, i64, vp, i64, i64, i64, vp, i64, vp]
    lib.rfsf_ts_normalize_features.restype = ctypes.c_int
    lib.rfsf_ts_normalize_features.argtypes = [vp, i64, i64, i32, i32, vp]
    lib.rfsf_dp1d_features.restype = ctypes.c_int
    lib.rfsf_dp1d_features.argtypes = [i64, i64, i32, i32, i32, vp, vp, vp, ctypes.c_float, vp, i64, vp]
    lib.rfsf_trp_workspace_bytes.restype = ctypes.c_int
    lib.rfsf_trp_workspace_bytes.argtypes = [ctypes.POINTER(_Shape), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.rfsf_trp_features.restype = ctypes.c_int
    lib.rfsf_trp_features.argtypes = [ctypes.POINTER(_Shape), vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.rfsf_ts_profile_enable.restype = ctypes.c_int
    lib.rfsf_ts_profile_enable.argtypes = [ctypes.c_int]
    lib.rfsf_ts_probe_peaks.restype = ctypes.c_int
    lib.rfsf_ts_probe_peaks.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(_Peaks), ctypes.c_void_p]
    lib.rfsf_ts_profile_read.restype = ctypes.c_int
    lib.rfsf_ts_profile_read.argtypes = [ctypes.POINTER(_Profile), ctypes.c_int]
    _lib = lib
    return lib


def _check(code: int):
    if code != 0:
        raise RfsfTsError(code, load_library().rfsf_ts_strerror(code).decode())


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _empty_on(stream: Optional[torch.cuda.Stream], *args, **kwargs) -> torch.Tensor:
    """torch.empty whose block belongs to `stream` for the caching allocator: memory the binding allocates is
    used by kernels on that stream, possibly after this function has returned and dropped its reference."""
    if stream is None:
        return torch.empty(*args, **kwargs)
    with torch.cuda.stream(stream):
        return torch.empty(*args, **kwargs)


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous {dtype}")
    return t


def _shape_of(X, W, hash_, D, ld_out, rff_bf16, order=1) -> _Shape:
    if X.dim() != 3 or W.dim() != 3 or hash_.dim() != 2:
        raise ValueError("expected X[N,L,d], W[M,d,F], hash[M,2F]")
    N, L, d = X.shape
    M, d2, F = W.shape
    if d2 != d or tuple(hash_.shape) != (M, 2 * F):
        raise ValueError("inconsistent shapes")
    return _Shape(N, L, d, M, F, int(D), int(ld_out), int(bool(rff_bf16)), int(order))


def rfsf_ts_workspace_bytes(N: int, L: int, d: int, M: int, F: int, D: int, rff_bf16: bool = False, order: int = 1):
    """(recommended_bytes, minimum_bytes) of scratch for rfsf_ts_features."""
    shp = _Shape(N, L, d, M, F, D, 1 + M * D, int(bool(rff_bf16)), int(order))
    rec, mn = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().rfsf_ts_workspace_bytes(ctypes.byref(shp), ctypes.byref(rec), ctypes.byref(mn)))
    return int(rec.value), int(mn.value)


def rfsf_ts_time_cut(N: int, L: int, d: int, M: int, F: int, D: int, order: int = 1):
    """(pieces, pairs_per_piece): how rfsf_ts_features cuts the sequences of this shape in time
    (pieces = 1: not at all)."""
    shp = _Shape(N, L, d, M, F, D, 1 + M * D, 0, int(order))
    pieces, pairs = ctypes.c_int32(0), ctypes.c_int64(0)
    _check(load_library().rfsf_ts_time_cut(ctypes.byref(shp), ctypes.byref(pieces), ctypes.byref(pairs)))
    return int(pieces.value), int(pairs.value)


def feature_row_stride(M: int, D: int) -> int:
    """Row stride (floats) the binding gives to feature matrices it allocates: 1 + M*D
    rounded up to a multiple of 4 so that rows stay 16-byte aligned for the Gram."""
    return (1 + M * D + 3) // 4 * 4


def rfsf_ts_features(X: torch.Tensor, W: torch.Tensor, hash: torch.Tensor, sign: torch.Tensor,
                     lengthscale: float, D: int, out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, rff_bf16: bool = False,
                     stream: Optional[torch.cuda.Stream] = None, order: int = 1,
                     lengths: Optional[torch.Tensor] = None) -> torch.Tensor:
    """RFSF-TS features of a batch: returns a [N, 1 + M*D] float32 view (row stride
    feature_row_stride(M, D) when allocated here). `out` may be any 2-D float32 device
    tensor with unit column stride and at least 1 + M*D columns; `workspace` any
    contiguous uint8 device tensor of at least the minimum size. `lengths` (int64 [N] on the
    device) gives each sequence's own number of points when X is a padded variable-length batch."""
    lib = load_library()
    X = _dev(X, torch.float32, "X")
    W = _dev(W, torch.float32, "W")
    hash = _dev(hash, torch.int32, "hash")
    sign = _dev(sign, torch.float32, "sign")
    N, M = X.shape[0], W.shape[0]
    ncols = 1 + M * int(D)
    if out is None:
        ld = feature_row_stride(M, int(D))
        out = _empty_on(stream, (N, ld), dtype=torch.float32, device=X.device)[:, :ncols]
    if out.dim() != 2 or out.dtype != torch.float32 or not out.is_cuda or out.shape[0] != N or \
            out.shape[1] < ncols or (out.shape[1] > 0 and out.stride(1) != 1):
        raise ValueError("out must be float32 [N, >= 1+M*D] on the device with unit column stride")
    ld_out = out.stride(0) if N > 1 else max(out.stride(0), out.shape[1])
    shp = _shape_of(X, W, hash, D, ld_out, rff_bf16, order)
    if workspace is None:
        rec, _ = rfsf_ts_workspace_bytes(shp.N, shp.L, shp.d, shp.M, shp.F, shp.D, rff_bf16, order)
        workspace = _empty_on(stream, rec, dtype=torch.uint8, device=X.device)
    workspace = _dev(workspace, torch.uint8, "workspace")
    if lengths is not None:
        lengths = _dev(lengths, torch.int64, "lengths")
        if tuple(lengths.shape) != (N,):
            raise ValueError("lengths must have shape [N]")
        _check(lib.rfsf_ts_features_ragged(ctypes.byref(shp), X.data_ptr(), lengths.data_ptr(), W.data_ptr(),
                                           hash.data_ptr(), sign.data_ptr(), float(lengthscale), out.data_ptr(),
                                           workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
        return out[:, :ncols]
    _check(lib.rfsf_ts_features(ctypes.byref(shp), X.data_ptr(), W.data_ptr(), hash.data_ptr(),
                                sign.data_ptr(), float(lengthscale), out.data_ptr(),
                                workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out[:, :ncols]


def rfsf_ts_features_static(X: torch.Tensor, W: torch.Tensor, hash: torch.Tensor, sign: torch.Tensor,
                            lengthscale: float, D: int, out: torch.Tensor, rff_bf16: bool = False,
                            stream: Optional[torch.cuda.Stream] = None, order: int = 1) -> torch.Tensor:
    """rfsf_ts_features through the entry point that allocates nothing: the caller passes `out`, the
    library uses its built-in 64 MiB scratch. Nothing is allocated here either."""
    lib = load_library()
    X = _dev(X, torch.float32, "X")
    W = _dev(W, torch.float32, "W")
    hash = _dev(hash, torch.int32, "hash")
    sign = _dev(sign, torch.float32, "sign")
    N, M = X.shape[0], W.shape[0]
    ncols = 1 + M * int(D)
    if out.dim() != 2 or out.dtype != torch.float32 or not out.is_cuda or out.shape[0] != N or \
            out.shape[1] < ncols or (out.shape[1] > 0 and out.stride(1) != 1):
        raise ValueError("out must be float32 [N, >= 1+M*D] on the device with unit column stride")
    ld_out = out.stride(0) if N > 1 else max(out.stride(0), out.shape[1])
    shp = _shape_of(X, W, hash, D, ld_out, rff_bf16, order)
    _check(lib.rfsf_ts_features_static(ctypes.byref(shp), X.data_ptr(), W.data_ptr(), hash.data_ptr(),
                                       sign.data_ptr(), float(lengthscale), out.data_ptr(), _stream_ptr(stream)))
    return out[:, :ncols]


def rfsf_ts_normalize_features(Phi: torch.Tensor, M: int, D: int,
                               stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Level-wise normalisation of feature rows [N, >= 1 + M*D], in place; returns Phi."""
    if Phi.dim() != 2 or Phi.dtype != torch.float32 or not Phi.is_cuda or Phi.shape[1] < 1 + M * D or \
            (Phi.shape[1] > 0 and Phi.stride(1) != 1):
        raise ValueError("Phi must be float32 [N, >= 1+M*D] on the device with unit column stride")
    N = Phi.shape[0]
    ld = Phi.stride(0) if N > 1 else max(Phi.stride(0), Phi.shape[1])
    _check(load_library().rfsf_ts_normalize_features(Phi.data_ptr(), N, ld, int(M), int(D), _stream_ptr(stream)))
    return Phi


def rfsf_dp1d_features(X: torch.Tensor, W: torch.Tensor, bias: torch.Tensor, lengthscale: float,
                       out: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """RFSF-DP-1D features [N, 1 + M*F] of X[N,L,d] with W[M,d,F], bias[M,F]."""
    X = _dev(X, torch.float32, "X")
    W = _dev(W, torch.float32, "W")
    bias = _dev(bias, torch.float32, "bias")
    if X.dim() != 3 or W.dim() != 3 or bias.dim() != 2 or W.shape[1] != X.shape[2] or \
            tuple(bias.shape) != (W.shape[0], W.shape[2]):
        raise ValueError("expected X[N,L,d], W[M,d,F], bias[M,F]")
    N, L, d = X.shape
    M, _, F = W.shape
    ncols = 1 + M * F
    if out is None:
        out = _empty_on(stream, (N, (ncols + 3) // 4 * 4), dtype=torch.float32, device=X.device)[:, :ncols]
    if out.dim() != 2 or out.dtype != torch.float32 or not out.is_cuda or out.shape[0] != N or \
            out.shape[1] < ncols or (out.shape[1] > 0 and out.stride(1) != 1):
        raise ValueError("out must be float32 [N, >= 1+M*F] on the device with unit column stride")
    ld_out = out.stride(0) if N > 1 else max(out.stride(0), out.shape[1])
    _check(load_library().rfsf_dp1d_features(N, L, d, M, F, X.data_ptr(), W.data_ptr(), bias.data_ptr(),
                                             float(lengthscale), out.data_ptr(), ld_out, _stream_ptr(stream)))
    return out[:, :ncols]


def rfsf_trp_workspace_bytes(N: int, L: int, d: int, M: int, F: int, Q: int, rff_bf16: bool = False):
    """(recommended_bytes, minimum_bytes) of scratch for rfsf_trp_features."""
    shp = _Shape(N, L, d, M, F, Q, 1 + M * Q, int(bool(rff_bf16)))
    rec, mn = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().rfsf_trp_workspace_bytes(ctypes.byref(shp), ctypes.byref(rec), ctypes.byref(mn)))
    return int(rec.value), int(mn.value)


def rfsf_trp_features(X: torch.Tensor, W: torch.Tensor, Z: torch.Tensor, lengthscale: float,
                      out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                      rff_bf16: bool = False, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """RFSF-TRP features [N, 1 + M*Q] of X[N,L,d] with W[M,d,F] and Gaussian projections Z[M,Q,2F]."""
    X = _dev(X, torch.float32, "X")
    W = _dev(W, torch.float32, "W")
    Z = _dev(Z, torch.float32, "Z")
    if X.dim() != 3 or W.dim() != 3 or Z.dim() != 3 or W.shape[1] != X.shape[2] or Z.shape[0] != W.shape[0] or \
            Z.shape[2] != 2 * W.shape[2]:
        raise ValueError("expected X[N,L,d], W[M,d,F], Z[M,Q,2F]")
    N, L, d = X.shape
    M, _, F = W.shape
    Q = Z.shape[1]
    ncols = 1 + M * Q
    if out is None:
        out = _empty_on(stream, (N, (ncols + 3) // 4 * 4), dtype=torch.float32, device=X.device)[:, :ncols]
    if out.dim() != 2 or out.dtype != torch.float32 or not out.is_cuda or out.shape[0] != N or \
            out.shape[1] < ncols or (out.shape[1] > 0 and out.stride(1) != 1):
        raise ValueError("out must be float32 [N, >= 1+M*Q] on the device with unit column stride")
    ld_out = out.stride(0) if N > 1 else max(out.stride(0), out.shape[1])
    shp = _Shape(N, L, d, M, F, Q, ld_out, int(bool(rff_bf16)))
    if workspace is None:
        rec, _ = rfsf_trp_workspace_bytes(N, L, d, M, F, Q, rff_bf16)
        workspace = _empty_on(stream, rec, dtype=torch.uint8, device=X.device)
    workspace = _dev(workspace, torch.uint8, "workspace")
    _check(load_library().rfsf_trp_features(ctypes.byref(shp), X.data_ptr(), W.data_ptr(), Z.data_ptr(),
                                            float(lengthscale), out.data_ptr(), workspace.data_ptr(),
                                            workspace.numel(), _stream_ptr(stream)))
    return out[:, :ncols]


def rfsf_ts_validate_tables(hash: torch.Tensor, sign: torch.Tensor, D: int,
                            stream: Optional[torch.cuda.Stream] = None) -> None:
    """Raises RfsfTsError(RFSF_E_BAD_TABLE) unless hash is in [0, D) and sign in {+1, -1}."""
    hash = _dev(hash, torch.int32, "hash")
    sign = _dev(sign, torch.float32, "sign")
    M, twoF = hash.shape
    _check(load_library().rfsf_ts_validate_tables(hash.data_ptr(), sign.data_ptr(), M, twoF // 2, int(D),
                                                  _stream_ptr(stream)))


def rfsf_ts_gram(PhiX: torch.Tensor, PhiY: Optional[torch.Tensor] = None,
                 K: Optional[torch.Tensor] = None,
                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """K = PhiX PhiY^T (PhiY defaults to PhiX). Inputs are 2-D float32 device tensors with unit
    column stride (row strides are passed as leading dimensions)."""
    lib = load_library()
    PhiY = PhiX if PhiY is None else PhiY
    for name, t in (("PhiX", PhiX), ("PhiY", PhiY)):
        if t.dim() != 2 or t.dtype != torch.float32 or not t.is_cuda or (t.shape[1] > 0 and t.stride(1) != 1):
            raise ValueError(f"{name} must be float32 [rows, cols] on the device with unit column stride")
    if PhiX.shape[1] != PhiY.shape[1]:
        raise ValueError("PhiX and PhiY need the same number of columns")
    Nx, Ny, ncols = PhiX.shape[0], PhiY.shape[0], PhiX.shape[1]
    if K is None:
        K = _empty_on(stream, (Nx, Ny), dtype=torch.float32, device=PhiX.device)
    if K.dim() != 2 or K.dtype != torch.float32 or tuple(K.shape) != (Nx, Ny) or (Ny > 0 and K.stride(1) != 1):
        raise ValueError("K must be float32 [Nx, Ny] with unit column stride")
    ldx = PhiX.stride(0) if Nx > 1 else max(ncols, 1)
    ldy = PhiY.stride(0) if Ny > 1 else max(ncols, 1)
    ldk = K.stride(0) if Nx > 1 else max(Ny, 1)
    _check(lib.rfsf_ts_gram(PhiX.data_ptr(), Nx, ldx, PhiY.data_ptr(), Ny, ldy, ncols,
                            K.data_ptr(), ldk, _stream_ptr(stream)))
    return K


def rfsf_ts_profile_enable(on: bool) -> None:
    _check(load_library().rfsf_ts_profile_enable(int(bool(on))))


def rfsf_ts_probe_peaks(scratch: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> dict:
    """What the GPU gives plain streaming kernels (GB/s) and fp32 issue loops (TFLOP/s); `scratch` is any
    contiguous device tensor, its contents are destroyed."""
    if not scratch.is_cuda or not scratch.is_contiguous():
        raise ValueError("scratch must be a contiguous device tensor")
    p = _Peaks()
    _check(load_library().rfsf_ts_probe_peaks(ctypes.c_void_p(scratch.data_ptr()), scratch.numel() * scratch.element_size(),
                                              ctypes.byref(p), ctypes.c_void_p(_stream_ptr(stream))))
    return {f: getattr(p, f) for f, _ in _Peaks._fields_}


def rfsf_ts_profile_read(reset: bool = True) -> dict:
    """Per-kernel-class device time (ms) and launch counts recorded since the last reset."""
    p = _Profile()
    _check(load_library().rfsf_ts_profile_read(ctypes.byref(p), int(bool(reset))))
    return {f: getattr(p, f) for f, _ in _Profile._fields_}
