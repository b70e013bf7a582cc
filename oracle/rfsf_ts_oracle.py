"""ctypes loader for the fp64 CPU oracle in rfsf_ts_oracle.c.

Test infrastructure only: imported by tests/, the smoke check and the
CPU-baseline leg of the benchmark. The product path never imports this.
The C file states what is computed and cites the paper passage for each step;
this file only builds it with gcc, marshals numpy arrays and checks shapes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rfsf_ts_oracle.c")
_LIB = os.path.join(_HERE, "librfsf_ts_oracle.so")
_lib = None


def lib_path() -> str:
    return _LIB


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over sequences, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build(force=True)
        lib = ctypes.CDLL(_LIB)
        i64, i32, dbl = ctypes.c_int64, ctypes.c_int, ctypes.c_double
        vp = ctypes.c_void_p
        lib.rfsf_ts_oracle_threads.restype = ctypes.c_int
        lib.rfsf_ts_oracle_features.restype = ctypes.c_int
        lib.rfsf_ts_oracle_features.argtypes = [i64, i64, i32, i32, i32, i32, vp, vp, vp, vp, dbl, vp, i64]
        lib.rfsf_ts_oracle_increments.restype = ctypes.c_int
        lib.rfsf_ts_oracle_increments.argtypes = [i64, i64, i32, i32, i32, vp, vp, dbl, vp]
        lib.rfsf_ts_oracle_gram.restype = ctypes.c_int
        lib.rfsf_ts_oracle_gram.argtypes = [vp, i64, i64, vp, i64, i64, i64, vp, i64]
        lib.rfsf_dp1d_oracle_features.restype = ctypes.c_int
        lib.rfsf_dp1d_oracle_features.argtypes = [i64, i64, i32, i32, i32, vp, vp, vp, dbl, vp, i64]
        lib.rfsf_trp_oracle_features.restype = ctypes.c_int
        lib.rfsf_trp_oracle_features.argtypes = [i64, i64, i32, i32, i32, i32, vp, vp, vp, dbl, vp, i64]
        lib.rfsf_ts_oracle_features_order.restype = ctypes.c_int
        lib.rfsf_ts_oracle_features_order.argtypes = [i64, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp, dbl, vp, i64]
        lib.rfsf_ts_oracle_normalize.restype = ctypes.c_int
        lib.rfsf_ts_oracle_normalize.argtypes = [vp, i64, i64, i32, i32]
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().rfsf_ts_oracle_threads())


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _check_inputs(X, W, hash_, sign):
    X, W, sign = _f32(X), _f32(W), _f32(sign)
    hash_ = np.ascontiguousarray(hash_, dtype=np.int32)
    if X.ndim != 3 or W.ndim != 3 or hash_.ndim != 2 or sign.shape != hash_.shape:
        raise ValueError("expected X[N,L,d], W[M,d,F], hash[M,2F], sign[M,2F]")
    N, L, d = X.shape
    M, d2, F = W.shape
    if d2 != d or hash_.shape != (M, 2 * F):
        raise ValueError("inconsistent shapes")
    return X, W, hash_, sign, N, L, d, M, F


def features(X, W, hash_, sign, lengthscale: float, D: int, order: int = 1) -> np.ndarray:
    """float64 [N, 1 + M*D]: column 0 is level 0 (= 1), then M blocks of D. order = signature order p."""
    X, W, hash_, sign, N, L, d, M, F = _check_inputs(X, W, hash_, sign)
    out = np.empty((N, 1 + M * D), dtype=np.float64)
    if order != 1:
        rc = _load().rfsf_ts_oracle_features_order(N, L, d, M, F, int(D), int(order), X.ctypes.data, W.ctypes.data,
                                                   hash_.ctypes.data, sign.ctypes.data, float(lengthscale),
                                                   out.ctypes.data, out.shape[1])
        if rc != 0:
            raise RuntimeError(f"rfsf_ts_oracle_features_order failed with code {rc}")
        return out
    rc = _load().rfsf_ts_oracle_features(N, L, d, M, F, int(D), X.ctypes.data, W.ctypes.data,
                                         hash_.ctypes.data, sign.ctypes.data, float(lengthscale),
                                         out.ctypes.data, out.shape[1])
    if rc != 0:
        raise RuntimeError(f"rfsf_ts_oracle_features failed with code {rc}")
    return out


def features_ragged(X, lengths, W, hash_, sign, lengthscale: float, D: int, order: int = 1) -> np.ndarray:
    """Variable-length batch (appendix, ksig.preprocessing: sequences of different lengths): X[N, L, d] padded,
    lengths[n] in [1, L] points of sequence n exist. Row n is the feature map of X[n, :lengths[n]] alone: the
    routine above is called once per distinct length on the sequences of that length, truncated."""
    X = _f32(X)
    lengths = np.asarray(lengths, dtype=np.int64)
    if X.ndim != 3 or lengths.shape != (X.shape[0],) or np.any(lengths < 1) or np.any(lengths > X.shape[1]):
        raise ValueError("expected X[N,L,d] and lengths[N] in [1, L]")
    M = np.asarray(W).shape[0]
    out = np.empty((X.shape[0], 1 + M * int(D)), dtype=np.float64)
    for ell in np.unique(lengths):
        idx = np.nonzero(lengths == ell)[0]
        out[idx] = features(X[idx, :int(ell)], W, hash_, sign, lengthscale, D, order)
    return out


def increments(X, W, lengthscale: float) -> np.ndarray:
    """float64 [N, T, M, 2F]: time increments of the per-level random Fourier features."""
    X, W = _f32(X), _f32(W)
    N, L, d = X.shape
    M, d2, F = W.shape
    if d2 != d:
        raise ValueError("inconsistent shapes")
    out = np.empty((N, L - 1, M, 2 * F), dtype=np.float64)
    rc = _load().rfsf_ts_oracle_increments(N, L, d, M, F, X.ctypes.data, W.ctypes.data,
                                           float(lengthscale), out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"rfsf_ts_oracle_increments failed with code {rc}")
    return out


def gram(PhiX, PhiY=None) -> np.ndarray:
    """float64 [Nx, Ny] = PhiX PhiY^T by three explicit loops."""
    PhiX = np.ascontiguousarray(PhiX, dtype=np.float64)
    PhiY = PhiX if PhiY is None else np.ascontiguousarray(PhiY, dtype=np.float64)
    if PhiX.ndim != 2 or PhiY.ndim != 2 or PhiX.shape[1] != PhiY.shape[1]:
        raise ValueError("expected PhiX[Nx,C], PhiY[Ny,C]")
    K = np.empty((PhiX.shape[0], PhiY.shape[0]), dtype=np.float64)
    rc = _load().rfsf_ts_oracle_gram(PhiX.ctypes.data, PhiX.shape[0], PhiX.shape[1],
                                     PhiY.ctypes.data, PhiY.shape[0], PhiY.shape[1],
                                     PhiX.shape[1], K.ctypes.data, K.shape[1])
    if rc != 0:
        raise RuntimeError(f"rfsf_ts_oracle_gram failed with code {rc}")
    return K


def normalize(Phi, M: int, D: int) -> np.ndarray:
    """Level-wise normalised copy of feature rows [N, 1 + M*D] (float64)."""
    out = np.array(Phi, dtype=np.float64, order="C", copy=True)
    if out.ndim != 2 or out.shape[1] != 1 + M * D:
        raise ValueError("expected Phi[N, 1 + M*D]")
    rc = _load().rfsf_ts_oracle_normalize(out.ctypes.data, out.shape[0], out.shape[1], int(M), int(D))
    if rc != 0:
        raise RuntimeError(f"rfsf_ts_oracle_normalize failed with code {rc}")
    return out


def dp1d_features(X, W, bias, lengthscale: float) -> np.ndarray:
    """RFSF-DP-1D features, float64 [N, 1 + M*F]: X[N,L,d], W[M,d,F], bias[M,F]."""
    X, W, bias = _f32(X), _f32(W), _f32(bias)
    if X.ndim != 3 or W.ndim != 3 or bias.ndim != 2:
        raise ValueError("expected X[N,L,d], W[M,d,F], bias[M,F]")
    N, L, d = X.shape
    M, d2, F = W.shape
    if d2 != d or bias.shape != (M, F):
        raise ValueError("inconsistent shapes")
    out = np.empty((N, 1 + M * F), dtype=np.float64)
    rc = _load().rfsf_dp1d_oracle_features(N, L, d, M, F, X.ctypes.data, W.ctypes.data, bias.ctypes.data,
                                           float(lengthscale), out.ctypes.data, out.shape[1])
    if rc != 0:
        raise RuntimeError(f"rfsf_dp1d_oracle_features failed with code {rc}")
    return out


def trp_features(X, W, Z, lengthscale: float) -> np.ndarray:
    """RFSF-TRP features, float64 [N, 1 + M*Q]: X[N,L,d], W[M,d,F], Z[M,Q,2F]."""
    X, W, Z = _f32(X), _f32(W), _f32(Z)
    if X.ndim != 3 or W.ndim != 3 or Z.ndim != 3:
        raise ValueError("expected X[N,L,d], W[M,d,F], Z[M,Q,2F]")
    N, L, d = X.shape
    M, d2, F = W.shape
    if d2 != d or Z.shape[0] != M or Z.shape[2] != 2 * F:
        raise ValueError("inconsistent shapes")
    Q = Z.shape[1]
    out = np.empty((N, 1 + M * Q), dtype=np.float64)
    rc = _load().rfsf_trp_oracle_features(N, L, d, M, F, Q, X.ctypes.data, W.ctypes.data, Z.ctypes.data,
                                          float(lengthscale), out.ctypes.data, out.shape[1])
    if rc != 0:
        raise RuntimeError(f"rfsf_trp_oracle_features failed with code {rc}")
    return out


def features_order(X, W, hash_, sign, lengthscale: float, D: int, order: int) -> np.ndarray:
    """The order-p routine itself (also for order = 1, where it must agree with `features`)."""
    X, W, hash_, sign, N, L, d, M, F = _check_inputs(X, W, hash_, sign)
    out = np.empty((N, 1 + M * D), dtype=np.float64)
    rc = _load().rfsf_ts_oracle_features_order(N, L, d, M, F, int(D), int(order), X.ctypes.data, W.ctypes.data,
                                               hash_.ctypes.data, sign.ctypes.data, float(lengthscale),
                                               out.ctypes.data, out.shape[1])
    if rc != 0:
        raise RuntimeError(f"rfsf_ts_oracle_features_order failed with code {rc}")
    return out
