"""Seeded synthetic inputs for the RFSF-TS hot path.

This module only draws random numbers and integrates them into paths. It holds
none of the method's arithmetic (no Fourier features, no sketching, no
recursion) so that the CPU oracle and the HIP path can both be fed from it
without sharing any code of the method itself.

The paper's scalability workload is d-dimensional Brownian motion on [0, 1]
(Sec. 4, "Scalability"); the five workloads below have that shape, with the
sizes of the build's configuration table. Nothing here reads a dataset.

Recipe (all workloads):
  * two independent streams per seed s:
      paths  = numpy Generator(PCG64(SeedSequence([s, 0])))
      tables = numpy Generator(PCG64(SeedSequence([s, 1])))
  * `paths` draws the standard-normal increments sequence by sequence
    (C order over [N, L-1, d]) and then, if the workload has them, the
    per-channel scales; drawing is chunked over N but the stream is the same
    for every chunk size;
  * `tables` draws Z ~ N(0,1) of shape [M, d, F] (passed to the library as W,
    which divides by the lengthscale itself), then hash ~ U{0..D-1} of shape
    [M, 2F], then sign ~ U{-1,+1} of shape [M, 2F];
  * arrays are cast once to float32 / int32; both implementations read those.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload (repo symbols: F frequencies, D buckets,
    L time points per sequence, T = L - 1 increments)."""
    name: str
    N: int
    L: int
    d: int              # state dimension as seen by the library (time channel included)
    M: int
    F: int
    D: int
    lengthscale: float
    kind: str           # "brownian" | "brownian_scaled" | "brownian_time" | "ou"
    rff_bf16: bool = False
    N2: int = 0         # size of the second batch for a cross Gram (0: Gram of the batch with itself)

    @property
    def T(self) -> int:
        return self.L - 1

    @property
    def ncols(self) -> int:
        return 1 + self.M * self.D

    def scaled(self, N: Optional[int] = None, L: Optional[int] = None, N2: Optional[int] = None) -> "Workload":
        """Same workload with fewer sequences / time points (tables are unchanged
        because they come from their own stream)."""
        return dataclasses.replace(
            self,
            N=self.N if N is None else N,
            L=self.L if L is None else L,
            N2=self.N2 if N2 is None else N2,
        )


WORKLOADS = {
    "tiny": Workload("tiny", N=16, L=32, d=3, M=3, F=32, D=64, lengthscale=1.0, kind="brownian"),
    "small": Workload("small", N=1000, L=100, d=8, M=4, F=128, D=256,
                      lengthscale=math.sqrt(8.0), kind="brownian_scaled"),
    "medium": Workload("medium", N=10000, L=200, d=17, M=5, F=512, D=1024,
                       lengthscale=4.0, kind="brownian_time"),
    "long": Workload("long", N=2000, L=2000, d=32, M=4, F=256, D=512,
                     lengthscale=math.sqrt(32.0), kind="ou"),
    "large": Workload("large", N=50000, L=64, d=64, M=5, F=1024, D=2048,
                      lengthscale=8.0, kind="brownian", rff_bf16=True, N2=5000),
    # shaped like the paper's own scalability runs (Sec. 4: 5-dimensional Brownian motion, M = 5, static
    # feature and projection sizes 100, batches of 10-100 sequences of length 100 .. 1e5); its bucket
    # count is no power of two
    "paper": Workload("paper", N=100, L=1000, d=5, M=5, F=50, D=100, lengthscale=math.sqrt(5.0), kind="brownian"),
    # the long end of the paper's sequence-length runs (Sec. 4: N = 10, L increased until memory runs out,
    # 1e5 and more for the primal methods): few long sequences, which the library cuts in time
    "paper_long": Workload("paper_long", N=10, L=100000, d=5, M=5, F=50, D=100, lengthscale=math.sqrt(5.0),
                           kind="brownian"),
}


def _path_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), 0])))


def _table_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), 1])))


def make_paths(w: Workload, seed: int = 0, chunk: int = 2048) -> np.ndarray:
    """X[N, L, d] float32.

    brownian        x_0 = 0, x_t = x_{t-1} + xi_t, xi ~ N(0, 1/L) per channel
    brownian_scaled the same, channel c multiplied by s_c ~ U[0.5, 2]
    brownian_time   d-1 Brownian channels plus a last channel t / L, t = 0..L-1
    ou              Ornstein-Uhlenbeck, theta = sigma = 1, dt = 1/L, x_0 = 0,
                    Euler-Maruyama x_{t+1} = x_t - theta x_t dt + sigma sqrt(dt) xi
    """
    rng = _path_rng(seed)
    N, L, d = w.N, w.L, w.d
    d_rand = d - 1 if w.kind == "brownian_time" else d
    X = np.zeros((N, L, d), dtype=np.float32)
    dt = 1.0 / L
    for n0 in range(0, N, chunk):
        n1 = min(N, n0 + chunk)
        xi = rng.standard_normal((n1 - n0, L - 1, d_rand)) if L > 1 else np.zeros((n1 - n0, 0, d_rand))
        if w.kind == "ou":
            x = np.zeros((n1 - n0, d_rand))
            for t in range(1, L):
                x = x - x * dt + math.sqrt(dt) * xi[:, t - 1, :]
                X[n0:n1, t, :d_rand] = x
        else:
            X[n0:n1, 1:, :d_rand] = np.cumsum(xi * math.sqrt(dt), axis=1)
    if w.kind == "brownian_scaled":
        s = rng.uniform(0.5, 2.0, size=d_rand)
        X *= s.astype(np.float32)[None, None, :]
    if w.kind == "brownian_time":
        X[:, :, d - 1] = (np.arange(L, dtype=np.float64) / L).astype(np.float32)[None, :]
    return X


def make_tables(w: Workload, seed: int = 0):
    """(W[M, d, F] float32 ~ N(0, 1), hash[M, 2F] int32 in [0, D), sign[M, 2F] float32 in {-1, +1})."""
    rng = _table_rng(seed)
    W = rng.standard_normal((w.M, w.d, w.F)).astype(np.float32)
    hash_ = rng.integers(0, w.D, size=(w.M, 2 * w.F), dtype=np.int64).astype(np.int32)
    sign = (2.0 * rng.integers(0, 2, size=(w.M, 2 * w.F)) - 1.0).astype(np.float32)
    return W, hash_, sign


def make_bias(w: Workload, seed: int = 0) -> np.ndarray:
    """bias[M, F] float32 ~ U[0, 2 pi) for the one-dimensional random Fourier features of the DP-1D
    variant; its own stream PCG64(SeedSequence([seed, 2])), so the other tables are unchanged."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), 2])))
    return rng.uniform(0.0, 2.0 * math.pi, size=(w.M, w.F)).astype(np.float32)


def make_projections(w: Workload, seed: int = 0, Q: Optional[int] = None) -> np.ndarray:
    """Z[M, Q, 2F] float32 ~ N(0, 1): Gaussian projection vectors of the TRP variant (Q defaults to the
    workload's D); its own stream PCG64(SeedSequence([seed, 3]))."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), 3])))
    return rng.standard_normal((w.M, w.D if Q is None else Q, 2 * w.F)).astype(np.float32)


def make_inputs(w: Workload, seed: int = 0):
    """dict with X, W, hash, sign, lengthscale for one batch."""
    W, hash_, sign = make_tables(w, seed)
    return {"X": make_paths(w, seed), "W": W, "hash": hash_, "sign": sign,
            "lengthscale": float(np.float32(w.lengthscale))}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round a float32 array to the nearest bfloat16 (ties to even), returned as float32.
    Input preparation for the bf16 projection variant; pure bit manipulation."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return r.view(np.float32).reshape(a.shape)
