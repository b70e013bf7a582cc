"""Error measures shared by the GPU parity tests, smoke check and benchmark report."""
from __future__ import annotations

import numpy as np

FP32_BLOCK_TOL = 1e-4      # max relative error per feature block, fp32 path
BF16_BLOCK_TOL = 2e-2      # the same for the bf16-input projection, against the fp32-input oracle
GRAM_TOL = 1e-4            # max |K_gpu - K_oracle| / max |K_oracle|


def block_errors(got: np.ndarray, want: np.ndarray, M: int, D: int, level0: float = 1.0) -> np.ndarray:
    """err[m] = max over sequences of |got_block - want_block|_inf / |want_block|_inf, where a
    block is one level of one sequence (D numbers). Blocks that are exactly zero in the oracle
    (levels above the number of increments) must be exactly zero in `got` (error inf otherwise).
    Column 0 (level 0) must be exactly 1 (or within 1e-6 of `level0` for normalised rows)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape == (want.shape[0], 1 + M * D), (got.shape, want.shape)
    if want.shape[0] == 0:
        return np.zeros(M)
    if level0 == 1.0:
        assert np.all(got[:, 0] == 1.0), "level-0 column must be exactly 1"
    else:
        assert np.all(np.abs(got[:, 0] - level0) <= 1e-6 * abs(level0)), "level-0 column is off"
    g = got[:, 1:].reshape(-1, M, D)
    w = want[:, 1:].reshape(-1, M, D)
    num = np.abs(g - w).max(axis=2)
    den = np.abs(w).max(axis=2)
    err = np.where(den > 0, num / np.where(den > 0, den, 1.0), np.where(num > 0, np.inf, 0.0))
    return err.max(axis=0)


def gram_error(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    return float(np.abs(got - want).max() / np.abs(want).max())
