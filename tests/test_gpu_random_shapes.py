"""Seeded random shapes through the C ABI against the oracle: bucket counts of every kind (powers of two, the
exact lengths 100 .. 1000, linear-convolution lengths up to 8192), one to eight levels, orders 1-3, few to many
random features, batches of different lengths. Whatever kernel the library picks for a shape, the result must
be the oracle's; the only refusal allowed is order 3 where the shape leaves the tuned kernels."""
import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import binding
from tests.parity import FP32_BLOCK_TOL, block_errors

pytestmark = pytest.mark.gpu

BUCKETS = [64, 100, 128, 200, 256, 300, 500, 512, 600, 1000, 1024, 1500, 2048, 3000, 4096]


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_shapes(oracle, seed):
    rng = np.random.default_rng(seed)
    refused = 0
    for _ in range(40):
        D = int(rng.choice(BUCKETS))
        M = int(rng.integers(1, 9))
        order = int(rng.integers(1, 4))
        big = D >= 1500
        if big:
            M = min(M, 3)                                   # keeps the oracle's O(D^2) convolutions short
        exact = (D & (D - 1)) == 0 or D in (100, 200, 500, 1000)
        if not exact and M * (D - 1) + 1 > 8192:
            M = max(1, 8192 // D)
        L = int(rng.integers(2, 9 if big else 24))
        N = int(rng.integers(1, 4))
        d = int(rng.integers(1, 6))
        F = int(rng.integers(1, min(2 * D, 2500) + 1))
        X = np.cumsum(rng.standard_normal((N, L, d)) * 0.3, axis=1).astype(np.float32)
        W = rng.standard_normal((M, d, F)).astype(np.float32)
        hash_ = rng.integers(0, D, size=(M, 2 * F)).astype(np.int32)
        sign = (2.0 * rng.integers(0, 2, size=(M, 2 * F)) - 1.0).astype(np.float32)
        lengths = rng.integers(1, L + 1, size=N)
        case = (N, L, d, M, F, D, order)
        try:
            got = rfsf.rfsf_ts_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(),
                                        torch.from_numpy(hash_).cuda(), torch.from_numpy(sign).cuda(), 1.5, D,
                                        order=order, lengths=torch.from_numpy(lengths).cuda()).cpu().numpy()
        except binding.RfsfTsError as e:
            assert e.code == -9 and order == 3, case
            refused += 1
            continue
        want = oracle.features_ragged(X, lengths, W, hash_, sign, 1.5, D, order=order)
        err = block_errors(got, want, M, D)
        assert np.all(err <= FP32_BLOCK_TOL), (case, err)
    assert refused <= 6


@pytest.mark.parametrize("seed", [21])
def test_random_shapes_of_few_long_sequences(oracle, seed):
    """The same for shapes that the library cuts in time (at most 64 sequences, long enough for M + 1 pieces of
    32 pairs of steps): every kernel family, orders 1-3, batches of different lengths."""
    rng = np.random.default_rng(seed)
    cut = 0
    for _ in range(12):
        D = int(rng.choice([64, 100, 128, 200, 256, 300, 500, 512, 1000, 1024, 2048]))
        M = int(rng.integers(2, 9))
        order = int(rng.integers(1, 4))
        big = D >= 500
        if big:
            M = min(M, 4)                                   # keeps the oracle's O(D^2) convolutions short
        exact = (D & (D - 1)) == 0 or D in (100, 200, 500, 1000)
        if not exact and M * (D - 1) + 1 > 8192:
            M = max(2, 8192 // D)
        L = int(rng.integers(64 * (M + 1), 64 * (M + 1) + (150 if big else 1200)))
        N = int(rng.integers(1, 4))
        d = int(rng.integers(1, 6))
        F = int(rng.integers(1, min(2 * D, 700) + 1))
        X = np.cumsum(rng.standard_normal((N, L, d)) * 0.1, axis=1).astype(np.float32)
        W = rng.standard_normal((M, d, F)).astype(np.float32)
        hash_ = rng.integers(0, D, size=(M, 2 * F)).astype(np.int32)
        sign = (2.0 * rng.integers(0, 2, size=(M, 2 * F)) - 1.0).astype(np.float32)
        lengths = np.where(rng.random(N) < 0.5, L, rng.integers(1, L + 1, size=N)).astype(np.int64)
        case = (N, L, d, M, F, D, order)
        try:
            got = rfsf.rfsf_ts_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(),
                                        torch.from_numpy(hash_).cuda(), torch.from_numpy(sign).cuda(), 1.5, D,
                                        order=order, lengths=torch.from_numpy(lengths).cuda()).cpu().numpy()
        except binding.RfsfTsError as e:
            assert e.code == -9 and order == 3, case
            continue
        cut += rfsf.rfsf_ts_time_cut(N, L, d, M, F, D, order=order)[0] > 1
        want = oracle.features_ragged(X, lengths, W, hash_, sign, 1.5, D, order=order)
        err = block_errors(got, want, M, D)
        assert np.all(err <= FP32_BLOCK_TOL), (case, err)
    assert cut >= 8
