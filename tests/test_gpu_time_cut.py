"""Few long sequences: the library cuts them in time, runs the recurrence on the pieces and joins them
(rfsf_ts_time_cut). The result must be the feature map of the whole sequence: checked against the oracle,
which knows nothing of pieces, block-normalised as everywhere else."""
import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from tests.parity import FP32_BLOCK_TOL, block_errors

pytestmark = pytest.mark.gpu


def _case(seed, N, L, d, M, F, D, ls=1.5, step=0.2):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) * step, axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    hash_ = rng.integers(0, D, size=(M, 2 * F)).astype(np.int32)
    sign = (2.0 * rng.integers(0, 2, size=(M, 2 * F)) - 1.0).astype(np.float32)
    return X, W, hash_, sign, float(np.float32(ls))


def _gpu(X, W, hash_, sign, ls, D, **kw):
    out = rfsf.rfsf_ts_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), torch.from_numpy(hash_).cuda(),
                                torch.from_numpy(sign).cuda(), ls, D, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("N,L,d,M,F,D", [
    (3, 1000, 5, 5, 50, 100),      # the paper's own shape (Sec. 4): exact transform of 100 points, 15 pieces
    (2, 401, 3, 2, 16, 64),        # two levels, an even number of steps, the last piece shorter
    (2, 400, 3, 3, 16, 64),        # an odd number of steps: the last pair of the last piece has one step
    (1, 2600, 2, 8, 8, 128),       # eight levels on one sequence
    (5, 700, 4, 4, 128, 256),      # four transforms per wavefront
    (2, 900, 6, 5, 96, 1024),      # items dealt to eight wavefronts, more buckets than coordinates
    (3, 500, 3, 3, 40, 300),       # buckets that are no power of two: linear route in 1024 points, folded per piece
    (2, 300, 3, 3, 24, 1500),      # the 8192-point kernel
    (2, 330, 5, 4, 512, 2048),     # 2048 points in one wavefront
])
def test_cut_sequences_match_the_oracle(oracle, N, L, d, M, F, D):
    pieces, pairs = rfsf.rfsf_ts_time_cut(N, L, d, M, F, D)
    assert pieces > M and pieces * pairs >= L // 2 and (pieces - 1) * pairs < L // 2 and pairs >= 32
    X, W, hash_, sign, ls = _case(N + L + D, N, L, d, M, F, D)
    got = _gpu(X, W, hash_, sign, ls, D)
    want = oracle.features(X, W, hash_, sign, ls, D)
    err = block_errors(got, want, M, D)
    print(f"N={N} L={L} M={M} F={F} D={D}: {pieces} pieces of {pairs} pairs, block errors {err}")
    assert np.all(err <= FP32_BLOCK_TOL)


def test_cut_sequences_of_different_lengths(oracle):
    """Sequences that end inside a piece, exactly at a piece's end, before the second piece, and with no step at all."""
    N, L, d, M, F, D = 6, 800, 3, 4, 32, 128
    pieces, pairs = rfsf.rfsf_ts_time_cut(N, L, d, M, F, D)
    assert pieces > M
    X, W, hash_, sign, ls = _case(77, N, L, d, M, F, D)
    lengths = np.array([L, 2 * pairs + 1, 2 * pairs + 2, 7, 1, 2 * pairs * (pieces - 1) + 1], dtype=np.int64)
    got = _gpu(X, W, hash_, sign, ls, D, lengths=torch.from_numpy(lengths).cuda())
    want = oracle.features_ragged(X, lengths, W, hash_, sign, ls, D)
    err = block_errors(got, want, M, D)
    print("block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
    assert np.array_equal(got[4], np.concatenate([[1.0], np.zeros(M * D)]).astype(np.float32))


@pytest.mark.parametrize("order,N,L,d,M,F,D", [
    (2, 2, 600, 3, 3, 16, 64),
    (2, 3, 500, 5, 5, 50, 100),
    (3, 2, 700, 3, 4, 24, 128),
    (3, 1, 451, 4, 5, 96, 1024),
])
def test_cut_sequences_of_higher_signature_order(oracle, order, N, L, d, M, F, D):
    """A time step used up to `order` times in a row never spans two pieces, so the pieces join the same way."""
    assert rfsf.rfsf_ts_time_cut(N, L, d, M, F, D, order=order)[0] > M
    X, W, hash_, sign, ls = _case(5 + order + L, N, L, d, M, F, D)
    got = _gpu(X, W, hash_, sign, ls, D, order=order)
    want = oracle.features_order(X, W, hash_, sign, ls, D, order)
    err = block_errors(got, want, M, D)
    print(f"order {order} N={N} L={L} M={M} D={D}: block errors {err}")
    assert np.all(err <= FP32_BLOCK_TOL)


def test_cut_sequences_through_the_smallest_workspace(oracle):
    """One sequence per launch series: the plan does not depend on the workspace, the result does not either."""
    N, L, d, M, F, D = 3, 700, 3, 3, 20, 64
    assert rfsf.rfsf_ts_time_cut(N, L, d, M, F, D)[0] > M
    X, W, hash_, sign, ls = _case(11, N, L, d, M, F, D)
    rec, mn = rfsf.rfsf_ts_workspace_bytes(N, L, d, M, F, D)
    assert mn < rec
    small = _gpu(X, W, hash_, sign, ls, D, workspace=torch.empty(mn, dtype=torch.uint8, device="cuda"))
    full = _gpu(X, W, hash_, sign, ls, D, workspace=torch.empty(rec, dtype=torch.uint8, device="cuda"))
    assert np.array_equal(small, full)
    want = oracle.features(X, W, hash_, sign, ls, D)
    assert np.all(block_errors(small, want, M, D) <= FP32_BLOCK_TOL)
