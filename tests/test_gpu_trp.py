"""RFSF-TRP on the GPU against the oracle, block-normalised error per level."""
import math

import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import binding
from tests.parity import FP32_BLOCK_TOL, block_errors

pytestmark = pytest.mark.gpu


def _case(seed, N, L, d, M, F, Q, ls):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) / math.sqrt(L), axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    Z = rng.standard_normal((M, Q, 2 * F)).astype(np.float32)
    return X, W, Z, float(np.float32(ls))


def _run(X, W, Z, ls, **kw):
    out = rfsf.rfsf_trp_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), torch.from_numpy(Z).cuda(),
                                 ls, **kw)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("N,L,d,M,F,Q", [
    (16, 32, 3, 3, 32, 64),       # tiny-like
    (24, 100, 8, 4, 128, 256),    # small-like
    (5, 37, 5, 3, 24, 50),        # Q not a power of two, ragged everything
    (3, 9, 4, 2, 7, 33),          # odd F: 2F not a multiple of 4, plain GEMM path
    (2, 2, 3, 4, 16, 16),         # one increment
    (2, 1, 3, 2, 8, 8),           # no increments
    (1, 300, 2, 6, 16, 300),      # long, six levels, two component blocks
    (3, 30, 3, 1, 8, 12),         # one level; 29 increments in batches of eight
    (2, 23, 4, 5, 16, 1024),      # five levels, a whole 4 KB row of the projections per sequence
    (2, 18, 3, 7, 8, 36),         # seven levels: batches of three, sequences sharing a workgroup
    (2, 11, 3, 9, 8, 20),         # more than eight levels: the 16-level kernel, one step per batch
    (2, 14, 3, 12, 8, 18),        # the same with components that are no multiple of four
    (300, 5, 2, 2, 4, 8),         # many short sequences: 150 per workgroup
])
def test_trp_matches_oracle(oracle, N, L, d, M, F, Q):
    X, W, Z, ls = _case(N + L + Q, N, L, d, M, F, Q, ls=math.sqrt(d))
    got = _run(X, W, Z, ls).cpu().numpy()
    want = oracle.trp_features(X, W, Z, ls)
    err = block_errors(got, want, M, Q)
    print(f"N={N} L={L} d={d} M={M} F={F} Q={Q} block errors {err}")
    assert np.all(err <= FP32_BLOCK_TOL)


def test_trp_chunks_padding_and_errors(oracle):
    X, W, Z, ls = _case(3, 7, 12, 3, 2, 16, 20, 1.0)
    _, mn = rfsf.rfsf_trp_workspace_bytes(7, 12, 3, 2, 16, 20)
    rec2, _ = rfsf.rfsf_trp_workspace_bytes(2, 12, 3, 2, 16, 20)
    ws = torch.empty(mn + 2 * (rec2 - mn), dtype=torch.uint8, device="cuda")     # three sequences per chunk
    buf = torch.full((7, 41 + 3), -5.0, dtype=torch.float32, device="cuda")
    _run(X, W, Z, ls, out=buf, workspace=ws)
    assert torch.all(buf[:, 41:] == -5.0)
    assert np.all(block_errors(buf[:, :41].cpu().numpy(), oracle.trp_features(X, W, Z, ls), 2, 20) <= FP32_BLOCK_TOL)
    with pytest.raises(binding.RfsfTsError) as e:
        _run(X, W, Z, ls, workspace=torch.empty(mn - 1, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -6


def test_trp_more_sequences_than_one_launch_may_take(oracle):
    # 70000 sequences: the scan kernel puts sequences on grid.y (at most 65535), so the call must split
    # the batch even though the workspace would hold it whole
    N, L, d, M, F, Q = 70000, 3, 2, 2, 2, 4
    X, W, Z, ls = _case(11, N, L, d, M, F, Q, 1.0)
    got = _run(X, W, Z, ls).cpu().numpy()
    sel = np.r_[0:40, 34990:35010, 65530:65540, N - 40:N]
    want = oracle.trp_features(X[sel], W, Z, ls)
    assert np.all(block_errors(got[sel], want, M, Q) <= FP32_BLOCK_TOL)
    assert np.all(got[:, 0] == 1.0) and np.all(np.isfinite(got))
