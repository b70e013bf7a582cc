"""RFSF-DP-1D on the GPU against the oracle, block-normalised error per level as for RFSF-TS."""
import math

import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import binding
from tests.parity import FP32_BLOCK_TOL, block_errors

pytestmark = pytest.mark.gpu


def _case(seed, N, L, d, M, F, ls):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) / math.sqrt(L), axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    b = rng.uniform(0.0, 2.0 * math.pi, size=(M, F)).astype(np.float32)
    return X, W, b, float(np.float32(ls))


@pytest.mark.parametrize("N,L,d,M,F", [
    (16, 32, 3, 3, 32),        # tiny-like
    (40, 100, 8, 4, 128),      # small-like
    (5, 37, 5, 3, 70),         # ragged components and rows
    (3, 65, 17, 5, 300),       # two component slabs, odd d
    (2, 1, 4, 2, 16),          # no increments
    (2, 2, 64, 6, 40),         # one increment, widest state
    (1, 1000, 2, 8, 9),        # long and narrow
    (2, 40, 64, 8, 70),        # widest state with eight levels: more than 64 KB of LDS per workgroup
    (2, 33, 3, 16, 20),        # the largest supported number of levels
    (1, 20, 40, 13, 300),      # 13 levels on a wide state, two component slabs
    (2, 50, 10, 3, 100),       # d well below the kernel's 32 projection rows: eleven pairs of rows read as zero
    (2, 70, 33, 2, 130),       # odd d just above 32: the last pair of rows is half empty, three tiles
    (3, 96, 12, 4, 64),        # whole tiles only, exactly one wavefront of components
])
def test_dp1d_matches_oracle(oracle, N, L, d, M, F):
    X, W, b, ls = _case(N + L + F, N, L, d, M, F, ls=math.sqrt(d))
    got = rfsf.rfsf_dp1d_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(),
                                  torch.from_numpy(b).cuda(), ls)
    torch.cuda.synchronize()
    want = oracle.dp1d_features(X, W, b, ls)
    err = block_errors(got.cpu().numpy(), want, M, F)
    print(f"N={N} L={L} d={d} M={M} F={F} block errors {err}")
    assert np.all(err <= FP32_BLOCK_TOL)


def test_dp1d_limits_and_padding(oracle):
    X, W, b, ls = _case(9, 3, 10, 3, 2, 20, 1.0)
    buf = torch.full((3, 1 + 2 * 20 + 5), -4.0, dtype=torch.float32, device="cuda")
    rfsf.rfsf_dp1d_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), torch.from_numpy(b).cuda(),
                            ls, out=buf)
    torch.cuda.synchronize()
    assert torch.all(buf[:, 41:] == -4.0)
    assert np.all(block_errors(buf[:, :41].cpu().numpy(), oracle.dp1d_features(X, W, b, ls), 2, 20) <= FP32_BLOCK_TOL)
    with pytest.raises(binding.RfsfTsError) as e:
        rfsf.rfsf_dp1d_features(torch.zeros(1, 4, 70, device="cuda"), torch.zeros(2, 70, 8, device="cuda"),
                                torch.zeros(2, 8, device="cuda"), 1.0)
    assert e.value.code == -9
