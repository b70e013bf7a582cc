"""Level-wise normalisation on the GPU against the oracle's, and the properties it must have."""
import math

import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import binding, workloads as wl
from tests.parity import FP32_BLOCK_TOL, GRAM_TOL, block_errors, gram_error

pytestmark = pytest.mark.gpu


def _features(inp, D):
    t = {k: torch.from_numpy(v).cuda() for k, v in inp.items() if isinstance(v, np.ndarray)}
    return rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], D)


@pytest.mark.parametrize("name,N", [("tiny", 16), ("small", 64)])
def test_normalised_features_match_oracle(oracle, name, N):
    w = wl.WORKLOADS[name].scaled(N=N)
    inp = wl.make_inputs(w, 0)
    Phi = _features(inp, w.D)
    rfsf.rfsf_ts_normalize_features(Phi, w.M, w.D)
    torch.cuda.synchronize()
    want = oracle.normalize(oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], w.D),
                            w.M, w.D)
    err = block_errors(Phi.cpu().numpy(), want, w.M, w.D, level0=1.0 / math.sqrt(w.M + 1))
    assert np.all(err <= FP32_BLOCK_TOL), err
    K = rfsf.rfsf_ts_gram(Phi)
    torch.cuda.synchronize()
    assert gram_error(K.cpu().numpy(), oracle.gram(want)) <= GRAM_TOL
    assert torch.allclose(torch.diagonal(K), torch.ones(N, device="cuda"), atol=1e-5)


def test_zero_levels_padding_and_odd_sizes(oracle):
    """Two increments and four levels (levels 3, 4 vanish), D not a power of two, padded rows."""
    rng = np.random.default_rng(3)
    M, D, N = 4, 12, 5
    P = rng.standard_normal((N, 1 + M * D)).astype(np.float32)
    P[:, 0] = 1.0
    P[:, 1 + 2 * D:] = 0.0
    buf = torch.full((N, 1 + M * D + 6), -2.0, dtype=torch.float32, device="cuda")
    buf[:, :1 + M * D] = torch.from_numpy(P).cuda()
    rfsf.rfsf_ts_normalize_features(buf, M, D)
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    want = oracle.normalize(P.astype(np.float64), M, D)
    assert np.all(got[:, 1 + M * D:] == -2.0)
    assert np.all(got[:, 1 + 2 * D:1 + M * D] == 0.0)
    np.testing.assert_allclose(got[:, :1 + M * D], want, rtol=2e-6, atol=1e-7)
    with pytest.raises(binding.RfsfTsError):
        binding._check(binding.load_library().rfsf_ts_normalize_features(buf.data_ptr(), N, 10, M, D, None))
