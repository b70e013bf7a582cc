"""bf16-operand variant of the random-Fourier projection (fp32 accumulate): stated separately
from the fp32 path. Two numbers per case: against the oracle on the original fp32 inputs
(tolerance 2e-2 per block) and against the oracle fed exactly the operands the kernel
multiplies -- W rounded to bf16, X replaced by the sum of its two bf16 terms -- which isolates
the kernel's own error (tolerance 1e-4)."""
import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import binding, workloads as wl
from tests.parity import BF16_BLOCK_TOL, FP32_BLOCK_TOL, block_errors

pytestmark = pytest.mark.gpu


def _case(seed, N, L, d, M, F, D, ls):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) / np.sqrt(L), axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    hash_ = rng.integers(0, D, size=(M, 2 * F)).astype(np.int32)
    sign = (2.0 * rng.integers(0, 2, size=(M, 2 * F)) - 1.0).astype(np.float32)
    return X, W, hash_, sign, float(np.float32(ls))


def _operands_as_multiplied(X, W):
    hi = wl.round_to_bf16(X)
    lo = wl.round_to_bf16(X - hi)
    return (hi + lo).astype(np.float32), wl.round_to_bf16(W)


@pytest.mark.parametrize("N,L,d,M,F,D", [(6, 64, 64, 3, 96, 128), (4, 40, 5, 2, 32, 64), (3, 33, 100, 2, 40, 64),
                                          (5, 70, 20, 4, 64, 256)])
def test_bf16_projection(oracle, N, L, d, M, F, D):
    X, W, hash_, sign, ls = _case(N + d, N, L, d, M, F, D, ls=np.sqrt(d))
    got = rfsf.rfsf_ts_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(),
                                torch.from_numpy(hash_).cuda(), torch.from_numpy(sign).cuda(), ls, D,
                                rff_bf16=True)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    err_orig = block_errors(got, oracle.features(X, W, hash_, sign, ls, D), M, D)
    Xm, Wm = _operands_as_multiplied(X, W)
    err_same = block_errors(got, oracle.features(Xm, Wm, hash_, sign, ls, D), M, D)
    print(f"d={d}: vs fp32-input oracle {err_orig}, vs same-operand oracle {err_same}")
    assert np.all(err_orig <= BF16_BLOCK_TOL)
    assert np.all(err_same <= FP32_BLOCK_TOL)
    assert np.any(err_orig > 10 * err_same.max())      # the bf16 rounding of W is really there


def test_bf16_rejects_wide_state():
    X = torch.zeros(2, 4, 200, device="cuda")
    W = torch.zeros(2, 200, 8, device="cuda")
    h = torch.zeros(2, 16, dtype=torch.int32, device="cuda")
    s = torch.ones(2, 16, device="cuda")
    with pytest.raises(binding.RfsfTsError) as e:
        rfsf.rfsf_ts_features(X, W, h, s, 1.0, 16, rff_bf16=True)
    assert e.value.code == -9
