"""CPU pins of the oracle's RFSF-DP-1D variant (Sec. 3.3): brute force over the definition, closed
forms, invariants, and unbiasedness for the truncated signature kernel."""
import itertools
import math

import numpy as np
import pytest

from tests import pins


def _case(seed, N, L, d, M, F, ls=1.2):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) * 0.4, axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    b = rng.uniform(0.0, 2.0 * math.pi, size=(M, F)).astype(np.float32)
    return X, W, b, float(np.float32(ls))


def _phi(X, W, b, ls):
    """sqrt(2) cos(x.W/l + b), fp64, [N, L, M, F] (eq. (rff_1d) with the size-1 scale)."""
    th = np.einsum("nlc,mcf->nlmf", X.astype(np.float64), W.astype(np.float64)) / ls + b.astype(np.float64)
    return math.sqrt(2.0) * np.cos(th)


@pytest.mark.parametrize("T,M,F", [(6, 3, 3), (4, 4, 2), (5, 2, 5), (2, 3, 2)])
def test_bruteforce_tuples(oracle, T, M, F):
    """Sec. 3.2 eq. (rfsf) with p = 1 applied to each size-1 copy, then eq. (dp1d)."""
    X, W, b, ls = _case(T + M + F, N=2, L=T + 1, d=2, M=M, F=F)
    got = oracle.dp1d_features(X, W, b, ls)
    u = np.diff(_phi(X, W, b, ls), axis=1)                       # [N, T, M, F]
    want = np.zeros((2, M, F))
    for m in range(1, M + 1):
        for idx in itertools.combinations(range(T), m):
            prod = np.ones((2, F))
            for k in range(m):
                prod *= u[:, idx[k], k, :]
            want[:, m - 1, :] += prod
    assert np.all(got[:, 0] == 1.0)
    np.testing.assert_allclose(got[:, 1:].reshape(2, M, F), want / math.sqrt(F), rtol=0, atol=1e-13)


def test_closed_forms(oracle):
    """Level 1 telescopes to F^{-1/2} (phi(x_last) - phi(x_first)); a bias of pi/2 turns the cosine into
    minus a sine; one non-zero frequency entry pins the [M, d, F] indexing and the lengthscale."""
    X, W, b, ls = _case(3, N=3, L=9, d=3, M=2, F=4)
    got = oracle.dp1d_features(X, W, b, ls)
    phi = _phi(X, W, b, ls)
    np.testing.assert_allclose(got[:, 1:5], (phi[:, -1, 0] - phi[:, 0, 0]) / 2.0, rtol=0, atol=1e-14)
    W1 = np.zeros_like(W)
    W1[0, 2, 1] = 0.5
    b1 = np.full_like(b, math.pi / 2)
    g1 = oracle.dp1d_features(X, W1, b1, 2.0)
    th = X[:, :, 2].astype(np.float64) * 0.5 / 2.0
    want = np.zeros((3, 4))
    want[:, 1] = -math.sqrt(2.0) * (np.sin(th[:, -1]) - np.sin(th[:, 0])) / 2.0
    np.testing.assert_allclose(g1[:, 1:5], want, rtol=0, atol=1e-8)    # float32(pi/2) is 4e-8 off pi/2
    assert np.all(np.abs(g1[:, 5:]) < 1e-15)                      # level 2: constant features, no increments


def test_short_sequences_and_repeated_points(oracle):
    X, W, b, ls = _case(4, N=2, L=3, d=2, M=3, F=3)
    one = oracle.dp1d_features(X[:, :1], W, b, ls)
    assert np.all(one[:, 0] == 1.0) and np.all(one[:, 1:] == 0.0)
    two = oracle.dp1d_features(X[:, :2], W, b, ls)
    assert np.any(two[:, 1:4] != 0.0) and np.all(two[:, 4:] == 0.0)
    Xr = np.concatenate([X[:, :2], X[:, 1:2], X[:, 2:]], axis=1)
    np.testing.assert_allclose(oracle.dp1d_features(Xr, W, b, ls), oracle.dp1d_features(X, W, b, ls),
                               rtol=0, atol=1e-14)


def test_unbiased_for_truncated_signature_kernel(oracle):
    """E <Phi_m(x), Phi_m(y)> = k_m(x, y) level by level (Sec. 3.1: both random Fourier maps are unbiased;
    Sec. 3.3). Tolerance 4 standard errors over S independent draws of (W, bias)."""
    L, d, F, M, ls = 7, 2, 32, 3, 1.0
    rng = np.random.default_rng(5)
    X = np.cumsum(rng.standard_normal((2, L, d)) * 0.6, axis=1).astype(np.float32)
    S = 3000
    prods = np.zeros((S, 3, M))
    for s in range(S):
        r = np.random.default_rng([6, s])
        W = r.standard_normal((M, d, F)).astype(np.float32)
        b = r.uniform(0.0, 2.0 * math.pi, size=(M, F)).astype(np.float32)
        P = oracle.dp1d_features(X, W, b, ls)[:, 1:].reshape(2, M, F)
        prods[s, 0] = np.einsum("mf,mf->m", P[0], P[0])
        prods[s, 1] = np.einsum("mf,mf->m", P[0], P[1])
        prods[s, 2] = np.einsum("mf,mf->m", P[1], P[1])
    Xd = X.astype(np.float64)
    exact = np.stack([pins.truncated_sigkernel_levels(Xd[0], Xd[0], ls, M),
                      pins.truncated_sigkernel_levels(Xd[0], Xd[1], ls, M),
                      pins.truncated_sigkernel_levels(Xd[1], Xd[1], ls, M)])
    mean = prods.mean(axis=0)
    se = prods.std(axis=0, ddof=1) / math.sqrt(S)
    assert np.all(np.abs(mean - exact) <= 4.0 * se), (mean, exact, se)
    assert np.all(exact[[0, 2], 0] > 10.0 * se[[0, 2], 0])        # level 1 of the diagonal pairs has power
