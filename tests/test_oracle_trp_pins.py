"""CPU pins of the oracle's RFSF-TRP variant (Sec. 3.4): brute force over the definition, special
projections, invariants, and unbiasedness for the truncated signature kernel."""
import itertools
import math

import numpy as np
import pytest

from tests import pins


def _case(seed, N, L, d, M, F, Q, ls=1.2):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) * 0.4, axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    Z = rng.standard_normal((M, Q, 2 * F)).astype(np.float32)
    return X, W, Z, float(np.float32(ls))


@pytest.mark.parametrize("T,M,F,Q", [(6, 3, 2, 5), (4, 4, 1, 3), (5, 2, 3, 7), (2, 3, 2, 2)])
def test_bruteforce_tuples(oracle, T, M, F, Q):
    """Sec. 3.4 eq. (trp), p = 1: explicit sum over i_1 < ... < i_m of the Hadamard product of the
    projected increments (increments from the independent numpy formula)."""
    X, W, Z, ls = _case(T + M + Q, N=2, L=T + 1, d=2, M=M, F=F, Q=Q)
    got = oracle.trp_features(X, W, Z, ls)
    delta = pins.rff_increments_numpy(X, W, ls)                     # [N, T, M, 2F]
    P = np.einsum("ntma,mqa->ntmq", delta, Z.astype(np.float64))
    want = np.zeros((2, M, Q))
    for m in range(1, M + 1):
        for idx in itertools.combinations(range(T), m):
            prod = np.ones((2, Q))
            for k in range(m):
                prod *= P[:, idx[k], k, :]
            want[:, m - 1, :] += prod
    assert np.all(got[:, 0] == 1.0)
    np.testing.assert_allclose(got[:, 1:].reshape(2, M, Q), want / math.sqrt(Q), rtol=0, atol=1e-12)


def test_selection_matrix_gives_diagonal_products(oracle):
    """With Z_m = rows of the identity (Q = 2F) the projection is the identity, so level m holds
    Q^{-1/2} sum_{i_1<...<i_m} prod_k delta_k[i_k][a] coordinate by coordinate; level 1 telescopes."""
    F, M = 3, 3
    X, W, _, ls = _case(2, N=2, L=8, d=2, M=M, F=F, Q=2 * F)
    Z = np.tile(np.eye(2 * F, dtype=np.float32)[None], (M, 1, 1))
    got = oracle.trp_features(X, W, Z, ls)[:, 1:].reshape(2, M, 2 * F) * math.sqrt(2 * F)
    delta = pins.rff_increments_numpy(X, W, ls)
    e = np.zeros((2, M + 1, 2 * F))
    e[:, 0] = 1.0
    for t in range(delta.shape[1]):
        for m in range(M, 0, -1):
            e[:, m] += e[:, m - 1] * delta[:, t, m - 1]
    np.testing.assert_allclose(got, e[:, 1:], rtol=0, atol=1e-13)
    np.testing.assert_allclose(got[:, 0], delta[:, :, 0].sum(axis=1), rtol=0, atol=1e-13)


def test_short_sequences_and_layout(oracle):
    X, W, Z, ls = _case(4, N=2, L=3, d=2, M=3, F=2, Q=4)
    one = oracle.trp_features(X[:, :1], W, Z, ls)
    assert np.all(one[:, 0] == 1.0) and np.all(one[:, 1:] == 0.0)
    two = oracle.trp_features(X[:, :2], W, Z, ls)
    assert np.any(two[:, 1:5] != 0.0) and np.all(two[:, 5:] == 0.0)
    # one non-zero projection vector: only its component moves (pins the [M, Q, 2F] indexing)
    Z1 = np.zeros_like(Z)
    Z1[0, 2, 1] = 1.0
    g = oracle.trp_features(X, W, Z1, ls)
    assert np.all(g[:, [1, 2, 4]] == 0.0) and np.all(g[:, 3] != 0.0)


def test_unbiased_for_truncated_signature_kernel(oracle):
    """E <Phi_m(x), Phi_m(y)> = k_m(x, y): Gaussian projections preserve inner products in expectation and
    tensorised ones do so for tensor products (Sec. 3.4), on top of the unbiased RFSF of Sec. 3.2."""
    L, d, F, Q, M, ls = 7, 2, 12, 24, 3, 1.0
    rng = np.random.default_rng(8)
    X = np.cumsum(rng.standard_normal((2, L, d)) * 0.6, axis=1).astype(np.float32)
    S = 3000
    prods = np.zeros((S, 3, M))
    for s in range(S):
        r = np.random.default_rng([9, s])
        W = r.standard_normal((M, d, F)).astype(np.float32)
        Z = r.standard_normal((M, Q, 2 * F)).astype(np.float32)
        P = oracle.trp_features(X, W, Z, ls)[:, 1:].reshape(2, M, Q)
        prods[s, 0] = np.einsum("mq,mq->m", P[0], P[0])
        prods[s, 1] = np.einsum("mq,mq->m", P[0], P[1])
        prods[s, 2] = np.einsum("mq,mq->m", P[1], P[1])
    Xd = X.astype(np.float64)
    exact = np.stack([pins.truncated_sigkernel_levels(Xd[0], Xd[0], ls, M),
                      pins.truncated_sigkernel_levels(Xd[0], Xd[1], ls, M),
                      pins.truncated_sigkernel_levels(Xd[1], Xd[1], ls, M)])
    mean = prods.mean(axis=0)
    se = prods.std(axis=0, ddof=1) / math.sqrt(S)
    assert np.all(np.abs(mean - exact) <= 4.0 * se), (mean, exact, se)
    assert np.all(exact[[0, 2], 0] > 10.0 * se[[0, 2], 0])
