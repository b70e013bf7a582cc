"""CPU pins of the fp64 oracle: each test fixes the oracle against something other
than itself (closed forms, brute force over the definition, invariants, special
cases, a library routine, the exact kernel within a statistical bound)."""
import math

import numpy as np
import pytest

from tests import pins


def _tables(rng, M, F, D):
    hash_ = rng.integers(0, D, size=(M, 2 * F)).astype(np.int32)
    sign = (2.0 * rng.integers(0, 2, size=(M, 2 * F)) - 1.0).astype(np.float32)
    return hash_, sign


def _case(seed, N, L, d, M, F, D, ls=1.3):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) * 0.4, axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    hash_, sign = _tables(rng, M, F, D)
    return X, W, hash_, sign, float(np.float32(ls))


# ---------------------------------------------------------------- stage 1-2: RFF and increments
def test_rff_single_frequency_closed_form(oracle):
    """Sec. 3.1 eq. (rff): with one non-zero entry W[m, c0, a0] = w the only moving
    coordinates are cos/sin of x[c0] * w / l at positions a0 and F + a0; every other
    cos coordinate is the constant F^{-1/2} and every other sin coordinate is 0. Pins
    the [M, d, F] indexing, the division by the lengthscale, the cos-then-sin order
    and the F^{-1/2} scale."""
    N, L, d, M, F = 2, 5, 3, 2, 4
    rng = np.random.default_rng(1)
    X = rng.standard_normal((N, L, d)).astype(np.float32)
    for (m0, c0, a0) in [(0, 2, 1), (1, 0, 3)]:
        W = np.zeros((M, d, F), dtype=np.float32)
        W[m0, c0, a0] = 0.75
        ls = 2.0
        got = oracle.increments(X, W, ls)                       # [N, T, M, 2F]
        th = X[:, :, c0].astype(np.float64) * 0.75 / ls
        want = np.zeros((N, L - 1, M, 2 * F))
        want[:, :, m0, a0] = (np.cos(th[:, 1:]) - np.cos(th[:, :-1])) / math.sqrt(F)
        want[:, :, m0, F + a0] = (np.sin(th[:, 1:]) - np.sin(th[:, :-1])) / math.sqrt(F)
        np.testing.assert_allclose(got, want, atol=1e-15)


def test_rff_kernel_identity(oracle):
    """<phi(x), phi(y)> = (1/F) sum_a cos(w_a . (x - y) / l) and |phi(x)|^2 = 1, so a
    two-point 'sequence' (x, y) has |delta|^2 = 2 - 2 <phi(x), phi(y)> (eq. (rff))."""
    rng = np.random.default_rng(2)
    d, F, ls = 4, 16, 1.7
    x, y = rng.standard_normal(d), rng.standard_normal(d)
    X = np.stack([x, y])[None].astype(np.float32)
    W = rng.standard_normal((1, d, F)).astype(np.float32)
    delta = oracle.increments(X, W, ls)[0, 0, 0]
    xy = (X[0, 0].astype(np.float64) - X[0, 1].astype(np.float64))
    kern = np.mean(np.cos(xy @ W[0].astype(np.float64) / ls))
    assert abs(delta @ delta - (2.0 - 2.0 * kern)) < 1e-14


def test_increments_match_numpy(oracle):
    X, W, _, _, ls = _case(3, N=3, L=7, d=5, M=3, F=6, D=8)
    np.testing.assert_allclose(oracle.increments(X, W, ls), pins.rff_increments_numpy(X, W, ls),
                               rtol=0, atol=1e-14)


# ---------------------------------------------------------------- the closed definition, brute force
@pytest.mark.parametrize("T,F,M,D", [(6, 2, 3, 4), (5, 1, 3, 2), (4, 2, 2, 8), (6, 2, 3, 8), (3, 2, 3, 4)])
def test_bruteforce_tuples(oracle, T, F, M, D):
    """Sec. 3.5 eq. (ts), p = 1: explicit sum over i_1 < ... < i_m of the sketched
    tensor product, coordinate by coordinate."""
    X, W, hash_, sign, ls = _case(10 + T + D, N=2, L=T + 1, d=2, M=M, F=F, D=D)
    got = oracle.features(X, W, hash_, sign, ls, D)
    delta = oracle.increments(X, W, ls)
    assert np.all(got[:, 0] == 1.0)
    for n in range(X.shape[0]):
        want = pins.brute_force_tensor_sketch(delta[n], hash_, sign, D)
        np.testing.assert_allclose(got[n, 1:].reshape(M, D), want, rtol=0, atol=1e-13)


def test_bruteforce_tuples_numpy_increments(oracle):
    """Same as above, but the increments come from the numpy formula, so the whole
    oracle (stages 1-5) is compared with an implementation that shares nothing."""
    T, F, M, D = 5, 2, 3, 4
    X, W, hash_, sign, ls = _case(77, N=1, L=T + 1, d=3, M=M, F=F, D=D)
    delta = pins.rff_increments_numpy(X, W, ls)
    want = pins.brute_force_tensor_sketch(delta[0], hash_, sign, D)
    got = oracle.features(X, W, hash_, sign, ls, D)
    np.testing.assert_allclose(got[0, 1:].reshape(M, D), want, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- invariants
def test_level1_telescopes(oracle):
    """Linearity of the count sketch (eq. (cs)): Phi_1 = CS_1(phi_1(x_last) - phi_1(x_first))."""
    X, W, hash_, sign, ls = _case(4, N=5, L=23, d=3, M=2, F=8, D=16)
    got = oracle.features(X, W, hash_, sign, ls, 16)
    F = 8
    th0 = X[:, 0].astype(np.float64) @ W[0].astype(np.float64) / ls
    th1 = X[:, -1].astype(np.float64) @ W[0].astype(np.float64) / ls
    v = np.concatenate([np.cos(th1) - np.cos(th0), np.sin(th1) - np.sin(th0)], axis=1) / math.sqrt(F)
    want = np.zeros((5, 16))
    for a in range(2 * F):
        want[:, hash_[0, a]] += sign[0, a] * v[:, a]
    np.testing.assert_allclose(got[:, 1:17], want, rtol=0, atol=1e-14)


def test_dc_and_nyquist_bins(oracle):
    """Summing a level block over buckets removes the hash: with u_k[t] = sum_a
    sign_k[a] delta_k[t][a], sum_j Phi_m[j] = sum_{i_1<...<i_m} prod_k u_k[i_k]; with
    v_k[t] = sum_a (-1)^{hash_k[a]} sign_k[a] delta_k[t][a] the alternating sum gives
    the same for v (bucket index adds under convolution)."""
    X, W, hash_, sign, ls = _case(5, N=4, L=30, d=3, M=4, F=8, D=16)
    got = oracle.features(X, W, hash_, sign, ls, 16)[:, 1:].reshape(4, 4, 16)
    delta = pins.rff_increments_numpy(X, W, ls)                 # [N, T, M, 2F]
    alt = (-1.0) ** np.arange(16)
    for weights, red in ((np.ones_like(sign, dtype=np.float64), np.ones(16)),
                         ((-1.0) ** hash_.astype(np.float64), alt)):
        u = np.einsum("ntma,ma->ntm", delta, sign * weights)
        N, T, M = u.shape
        e = np.zeros((N, M + 1))
        e[:, 0] = 1.0
        for t in range(T):                                      # elementary-symmetric-like DP
            for m in range(M, 0, -1):
                e[:, m] += e[:, m - 1] * u[:, t, m - 1]
        np.testing.assert_allclose(got @ red, e[:, 1:], rtol=0, atol=1e-13)


def test_repeated_time_point_changes_nothing(oracle):
    """A repeated point adds a zero increment; every sum over tuples ignores it."""
    X, W, hash_, sign, ls = _case(6, N=3, L=9, d=2, M=3, F=4, D=8)
    Xr = np.concatenate([X[:, :4], X[:, 3:4], X[:, 4:]], axis=1)
    np.testing.assert_allclose(oracle.features(Xr, W, hash_, sign, ls, 8),
                               oracle.features(X, W, hash_, sign, ls, 8), rtol=0, atol=1e-14)


def test_variable_lengths_equal_padding_with_the_last_point(oracle):
    """A sequence of n points padded to L by repeating its last point has the same features (the padding adds
    zero increments), also for higher signature orders; and the padded region's content is irrelevant."""
    X, W, hash_, sign, ls = _case(16, N=5, L=9, d=2, M=3, F=4, D=8)
    lengths = np.array([9, 1, 4, 2, 7])
    Xp = X.copy()
    for n, ell in enumerate(lengths):
        Xp[n, ell:] = X[n, ell - 1]
    for order in (1, 2, 3):
        want = oracle.features(Xp, W, hash_, sign, ls, 8, order=order)
        got = oracle.features_ragged(X, lengths, W, hash_, sign, ls, 8, order=order)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)
    junk = X.copy()
    for n, ell in enumerate(lengths):
        junk[n, ell:] = 1e3
    np.testing.assert_array_equal(oracle.features_ragged(junk, lengths, W, hash_, sign, ls, 8),
                                  oracle.features_ragged(X, lengths, W, hash_, sign, ls, 8))
    assert np.all(oracle.features_ragged(X, lengths, W, hash_, sign, ls, 8)[1, 1:] == 0.0)      # one point: (1, 0, ..)
    with pytest.raises(ValueError):
        oracle.features_ragged(X, np.array([9, 0, 4, 2, 7]), W, hash_, sign, ls, 8)


def test_short_sequences(oracle):
    """Empty sums: L = 1 gives (1, 0, ..); level m vanishes when m > T."""
    X, W, hash_, sign, ls = _case(7, N=2, L=3, d=2, M=4, F=4, D=8)
    one = oracle.features(X[:, :1], W, hash_, sign, ls, 8)
    assert np.all(one[:, 0] == 1.0) and np.all(one[:, 1:] == 0.0)
    two = oracle.features(X[:, :2], W, hash_, sign, ls, 8)      # T = 1
    assert np.any(two[:, 1:9] != 0.0) and np.all(two[:, 9:] == 0.0)
    three = oracle.features(X, W, hash_, sign, ls, 8)           # T = 2
    assert np.any(three[:, 9:17] != 0.0) and np.all(three[:, 17:] == 0.0)


def test_constant_hash_collapses_to_bucket_zero(oracle):
    X, W, hash_, sign, ls = _case(8, N=2, L=12, d=2, M=3, F=4, D=8)
    h0 = np.zeros_like(hash_)
    got = oracle.features(X, W, h0, sign, ls, 8)[:, 1:].reshape(2, 3, 8)
    ref = oracle.features(X, W, hash_, sign, ls, 8)[:, 1:].reshape(2, 3, 8)
    assert np.all(got[:, :, 1:] == 0.0)
    np.testing.assert_allclose(got[:, :, 0], ref.sum(axis=2), rtol=0, atol=1e-13)


def test_injective_hash_gives_unsketched_coordinates(oracle):
    """With D large and hash_k[a] = a * (2F)^k the bucket index encodes the tensor
    coordinate uniquely, so level 2 holds the unprojected signature features
    sum_{i<j} delta_1[i][a] delta_2[j][b] (Sec. 3.2, eq. (rfsf)) at bucket a + 2F b."""
    F, M, D = 2, 2, 16
    X, W, _, _, ls = _case(9, N=1, L=8, d=2, M=M, F=F, D=D)
    hash_ = np.stack([np.arange(4), 4 * np.arange(4)]).astype(np.int32)
    sign = np.ones((M, 4), dtype=np.float32)
    got = oracle.features(X, W, hash_, sign, ls, D)[0, 1:].reshape(M, D)
    delta = pins.rff_increments_numpy(X, W, ls)[0]              # [T, M, 2F]
    T = delta.shape[0]
    want = np.zeros((4, 4))
    for i in range(T):
        for j in range(i + 1, T):
            want += np.outer(delta[i, 0], delta[j, 1])
    np.testing.assert_allclose(got[1].reshape(4, 4).T, want, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- the FFT route (library routine)
@pytest.mark.parametrize("D", [8, 32, 6])
def test_matches_library_fft_route(oracle, D):
    """Sec. 3.5 eq. (ts_rec), second line: the same features through numpy's real FFT
    and the per-bin streaming recurrence. D = 6 shows the oracle does not need a power
    of two."""
    X, W, hash_, sign, ls = _case(20 + D, N=3, L=17, d=3, M=4, F=5, D=D)
    got = oracle.features(X, W, hash_, sign, ls, D)
    delta = oracle.increments(X, W, ls)
    for n in range(3):
        want = pins.streaming_frequency_domain(delta[n], hash_, sign, D)
        np.testing.assert_allclose(got[n, 1:].reshape(4, D), want, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- statistics: unbiased for the signature kernel
def test_sigkernel_dp_matches_its_definition():
    """The dynamic programme used as the exact reference equals eq. (sigkernelm), p = 1."""
    rng = np.random.default_rng(11)
    x = np.cumsum(rng.standard_normal((5, 2)) * 0.5, axis=0)
    y = np.cumsum(rng.standard_normal((6, 2)) * 0.5, axis=0)
    np.testing.assert_allclose(pins.truncated_sigkernel_levels(x, y, 1.1, 3),
                               pins.truncated_sigkernel_levels_bruteforce(x, y, 1.1, 3),
                               rtol=1e-12, atol=1e-14)


def test_unbiased_for_truncated_signature_kernel(oracle):
    """E <Phi_m(x), Phi_m(y)> = k_m(x, y) level by level (unbiasedness of RFF, of RFSF and
    of the count / tensor sketch, Secs. 3.1, 3.2, 3.5). S independent table draws;
    tolerance |mean - k_m| <= 4 SE for every level and every pair, SE = std / sqrt(S);
    and SE shrinks like S^{-1/2}."""
    L, d, F, D, M, ls = 8, 2, 16, 32, 3, 1.0
    rng = np.random.default_rng(12)
    X = np.cumsum(rng.standard_normal((2, L, d)) * 0.6, axis=1).astype(np.float32)
    S = 2000
    prods = np.zeros((S, 3, M))                                  # pairs (x,x), (x,y), (y,y)
    for s in range(S):
        r = np.random.default_rng([13, s])
        W = r.standard_normal((M, d, F)).astype(np.float32)
        hash_, sign = _tables(r, M, F, D)
        P = oracle.features(X, W, hash_, sign, ls, D)[:, 1:].reshape(2, M, D)
        prods[s, 0] = np.einsum("md,md->m", P[0], P[0])
        prods[s, 1] = np.einsum("md,md->m", P[0], P[1])
        prods[s, 2] = np.einsum("md,md->m", P[1], P[1])
    Xd = X.astype(np.float64)
    exact = np.stack([pins.truncated_sigkernel_levels(Xd[0], Xd[0], ls, M),
                      pins.truncated_sigkernel_levels(Xd[0], Xd[1], ls, M),
                      pins.truncated_sigkernel_levels(Xd[1], Xd[1], ls, M)])
    mean = prods.mean(axis=0)
    se = prods.std(axis=0, ddof=1) / math.sqrt(S)
    assert np.all(np.abs(mean - exact) <= 4.0 * se), (mean, exact, se)
    assert np.all(exact[[0, 2]] > 10.0 * se[[0, 2]])             # the diagonal pairs have power
    se_quarter = prods[: S // 4].std(axis=0, ddof=1) / math.sqrt(S // 4)
    ratio = se_quarter / se
    assert np.all((ratio > 1.5) & (ratio < 2.6)), ratio


# ---------------------------------------------------------------- Gram
def test_gram_properties(oracle):
    rng = np.random.default_rng(14)
    A = rng.standard_normal((7, 13))
    B = rng.standard_normal((5, 13))
    K = oracle.gram(A, B)
    np.testing.assert_allclose(K, A @ B.T, rtol=1e-13, atol=1e-13)
    Kaa = oracle.gram(A)
    assert np.array_equal(Kaa, Kaa.T)
    np.testing.assert_allclose(np.diag(Kaa), np.sum(A * A, axis=1), rtol=1e-14)
    assert np.linalg.eigvalsh(Kaa).min() > -1e-12


def test_gram_of_features_is_kernel_estimate(oracle):
    """K = P_X P_X^T including the level-0 column: K[i,j] = 1 + sum_m <Phi_m(x_i), Phi_m(x_j)>."""
    X, W, hash_, sign, ls = _case(15, N=4, L=6, d=2, M=2, F=4, D=8)
    P = oracle.features(X, W, hash_, sign, ls, 8)
    K = oracle.gram(P)
    blocks = P[:, 1:].reshape(4, 2, 8)
    np.testing.assert_allclose(K, 1.0 + np.einsum("imd,jmd->ij", blocks, blocks), rtol=1e-13)


def test_rejects_bad_arguments(oracle):
    X, W, hash_, sign, ls = _case(16, N=1, L=4, d=2, M=2, F=2, D=4)
    bad = hash_.copy()
    bad[0, 0] = 4
    with pytest.raises(RuntimeError):
        oracle.features(X, W, bad, sign, ls, 4)
    with pytest.raises(RuntimeError):
        oracle.features(X, W, hash_, sign, 0.0, 4)


# ---------------------------------------------------------------- level-wise normalisation
def test_normalisation_matches_the_kernel_level_formula(oracle):
    """Appendix, class SignatureBase: the normalised kernel is 1/(M+1) sum_m k_m(x,y) /
    sqrt(k_m(x,x) k_m(y,y)). Evaluated here from the Grams of the unnormalised level blocks and
    compared with the Gram of the normalised feature rows."""
    M, D = 3, 16
    X, W, hash_, sign, ls = _case(30, N=6, L=9, d=2, M=M, F=8, D=D)
    P = oracle.features(X, W, hash_, sign, ls, D)
    Pn = oracle.normalize(P, M, D)
    blocks = P[:, 1:].reshape(6, M, D)
    Km = np.einsum("imd,jmd->mij", blocks, blocks)                  # per-level Grams
    dg = np.sqrt(np.einsum("mii->mi", Km))
    want = (1.0 + (Km / (dg[:, :, None] * dg[:, None, :])).sum(axis=0)) / (M + 1)
    np.testing.assert_allclose(oracle.gram(Pn), want, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(np.diag(oracle.gram(Pn)), 1.0, rtol=1e-13)


def test_normalisation_special_cases(oracle):
    M, D = 4, 8
    X, W, hash_, sign, ls = _case(31, N=3, L=3, d=2, M=M, F=4, D=D)   # two increments: levels 3, 4 vanish
    P = oracle.features(X, W, hash_, sign, ls, D)
    Pn = oracle.normalize(P, M, D)
    assert np.all(Pn[:, 1 + 2 * D:] == 0.0)
    np.testing.assert_allclose(np.sum(Pn * Pn, axis=1), 3.0 / (M + 1), rtol=1e-13)   # levels 0, 1, 2
    # invariant under a positive rescaling of any level block; a second pass leaves the blocks alone
    Q = P.copy()
    Q[:, 1:1 + D] *= 7.5
    np.testing.assert_allclose(oracle.normalize(Q, M, D), Pn, rtol=1e-13, atol=1e-16)
    again = oracle.normalize(Pn, M, D)          # blocks already have norm 1/sqrt(M+1): unchanged
    np.testing.assert_allclose(again[:, 1:], Pn[:, 1:], rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(again[:, 0], 1.0 / (M + 1), rtol=1e-14)


# ---------------------------------------------------------------- signature order p > 1
@pytest.mark.parametrize("T,F,M,D,order", [(5, 1, 3, 4, 2), (4, 2, 3, 8, 2), (4, 1, 4, 4, 3), (3, 2, 3, 4, 3), (5, 1, 2, 2, 2)])
def test_order_p_bruteforce(oracle, T, F, M, D, order):
    """Sec. 2.1 (the weights 1 / i!^(p)) and Sec. 3.5 eq. (ts): explicit sum over non-decreasing tuples."""
    X, W, hash_, sign, ls = _case(40 + T + D + order, N=2, L=T + 1, d=2, M=M, F=F, D=D)
    got = oracle.features(X, W, hash_, sign, ls, D, order=order)
    delta = pins.rff_increments_numpy(X, W, ls)
    for n in range(2):
        want = pins.brute_force_tensor_sketch_order(delta[n], hash_, sign, D, order)
        np.testing.assert_allclose(got[n, 1:].reshape(M, D), want, rtol=0, atol=1e-13)


def test_order_one_routine_agrees_and_orders_differ(oracle):
    """The general routine at p = 1 is the strict-tuple oracle; p = 2 changes levels >= 2 only; an order
    above the number of levels changes nothing more."""
    X, W, hash_, sign, ls = _case(50, N=3, L=9, d=3, M=4, F=4, D=8)
    base = oracle.features(X, W, hash_, sign, ls, 8)
    np.testing.assert_allclose(oracle.features_order(X, W, hash_, sign, ls, 8, 1), base, rtol=0, atol=1e-14)
    two = oracle.features(X, W, hash_, sign, ls, 8, order=2)
    np.testing.assert_allclose(two[:, :9], base[:, :9], rtol=0, atol=1e-14)          # levels 0, 1
    assert np.abs(two[:, 9:] - base[:, 9:]).max() > 1e-6
    np.testing.assert_allclose(oracle.features(X, W, hash_, sign, ls, 8, order=4),
                               oracle.features(X, W, hash_, sign, ls, 8, order=7), rtol=0, atol=1e-14)


def test_order_p_single_increment(oracle):
    """One increment (L = 2): only runs of that one time index exist, so level m = (1/m!) c_1 * ... * c_m
    when m <= p and zero otherwise -- with a constant hash the convolution is a plain product."""
    X, W, hash_, sign, ls = _case(51, N=2, L=2, d=2, M=3, F=3, D=4)
    h0 = np.zeros_like(hash_)
    got = oracle.features(X, W, h0, sign, ls, 4, order=2)[:, 1:].reshape(2, 3, 4)
    delta = pins.rff_increments_numpy(X, W, ls)[:, 0]                     # [N, M, 2F]
    u = np.einsum("nma,ma->nm", delta, sign.astype(np.float64))           # bucket-0 sums
    np.testing.assert_allclose(got[:, 0, 0], u[:, 0], rtol=0, atol=1e-14)
    np.testing.assert_allclose(got[:, 1, 0], u[:, 0] * u[:, 1] / 2.0, rtol=0, atol=1e-14)
    assert np.all(got[:, 2] == 0.0) and np.all(got[:, :, 1:] == 0.0)


# ---------------------------------------------------------------- concatenation of sequences
@pytest.mark.parametrize("order", [1, 2, 3])
def test_features_of_a_sequence_cut_in_two(oracle, order):
    """Sec. 3.5 eq. (ts_rec): the index tuples of a sequence x followed by y split by how many indices fall
    into x, so level m of the whole is  S^{(1..m)}(y) + S^{(1..m)}(x) + sum_{j=1}^{m-1} S^{(1..j)}(x) * S^{(j+1..m)}(y)
    with * the circular convolution over the buckets and S^{(a..b)} the features computed with the maps
    (W, hash, sign) of tensor positions a .. b. The GPU library relies on this to cut long sequences in time;
    here the oracle is held to it (the convolution is written out directly, the pieces share the boundary point)."""
    N, L, d, M, F, D = 2, 11, 3, 4, 5, 7
    X, W, hash_, sign, ls = _case(41, N, L, d, M, F, D)
    feats = (lambda *a: oracle.features(*a)) if order == 1 else (lambda *a: oracle.features_order(*a, order))
    whole = feats(X, W, hash_, sign, ls, D)[:, 1:].reshape(N, M, D)
    for cut in (1, 4, 9):
        x, y = X[:, :cut + 1], X[:, cut:]

        def S(piece, a, b):                                     # positions a .. b (1-based), blocks [N, b-a+1, D]
            return feats(piece, W[a - 1:b], hash_[a - 1:b], sign[a - 1:b], ls, D)[:, 1:].reshape(N, b - a + 1, D)

        for m in range(1, M + 1):
            want = S(y, 1, m)[:, m - 1] + S(x, 1, m)[:, m - 1]
            for j in range(1, m):
                left, right = S(x, 1, j)[:, j - 1], S(y, j + 1, m)[:, m - j - 1]
                conv = np.zeros((N, D))
                for p in range(D):
                    for q in range(D):
                        conv[:, (p + q) % D] += left[:, p] * right[:, q]
                want = want + conv
            np.testing.assert_allclose(whole[:, m - 1], want, rtol=1e-9, atol=1e-12)
