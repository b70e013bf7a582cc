"""Independent reference computations used to pin the CPU oracle.

Nothing here is shared with oracle/ or with the HIP library: each function is a
different route to a quantity the paper defines, so that a mistake in the oracle
(dropped term, wrong sign or index, transposed operand) shows up as a mismatch.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


def rff_increments_numpy(X, W, lengthscale):
    """delta[N, T, M, 2F] in fp64 from the definition of the random Fourier
    feature map (Sec. 3.1, eq. (rff)) and the time difference (Sec. 3.2, eq. (rfsf))."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    M, d, F = W.shape
    theta = np.einsum("nlc,mcf->nlmf", X, W) / float(lengthscale)
    phi = np.concatenate([np.cos(theta), np.sin(theta)], axis=-1) / math.sqrt(F)
    return phi[:, 1:] - phi[:, :-1]


def brute_force_tensor_sketch(delta, hash_, sign, D):
    """Phi[M, D] for ONE sequence from the closed definition (Sec. 3.5, eq. (ts) with
    p = 1): sum over strictly increasing time tuples i_1 < ... < i_m of the explicit
    tensor product delta_1[i_1] (x) ... (x) delta_m[i_m], each tensor coordinate
    (a_1..a_m) sent to bucket (sum_k hash_k[a_k]) mod D with sign prod_k sign_k[a_k]
    (the tensor sketch is a count sketch of the tensor product).

    delta: [T, M, 2F]; pure Python loops, tiny sizes only."""
    T, M, twoF = delta.shape
    out = np.zeros((M, D))
    for m in range(1, M + 1):
        for idx in itertools.combinations(range(T), m):
            for coords in itertools.product(range(twoF), repeat=m):
                bucket = 0
                val = 1.0
                for k in range(m):
                    a = coords[k]
                    bucket += int(hash_[k, a])
                    val *= float(sign[k, a]) * float(delta[idx[k], k, a])
                out[m - 1, bucket % D] += val
    return out


def rbf(x, y, lengthscale):
    """RBF static kernel exp(-|x-y|^2 / (2 l^2)) (appendix, class RBFKernel)."""
    diff = np.asarray(x, dtype=np.float64)[:, None, :] - np.asarray(y, dtype=np.float64)[None, :, :]
    return np.exp(-np.sum(diff * diff, axis=-1) / (2.0 * lengthscale ** 2))


def double_difference(Kmat):
    """nabla_{i,j} k = k(x_i,y_j) - k(x_{i-1},y_j) - k(x_i,y_{j-1}) + k(x_{i-1},y_{j-1})
    for i, j >= 1 (Sec. 2.1)."""
    return Kmat[1:, 1:] - Kmat[:-1, 1:] - Kmat[1:, :-1] + Kmat[:-1, :-1]


def truncated_sigkernel_levels(x, y, lengthscale, M):
    """[k_1 .. k_M]: order-1 level-m signature kernels with RBF static kernel by the
    dynamic programme of Sec. 2.2 (cumulative sums only):
        A_1 = nabla k,  A_m[i,j] = nabla k[i,j] * sum_{i'<i, j'<j} A_{m-1}[i',j']."""
    G = double_difference(rbf(x, y, lengthscale))
    A = G.copy()
    levels = [A.sum()]
    for _ in range(2, M + 1):
        S = np.cumsum(np.cumsum(A, axis=0), axis=1)
        Sx = np.zeros_like(A)
        Sx[1:, 1:] = S[:-1, :-1]               # exclusive in both indices
        A = G * Sx
        levels.append(A.sum())
    return np.array(levels)


def truncated_sigkernel_levels_bruteforce(x, y, lengthscale, M):
    """The same quantity from eq. (sigkernelm) with p = 1: explicit sum over pairs of
    strictly increasing tuples. Tiny lengths only."""
    G = double_difference(rbf(x, y, lengthscale))
    Tx, Ty = G.shape
    levels = []
    for m in range(1, M + 1):
        tot = 0.0
        for ii in itertools.combinations(range(Tx), m):
            for jj in itertools.combinations(range(Ty), m):
                p = 1.0
                for r in range(m):
                    p *= G[ii[r], jj[r]]
                tot += p
        levels.append(tot)
    return np.array(levels)


def streaming_frequency_domain(delta, hash_, sign, D):
    """Phi[M, D] for one sequence through the FFT route of eq. (ts_rec): sketch each
    increment, transform with the library real FFT, run the per-bin recurrence
        for m = M..2: A_m += A_{m-1} * C_m[k];  A_1 += C_1[k]
    over time, and invert once at the end. delta: [T, M, 2F]."""
    T, M, twoF = delta.shape
    A = np.zeros((M, D // 2 + 1), dtype=np.complex128)
    for k in range(T):
        Chat = []
        for m in range(M):
            c = np.zeros(D)
            np.add.at(c, hash_[m], sign[m] * delta[k, m])
            Chat.append(np.fft.rfft(c))
        for m in range(M - 1, 0, -1):
            A[m] += A[m - 1] * Chat[m]
        A[0] += Chat[0]
    return np.stack([np.fft.irfft(A[m], n=D) for m in range(M)])


def brute_force_tensor_sketch_order(delta, hash_, sign, D, order):
    """Phi[M, D] for ONE sequence from the closed definition with signature order p (Sec. 2.1 and Sec. 3.5
    eq. (ts)): sum over non-decreasing time tuples i_1 <= ... <= i_m in which no time index occurs more
    than p times, weighted by 1 / prod(multiplicity!), of the sketched explicit tensor product.
    delta: [T, M, 2F]; pure Python loops, tiny sizes only."""
    T, M, twoF = delta.shape
    out = np.zeros((M, D))
    for m in range(1, M + 1):
        for idx in itertools.combinations_with_replacement(range(T), m):
            mult = [len(list(g)) for _, g in itertools.groupby(idx)]
            if max(mult) > order:
                continue
            weight = 1.0
            for c in mult:
                weight /= math.factorial(c)
            for coords in itertools.product(range(twoF), repeat=m):
                bucket = 0
                val = weight
                for k in range(m):
                    a = coords[k]
                    bucket += int(hash_[k, a])
                    val *= float(sign[k, a]) * float(delta[idx[k], k, a])
                out[m - 1, bucket % D] += val
    return out
