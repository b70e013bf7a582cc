"""Parity at the full sizes of the configuration table, in the launch configuration the
benchmark times (recommended workspace, default stream): sampled rows against the oracle
(all levels), the hash-independent bucket-sum identity on more rows (a property that holds at
any size), and the Gram on sampled entries plus full rows."""
import math

import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import workloads as wl
from tests.parity import BF16_BLOCK_TOL, FP32_BLOCK_TOL, GRAM_TOL, block_errors, gram_error

pytestmark = pytest.mark.gpu


def _features(w, X, tables, workspace):
    W, hash_, sign = tables
    out = rfsf.rfsf_ts_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(),
                                torch.from_numpy(hash_).cuda(), torch.from_numpy(sign).cuda(),
                                float(np.float32(w.lengthscale)), w.D, workspace=workspace, rff_bf16=w.rff_bf16)
    torch.cuda.synchronize()
    return out


def _bucket_sum_identity(w, Xs, W, sign, got_rows, tol, batch=64):
    """sum_j Phi_m[j] = sum_{i_1<...<i_m} prod_k u_k[i_k] with the scalars u_k[t] = sum_a sign_k[a] delta_k[t][a]:
    summing a level block over its buckets removes the hash. u_k[t] = v_k[t+1] - v_k[t] with
    v_k[t] = F^-1/2 sum_f (sign_k[f] cos theta_f + sign_k[F+f] sin theta_f), evaluated here in fp64 with torch on
    the host cores (not the oracle's code)."""
    ls = float(np.float32(w.lengthscale))
    Wt = torch.from_numpy(W.astype(np.float64)) / ls
    sc = torch.from_numpy(sign[:, :w.F].astype(np.float64))
    ss = torch.from_numpy(sign[:, w.F:].astype(np.float64))
    worst = 0.0
    for r0 in range(0, Xs.shape[0], batch):
        Xb = torch.from_numpy(Xs[r0:r0 + batch].astype(np.float64))
        theta = torch.einsum("ntc,mcf->ntmf", Xb, Wt)
        v = ((torch.cos(theta) * sc).sum(dim=3) + (torch.sin(theta) * ss).sum(dim=3)) / math.sqrt(w.F)
        u = (v[:, 1:] - v[:, :-1]).numpy()
        e = np.zeros((u.shape[0], w.M + 1))
        e[:, 0] = 1.0
        for t in range(u.shape[1]):
            for m in range(w.M, 0, -1):
                e[:, m] += e[:, m - 1] * u[:, t, m - 1]
        blocks = got_rows[r0:r0 + batch, 1:].astype(np.float64).reshape(-1, w.M, w.D)
        scale = np.abs(blocks).sum(axis=2)                # the sum is compared against the block's 1-norm
        worst = max(worst, float((np.abs(blocks.sum(axis=2) - e[:, 1:]) / scale).max()))
    assert worst <= tol, worst
    return worst


def _sample_rows(w, rec_bytes, n_oracle, rng):
    """Rows for the oracle: first, last, the middle pair, both sides of every boundary between the launches the
    recommended workspace leads to, and random ones up to n_oracle."""
    if n_oracle >= w.N:
        return np.arange(w.N), 0
    _, mn = rfsf.rfsf_ts_workspace_bytes(w.N, w.L, w.d, w.M, w.F, w.D, w.rff_bf16)
    rec2, mn2 = rfsf.rfsf_ts_workspace_bytes(2, w.L, w.d, w.M, w.F, w.D, w.rff_bf16)
    chunk = (rec_bytes - mn) // (rec2 - mn2) + 1         # sequences per launch
    fixed = [0, w.N - 1, w.N // 2 - 1, w.N // 2]
    for b in range(chunk, w.N, chunk):
        fixed += [b - 1, b]
    fixed = np.unique(fixed)
    extra = rng.integers(0, w.N, size=max(0, n_oracle - len(fixed)))
    return np.unique(np.concatenate([fixed, extra])), (w.N + chunk - 1) // chunk


@pytest.mark.parametrize("name,n_oracle,n_identity", [("small", 1000, 0), ("medium", 64, 512), ("long", 16, 512),
                                                      ("large", 64, 512)])
def test_full_size(oracle, name, n_oracle, n_identity):
    w = wl.WORKLOADS[name]
    tables = wl.make_tables(w, 0)
    X = wl.make_paths(w, 0)
    rec, _ = rfsf.rfsf_ts_workspace_bytes(w.N, w.L, w.d, w.M, w.F, w.D, w.rff_bf16)
    workspace = torch.empty(rec, dtype=torch.uint8, device="cuda")
    out = _features(w, X, tables, workspace)
    ls = float(np.float32(w.lengthscale))
    tol = BF16_BLOCK_TOL if w.rff_bf16 else FP32_BLOCK_TOL

    rng = np.random.default_rng(5)
    sel, launches = _sample_rows(w, rec, n_oracle, rng)
    got = out[torch.from_numpy(sel).cuda()].cpu().numpy()
    want = oracle.features(X[sel], tables[0], tables[1], tables[2], ls, w.D)
    err = block_errors(got, want, w.M, w.D)
    print(f"{name}: {len(sel)} oracle rows ({launches} launches), block errors {err}")
    assert np.all(err <= tol)
    Xm, Wm = X, tables[0]
    if w.rff_bf16:      # kernel error alone: oracle on the operands as multiplied
        hi = wl.round_to_bf16(X)
        Xm = (hi + wl.round_to_bf16(X - hi)).astype(np.float32)
        Wm = wl.round_to_bf16(tables[0])
        same = oracle.features(Xm[sel], Wm, tables[1], tables[2], ls, w.D)
        err_same = block_errors(got, same, w.M, w.D)
        print(f"{name}: against same-operand oracle {err_same}")
        assert np.all(err_same <= FP32_BLOCK_TOL)

    if n_identity:      # for the bf16 projection: against the increments of the operands as multiplied
        rows = rng.integers(0, w.N, size=n_identity)
        worst = _bucket_sum_identity(w, Xm[rows], Wm, tables[2], out[torch.from_numpy(rows).cuda()].cpu().numpy(), 2e-5)
        print(f"{name}: bucket-sum identity on {n_identity} rows, worst relative deviation {worst:.2e}")

    # Gram: the second batch for the cross Gram, else the batch with itself
    if w.N2:
        X2 = wl.make_paths(w.scaled(N=w.N2), 1)
        out2 = _features(w.scaled(N=w.N2), X2, tables, workspace)
    else:
        out2 = out
    del workspace
    K = rfsf.rfsf_ts_gram(out, out2)
    torch.cuda.synchronize()
    ii = rng.integers(0, out.shape[0], size=4096)
    jj = rng.integers(0, out2.shape[0], size=4096)
    a = out[torch.from_numpy(ii).cuda()].double()
    b = out2[torch.from_numpy(jj).cuda()].double()
    ref = (a * b).sum(dim=1).cpu().numpy()            # fp64 dot products of the GPU features
    gotK = K[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy()
    kmax = float(K.abs().max())
    assert np.abs(gotK - ref).max() / kmax <= GRAM_TOL
    full_rows = np.array([0, out.shape[0] - 1, out.shape[0] // 3])
    ref_rows = oracle.gram(out[torch.from_numpy(full_rows).cuda()].cpu().numpy(), out2.cpu().numpy()) \
        if out2.shape[0] * out2.shape[1] <= 60_000_000 else None
    if ref_rows is not None:
        assert np.abs(K[torch.from_numpy(full_rows).cuda()].cpu().numpy() - ref_rows).max() / kmax <= GRAM_TOL
    # end to end on the oracle rows (only when both operands are the sampled batch itself)
    if not w.N2:
        Ksub = K[torch.from_numpy(sel).cuda()][:, torch.from_numpy(sel).cuda()].cpu().numpy()
        assert gram_error(Ksub, oracle.gram(want)) <= (5 * GRAM_TOL if w.rff_bf16 else GRAM_TOL)


@pytest.mark.parametrize("D,F,N", [(1000, 500, 3000), (500, 250, 4000), (3000, 256, 600)])
def test_projection_sizes_that_are_no_power_of_two(oracle, D, F, N):
    """Five levels with the paper's largest projection size (1000: exact transform, items dealt to eight
    wavefronts), with 500, and with 3000 buckets (linear route in 8192 points: wide kernel) at batch sizes that
    fill the chip several times: oracle on sampled rows, bucket-sum identity on more."""
    import dataclasses
    w = dataclasses.replace(wl.WORKLOADS["medium"], N=N, L=60, d=6, M=5 if D < 3000 else 2, F=F, D=D)
    tables = wl.make_tables(w, 3)
    X = wl.make_paths(w, 3)
    rec, _ = rfsf.rfsf_ts_workspace_bytes(w.N, w.L, w.d, w.M, w.F, w.D, w.rff_bf16)
    workspace = torch.empty(rec, dtype=torch.uint8, device="cuda")
    out = _features(w, X, tables, workspace)
    ls = float(np.float32(w.lengthscale))
    rng = np.random.default_rng(6)
    sel = np.unique(np.concatenate([[0, w.N - 1], rng.integers(0, w.N, size=6)]))
    got = out[torch.from_numpy(sel).cuda()].cpu().numpy()
    want = oracle.features(X[sel], tables[0], tables[1], tables[2], ls, w.D)
    err = block_errors(got, want, w.M, w.D)
    print(f"D={D}: {len(sel)} oracle rows, block errors {err}")
    assert np.all(err <= FP32_BLOCK_TOL)
    rows = rng.integers(0, w.N, size=256)
    worst = _bucket_sum_identity(w, X[rows], tables[0], tables[2], out[torch.from_numpy(rows).cuda()].cpu().numpy(), 2e-5)
    print(f"D={D}: bucket-sum identity on 256 rows, worst relative deviation {worst:.2e}")


def test_hundred_thousand_time_points(oracle):
    """The paper's scalability claim for the primal methods is sequence length 1e5 and beyond (Sec. 4).
    Two sequences of 100001 points in the paper's own shape (d = 5, M = 5, feature and projection size
    100); the accumulators run through 1e5 steps in fp32 and must stay within the tolerance."""
    N, L, d, M, F, D = 2, 100001, 5, 5, 50, 100
    rng = np.random.default_rng(0)
    X = np.cumsum(rng.standard_normal((N, L, d)) / math.sqrt(L), axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    hash_ = rng.integers(0, D, size=(M, 2 * F)).astype(np.int32)
    sign = (2.0 * rng.integers(0, 2, size=(M, 2 * F)) - 1.0).astype(np.float32)
    ls = float(np.float32(math.sqrt(d)))
    got = rfsf.rfsf_ts_features(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(),
                                torch.from_numpy(hash_).cuda(), torch.from_numpy(sign).cuda(), ls, D)
    torch.cuda.synchronize()
    err = block_errors(got.cpu().numpy(), oracle.features(X, W, hash_, sign, ls, D), M, D)
    print("L = 100001: block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
