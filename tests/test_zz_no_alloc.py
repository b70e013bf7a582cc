"""The entry point that allocates nothing (rfsf_ts_features_static, built-in 64 MiB scratch) against
rfsf_ts_features with a caller workspace: same kernels, same per-sequence arithmetic, so the results must be
identical bit for bit. Two calls in a row on the same GPU, the second with a smaller input, so that whatever
the first call left in the shared scratch is still there when the second runs."""
import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import binding, workloads as wl
from tests.parity import FP32_BLOCK_TOL, block_errors

pytestmark = pytest.mark.gpu


def _inputs(w):
    inp = wl.make_inputs(w, 0)
    return inp, {k: torch.from_numpy(v).cuda() for k, v in inp.items() if isinstance(v, np.ndarray)}


def _both(w, dev, ls, **kw):
    ld = rfsf.feature_row_stride(w.M, w.D)
    ref = rfsf.rfsf_ts_features(dev["X"], dev["W"], dev["hash"], dev["sign"], ls, w.D, **kw)
    out = torch.full((w.N, ld), -7.0, dtype=torch.float32, device="cuda")
    got = rfsf.rfsf_ts_features_static(dev["X"], dev["W"], dev["hash"], dev["sign"], ls, w.D, out, **kw)
    torch.cuda.synchronize()
    assert torch.all(out[:, w.ncols:] == -7.0)          # columns beyond 1 + M*D untouched
    return ref.cpu().numpy(), got.cpu().numpy()


def test_static_scratch_matches_workspace_path_twice(oracle):
    # first call: 1000 sequences of 0.41 MB of increments each, i.e. seven launches through the 64 MiB scratch
    big = wl.WORKLOADS["small"]
    inp, dev = _inputs(big)
    ref, got = _both(big, dev, inp["lengthscale"])
    assert np.array_equal(ref, got)
    sel = np.array([0, 158, 159, 160, 999])
    want = oracle.features(inp["X"][sel], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], big.D)
    assert np.all(block_errors(got[sel], want, big.M, big.D) <= FP32_BLOCK_TOL)
    # second call, smaller input of another shape (other table sizes, a bucket count that is no power of two)
    small = wl.WORKLOADS["paper"].scaled(N=5, L=40)
    inp2, dev2 = _inputs(small)
    ref2, got2 = _both(small, dev2, inp2["lengthscale"])
    assert np.array_equal(ref2, got2)
    want2 = oracle.features(inp2["X"], inp2["W"], inp2["hash"], inp2["sign"], inp2["lengthscale"], small.D)
    assert np.all(block_errors(got2, want2, small.M, small.D) <= FP32_BLOCK_TOL)
    # third: signature order 2 on the tiny workload
    tiny = wl.WORKLOADS["tiny"]
    inp3, dev3 = _inputs(tiny)
    ref3, got3 = _both(tiny, dev3, inp3["lengthscale"], order=2)
    assert np.array_equal(ref3, got3)
    # fourth: nine levels run the generic kernel, whose accumulator state also lives in the scratch
    gen = wl.Workload("generic", N=6, L=20, d=3, M=9, F=8, D=32, lengthscale=1.0, kind="brownian")
    inp4, dev4 = _inputs(gen)
    ref4, got4 = _both(gen, dev4, inp4["lengthscale"])
    assert np.array_equal(ref4, got4)
    want4 = oracle.features(inp4["X"], inp4["W"], inp4["hash"], inp4["sign"], inp4["lengthscale"], gen.D)
    assert np.all(block_errors(got4, want4, gen.M, gen.D) <= FP32_BLOCK_TOL)

    # fifth: three long sequences, cut in time; the accumulators of their pieces live in the scratch as well
    cut = wl.WORKLOADS["paper"].scaled(N=3, L=1000)
    assert rfsf.rfsf_ts_time_cut(cut.N, cut.L, cut.d, cut.M, cut.F, cut.D)[0] > 1
    inp5, dev5 = _inputs(cut)
    ref5, got5 = _both(cut, dev5, inp5["lengthscale"])
    assert np.array_equal(ref5, got5)
    want5 = oracle.features(inp5["X"], inp5["W"], inp5["hash"], inp5["sign"], inp5["lengthscale"], cut.D)
    assert np.all(block_errors(got5, want5, cut.M, cut.D) <= FP32_BLOCK_TOL)


def test_static_scratch_rejects_what_does_not_fit():
    # one sequence of the long workload has 2000 * 4 * 512 * 4 B = 16 MB of increments: fits; 20000 steps do not
    X = torch.zeros(1, 20000, 2, device="cuda")
    W = torch.zeros(4, 2, 256, device="cuda")
    h = torch.zeros(4, 512, dtype=torch.int32, device="cuda")
    s = torch.ones(4, 512, device="cuda")
    out = torch.zeros(1, 1 + 4 * 512, device="cuda")
    with pytest.raises(binding.RfsfTsError) as e:
        rfsf.rfsf_ts_features_static(X, W, h, s, 1.0, 512, out)
    assert e.value.code == -10
    assert torch.all(out == 0)
