"""Host-side checks of the seeded input generators (no method arithmetic involved)."""
import numpy as np
import pytest

from paper_2501_07145_amd import workloads as wl


def test_shapes_and_determinism():
    w = wl.WORKLOADS["tiny"]
    a, b = wl.make_inputs(w, 0), wl.make_inputs(w, 0)
    assert a["X"].shape == (16, 32, 3) and a["X"].dtype == np.float32
    assert a["W"].shape == (3, 3, 32) and a["hash"].shape == (3, 64) and a["sign"].shape == (3, 64)
    assert a["hash"].dtype == np.int32 and a["hash"].min() >= 0 and a["hash"].max() < 64
    assert set(np.unique(a["sign"])) == {-1.0, 1.0}
    for k in ("X", "W", "hash", "sign"):
        assert np.array_equal(a[k], b[k])
    assert not np.array_equal(a["X"], wl.make_paths(w, 1))
    assert np.all(a["X"][:, 0] == 0.0)


def test_chunking_does_not_change_the_stream():
    w = wl.WORKLOADS["small"].scaled(N=37)
    assert np.array_equal(wl.make_paths(w, 3, chunk=5), wl.make_paths(w, 3, chunk=64))


def test_tables_do_not_depend_on_batch_size():
    w = wl.WORKLOADS["large"]
    t0 = wl.make_tables(w, 0)
    t1 = wl.make_tables(w.scaled(N=8, N2=4), 0)
    for a, b in zip(t0, t1):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("name", ["tiny", "small", "medium", "long", "large"])
def test_path_statistics(name):
    w = wl.WORKLOADS[name].scaled(N=64)
    X = wl.make_paths(w, 0).astype(np.float64)
    assert X.shape == (64, w.L, w.d) and np.all(np.isfinite(X))
    inc = np.diff(X, axis=1)
    if w.kind == "brownian":
        assert abs(inc.var() * w.L - 1.0) < 0.1
    if w.kind == "brownian_time":
        assert np.allclose(X[:, :, -1], np.arange(w.L) / w.L)
        assert abs(inc[:, :, :-1].var() * w.L - 1.0) < 0.1
    if w.kind == "brownian_scaled":
        v = inc.var(axis=(0, 1)) * w.L
        assert np.all(v > 0.2) and np.all(v < 4.4)
    if w.kind == "ou":
        assert abs(inc.var() * w.L - 1.0) < 0.1           # sigma^2 dt dominates over one step
        assert X[:, -1].var() < 0.6                        # mean reversion: below Brownian's 1.0


def test_bf16_rounding_matches_torch():
    import torch
    a = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37.0
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(wl.round_to_bf16(a), want)
