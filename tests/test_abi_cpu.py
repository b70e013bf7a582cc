"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2501_07145_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(rfsf_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    lib = binding.load_library()
    names = _declared_functions()
    assert {"rfsf_ts_features", "rfsf_ts_gram", "rfsf_ts_workspace_bytes", "rfsf_ts_strerror",
            "rfsf_ts_validate_tables", "rfsf_ts_normalize_features", "rfsf_dp1d_features", "rfsf_trp_features",
            "rfsf_trp_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_covers_all_codes():
    lib = binding.load_library()
    seen = set()
    for code in range(0, -11, -1):
        s = lib.rfsf_ts_strerror(code).decode()
        assert s and "unknown" not in s
        seen.add(s)
    assert len(seen) == 11
    assert "unknown" in lib.rfsf_ts_strerror(-99).decode()


def _shape(**kw):
    base = dict(N=4, L=8, d=3, M=2, F=4, D=8, ld_out=17, rff_bf16=0, order=0)
    base.update(kw)
    return binding._Shape(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(N=-1), -2), (dict(L=0), -2), (dict(d=0), -2), (dict(M=0), -2), (dict(F=0), -2),
    (dict(D=4099, ld_out=8199), -3), (dict(D=8192, ld_out=16385), -3), (dict(D=3000, M=4, ld_out=12001), -3), (dict(D=0), -3), (dict(D=-4), -3),
    (dict(ld_out=16), -4),
])
def test_shape_validation(kw, code):
    lib = binding.load_library()
    rec, mn = ctypes.c_size_t(0), ctypes.c_size_t(0)
    shp = _shape(**kw)
    assert lib.rfsf_ts_workspace_bytes(ctypes.byref(shp), ctypes.byref(rec), ctypes.byref(mn)) == code
    # the feature call checks the shape before anything else (fake non-null pointers are never read)
    assert lib.rfsf_ts_features(ctypes.byref(shp), 256, 256, 256, 256, 1.0, 256, 256, 1 << 20, None) == code


def test_argument_validation_without_device_access():
    lib = binding.load_library()
    shp = _shape()
    assert lib.rfsf_ts_features(None, 256, 256, 256, 256, 1.0, 256, 256, 1 << 20, None) == -1
    assert lib.rfsf_ts_features(ctypes.byref(shp), None, 256, 256, 256, 1.0, 256, 256, 1 << 20, None) == -1
    assert lib.rfsf_ts_features(ctypes.byref(shp), 256, 256, 256, 256, 1.0, 256, None, 1 << 20, None) == -1
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        assert lib.rfsf_ts_features(ctypes.byref(shp), 256, 256, 256, 256, bad, 256, 256, 1 << 20, None) == -5
    assert lib.rfsf_ts_features(ctypes.byref(shp), 256, 256, 256, 256, 1.0, 256, 256, 16, None) == -6
    empty = _shape(N=0)
    assert lib.rfsf_ts_features(ctypes.byref(empty), None, None, None, None, 1.0, None, None, 0, None) == 0
    # Gram
    assert lib.rfsf_ts_gram(256, 4, 8, 256, 4, 8, 9, 256, 4, None) == -4
    assert lib.rfsf_ts_gram(256, 4, 9, 256, 4, 9, 9, 256, 3, None) == -4
    assert lib.rfsf_ts_gram(256, -1, 9, 256, 4, 9, 9, 256, 4, None) == -2
    assert lib.rfsf_ts_gram(None, 4, 9, 256, 4, 9, 9, 256, 4, None) == -1
    assert lib.rfsf_ts_gram(None, 0, 9, None, 4, 9, 9, None, 4, None) == 0
    assert lib.rfsf_ts_validate_tables(None, 256, 2, 4, 8, None) == -1
    assert lib.rfsf_ts_validate_tables(256, 256, 2, 4, 5000, None) == -3


def test_bucket_counts_that_are_no_power_of_two_are_accepted_when_small():
    lib = binding.load_library()
    rec, mn = ctypes.c_size_t(0), ctypes.c_size_t(0)
    # (1000, 5) is the paper's own largest projection size at its truncation level: a transform of 8192
    for D, M, ok in ((6, 2, True), (100, 5, True), (200, 5, True), (1000, 5, True), (1, 3, True), (2049, 2, True),
                     (1000, 9, False), (4097, 1, False)):
        shp = _shape(D=D, M=M, ld_out=1 + M * D)
        assert (lib.rfsf_ts_workspace_bytes(ctypes.byref(shp), ctypes.byref(rec), ctypes.byref(mn)) == 0) == ok


def test_order_three_outside_the_tuned_shapes_is_refused_before_anything_is_enqueued():
    # nine levels run the generic kernel, which has orders 1 and 2 only
    lib = binding.load_library()
    for D, M in ((16, 9), (64, 9)):
        shp = _shape(D=D, M=M, ld_out=1 + M * D, order=3)
        assert lib.rfsf_ts_features(ctypes.byref(shp), 256, 256, 256, 256, 1.0, 256, 256, 1 << 30, None) == -9
    # the tuned kernel addresses a slot with 16-bit byte offsets: 4032 random features at most
    for F, code in ((4032, -6), (4033, -9)):             # -6: accepted as far as the (too small) workspace
        shp = _shape(D=1024, M=1, F=F, ld_out=1 + 1024, order=3)
        assert lib.rfsf_ts_features(ctypes.byref(shp), 256, 256, 256, 256, 1.0, 256, 256, 1024, None) == code
    shp = _shape(D=64, ld_out=1 + 2 * 64, order=4)
    assert lib.rfsf_ts_features(ctypes.byref(shp), 256, 256, 256, 256, 1.0, 256, 256, 1 << 30, None) == -9


def test_trp_chunks_respect_the_grid_limit():
    # sequences per launch are capped at min(65535, 65535*64/L), whatever the workspace would hold
    lib = binding.load_library()
    rec, mn = ctypes.c_size_t(0), ctypes.c_size_t(0)
    shp = _shape(N=100000, L=32, d=2, M=2, F=4, D=8, ld_out=17)
    assert lib.rfsf_trp_workspace_bytes(ctypes.byref(shp), ctypes.byref(rec), ctypes.byref(mn)) == 0
    per = 32 * 2 * 8 * 4 + 32 * 2 * 8 * 4                # increments + projections of one sequence
    assert (rec.value - 768) // per == 50000             # two equal launches, each below 65535 sequences
    shp = _shape(N=100000, L=1 << 20, d=2, M=2, F=4, D=8, ld_out=17)
    assert lib.rfsf_trp_workspace_bytes(ctypes.byref(shp), ctypes.byref(rec), ctypes.byref(mn)) == 0
    per = (1 << 20) * 2 * 8 * 4 * 2
    assert (rec.value - 768) // per == 3                  # 65535*64 / 2^20 = 3 sequences per launch
    shp = _shape(N=4, L=1 << 23, d=2, M=2, F=4, D=8, ld_out=17)    # one sequence alone exceeds the grid
    assert lib.rfsf_trp_workspace_bytes(ctypes.byref(shp), ctypes.byref(rec), ctypes.byref(mn)) == -9


def test_workspace_sizes():
    rec, mn = binding.rfsf_ts_workspace_bytes(1000, 100, 8, 4, 128, 256)
    per_seq = 100 * 4 * 256 * 4 + 4 * 129 * 8           # increment rows + accumulator state
    assert rec - mn == 999 * per_seq                    # the rest is per-call tables and slack
    assert 0 < mn - per_seq < (1 << 20)
    rec_big, mn_big = binding.rfsf_ts_workspace_bytes(50000, 64, 64, 5, 1024, 2048)
    assert mn_big <= rec_big <= (49 << 30)


def test_binding_refuses_host_tensors():
    import torch
    X = torch.zeros(2, 4, 3)
    W = torch.zeros(2, 3, 4)
    h = torch.zeros(2, 8, dtype=torch.int32)
    s = torch.ones(2, 8)
    with pytest.raises(ValueError):
        binding.rfsf_ts_features(X, W, h, s, 1.0, 8)
    with pytest.raises(ValueError):
        binding.rfsf_ts_gram(torch.zeros(3, 5))


def test_time_cut_plan_is_a_function_of_the_shape():
    """Few long sequences are cut in time, many or short ones are not; host logic only."""
    cut = binding.rfsf_ts_time_cut
    pieces, pairs = cut(10, 100000, 5, 5, 50, 100)          # the paper's sequence-length runs (Sec. 4)
    assert 6 <= pieces <= 128 and pairs >= 32
    assert pieces * pairs >= 50000 > (pieces - 1) * pairs   # the pieces cover the L/2 pairs, none is empty
    assert cut(1, 100000, 5, 5, 50, 100)[0] == 128          # never more than 128 pieces
    assert cut(64, 100000, 5, 5, 50, 100)[0] == 16
    assert cut(65, 100000, 5, 5, 50, 100) == (1, 50000)     # from here on a workgroup per sequence is the better use of the chip
    assert cut(10000, 200, 17, 5, 512, 1024) == (1, 100)
    assert cut(10, 200, 5, 5, 50, 100) == (1, 100)          # too short for M + 1 pieces of 32 pairs
    assert cut(10, 100000, 5, 1, 50, 100)[0] == 1           # one level: nothing to join, nothing gained
    assert cut(10, 100000, 5, 5, 50, 100, order=2) == cut(10, 100000, 5, 5, 50, 100)   # any order the tuned kernels have
    assert cut(10, 100000, 5, 9, 50, 100)[0] == 1           # nine levels run the generic kernel
    # the workspace grows by the pieces' accumulators and stays consistent with the minimum
    rec, mn = binding.rfsf_ts_workspace_bytes(10, 100000, 5, 5, 50, 100)
    rec1, mn1 = binding.rfsf_ts_workspace_bytes(65, 100000, 5, 5, 50, 100)
    assert rec / 10 > rec1 / 65 and mn > mn1 and rec >= mn


def test_probe_peaks_refuses_bad_arguments():
    import ctypes
    lib = binding.load_library()
    out = binding._Peaks()
    assert lib.rfsf_ts_probe_peaks(None, 1 << 20, ctypes.byref(out), None) == -1           # no scratch
    assert lib.rfsf_ts_probe_peaks(ctypes.c_void_p(64), 1 << 20, None, None) == -1         # nowhere to write to
    assert lib.rfsf_ts_probe_peaks(ctypes.c_void_p(64), 8, ctypes.byref(out), None) == -6  # too small
