"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs, element by element, block-normalised (max relative error per feature block)."""
import numpy as np
import pytest
import torch

import paper_2501_07145_amd as rfsf
from paper_2501_07145_amd import binding, workloads as wl
from tests.parity import BF16_BLOCK_TOL, FP32_BLOCK_TOL, GRAM_TOL, block_errors, gram_error

pytestmark = pytest.mark.gpu


def _dev(inp):
    return {k: (torch.from_numpy(v).cuda() if isinstance(v, np.ndarray) else v) for k, v in inp.items()}


def _gpu_features(inp, D, **kw):
    t = _dev(inp)
    out = rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], D, **kw)
    torch.cuda.synchronize()
    return out


def _random_case(seed, N, L, d, M, F, D, ls=1.5, step=0.3):
    rng = np.random.default_rng(seed)
    X = np.cumsum(rng.standard_normal((N, L, d)) * step, axis=1).astype(np.float32)
    W = rng.standard_normal((M, d, F)).astype(np.float32)
    hash_ = rng.integers(0, D, size=(M, 2 * F)).astype(np.int32)
    sign = (2.0 * rng.integers(0, 2, size=(M, 2 * F)) - 1.0).astype(np.float32)
    return {"X": X, "W": W, "hash": hash_, "sign": sign, "lengthscale": float(np.float32(ls))}


def _check(inp, D, oracle, tol=FP32_BLOCK_TOL, **kw):
    M = inp["W"].shape[0]
    got = _gpu_features(inp, D, **kw).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D)
    err = block_errors(got, want, M, D)
    assert np.all(err <= tol), f"block errors {err} exceed {tol}"
    return got, want, err


def test_tiny_all_rows(oracle):
    w = wl.WORKLOADS["tiny"]
    inp = wl.make_inputs(w, 0)
    got, want, err = _check(inp, w.D, oracle)
    print("tiny block errors", err)
    K = rfsf.rfsf_ts_gram(torch.from_numpy(got).cuda())
    torch.cuda.synchronize()
    assert gram_error(K.cpu().numpy(), oracle.gram(want)) <= GRAM_TOL


def test_small_64_rows(oracle):
    w = wl.WORKLOADS["small"].scaled(N=64)
    inp = wl.make_inputs(w, 0)
    _, _, err = _check(inp, w.D, oracle)
    print("small[64] block errors", err)


@pytest.mark.parametrize("N,L,d,M,F,D", [
    (5, 37, 5, 3, 24, 32),      # F not a multiple of the tile, D != 2F, odd number of increments
    (3, 36, 1, 2, 1, 2),        # smallest d, F, D
    (4, 9, 7, 1, 40, 128),      # one level
    (2, 2, 3, 4, 16, 16),       # one increment: levels above 1 vanish
    (2, 3, 3, 4, 16, 16),       # two increments: levels above 2 vanish
    (3, 2, 3, 4, 32, 64),       # one increment on the tuned kernel: the padded second step adds exactly nothing
    (2, 4, 5, 5, 64, 1024),     # three increments, five levels
    (7, 65, 19, 6, 70, 64),     # several row tiles with a ragged tail, six levels, D < 2F
    (2, 20, 4, 2, 8, 4096),     # largest D
    (3, 300, 33, 3, 130, 512),  # d above one MFMA K-slab, F with a ragged column tile
    (1, 1000, 2, 5, 16, 8),     # long and narrow
    (3, 24, 6, 5, 100, 1024),   # D = 1024, three-pass transform
    (2, 11, 4, 2, 300, 2048),   # D = 2048: one transform per pair of wavefronts
    (1, 6, 2, 8, 16, 2048),     # D = 2048 with eight levels: 1024 threads, 155 KB of LDS
    (2, 5, 3, 5, 1100, 2048),   # D = 2048 with more coordinates than buckets: eight slots exceed the LDS, one wavefront per level
    (2, 7, 3, 5, 1500, 1024),   # the same for D = 1024 with five levels
    (3, 8, 3, 3, 700, 600),     # 600 buckets in a transform of 2048 (two wavefronts per transform), odd number of increments
    (2, 40, 3, 8, 20, 256),     # eight levels
    (2, 30, 3, 9, 12, 64),      # nine levels: generic kernel
    (3, 50, 5, 7, 33, 128),     # seven levels, D = 128
    (2, 9, 70, 2, 40, 64),      # d above 64: plain vector projection kernel
    (1, 4, 2, 1, 4100, 64),     # 2F above the 16-bit table offsets: generic sketch kernel
    (1, 5, 2, 1, 4032, 1024),    # the most coordinates the tuned sketch kernel takes (16-bit byte offsets into a slot)
    (1, 5, 2, 1, 4033, 1024),    # one more: generic sketch kernel
    (2, 12, 3, 2, 600, 256),    # 2F much larger than D: staging area beyond the transform length
])
def test_ragged_shapes(oracle, N, L, d, M, F, D):
    inp = _random_case(100 + N + L + D, N, L, d, M, F, D)
    _, _, err = _check(inp, D, oracle)
    print(f"N={N} L={L} d={d} M={M} F={F} D={D} block errors", err)


def test_no_increments_and_empty_batch(oracle):
    inp = _random_case(1, 3, 1, 2, 3, 4, 8)
    got = _gpu_features(inp, 8).cpu().numpy()
    assert np.all(got[:, 0] == 1.0) and np.all(got[:, 1:] == 0.0)
    empty = _random_case(2, 0, 5, 2, 3, 4, 8)
    assert tuple(_gpu_features(empty, 8).shape) == (0, 25)


def test_chunked_execution_matches(oracle):
    """A workspace that holds only a few sequences forces several launches per call."""
    inp = _random_case(3, 11, 21, 4, 3, 16, 32)
    _, mn = rfsf.rfsf_ts_workspace_bytes(11, 21, 4, 3, 16, 32)
    _, mn2 = rfsf.rfsf_ts_workspace_bytes(12, 21, 4, 3, 16, 32)
    rec2, _ = rfsf.rfsf_ts_workspace_bytes(2, 21, 4, 3, 16, 32)
    per_seq = rec2 - mn2                                 # recommended(N=2) - minimum = one more sequence
    assert mn == mn2
    for nseq in (1, 3):
        ws = torch.empty(mn + (nseq - 1) * per_seq, dtype=torch.uint8, device="cuda")
        _check(inp, 32, oracle, workspace=ws)
    with pytest.raises(binding.RfsfTsError) as e:
        _gpu_features(inp, 32, workspace=torch.empty(mn - 1, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -6


def test_row_stride_and_untouched_padding(oracle):
    inp = _random_case(4, 6, 15, 3, 2, 8, 16)
    ncols = 1 + 2 * 16
    buf = torch.full((6, ncols + 7), -7.0, dtype=torch.float32, device="cuda")
    _check(inp, 16, oracle, out=buf)
    assert torch.all(buf[:, ncols:] == -7.0)


def test_hash_is_reduced_modulo_D_and_sign_uses_only_the_sign_bit(oracle):
    inp = _random_case(5, 4, 12, 3, 2, 8, 16)
    wild = dict(inp)
    wild["hash"] = (inp["hash"] + 16 * np.arange(16, dtype=np.int32)[None, :]).astype(np.int32)
    wild["sign"] = (inp["sign"] * 3.5).astype(np.float32)
    got = _gpu_features(wild, 16).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], 16)
    assert np.all(block_errors(got, want, 2, 16) <= FP32_BLOCK_TOL)


def test_validate_tables():
    inp = _dev(_random_case(6, 1, 4, 2, 2, 8, 16))
    rfsf.rfsf_ts_validate_tables(inp["hash"], inp["sign"], 16)
    bad_h = inp["hash"].clone()
    bad_h[1, 3] = 16
    with pytest.raises(binding.RfsfTsError) as e:
        rfsf.rfsf_ts_validate_tables(bad_h, inp["sign"], 16)
    assert e.value.code == -8
    bad_s = inp["sign"].clone()
    bad_s[0, 0] = 0.5
    with pytest.raises(binding.RfsfTsError):
        rfsf.rfsf_ts_validate_tables(inp["hash"], bad_s, 16)


def test_large_angles(oracle):
    """Angles of a few hundred radians: the range reduction must stay accurate."""
    inp = _random_case(7, 4, 30, 3, 3, 32, 64, ls=0.02, step=0.05)
    _check(inp, 64, oracle)


def test_runs_on_a_side_stream(oracle):
    inp = _random_case(8, 5, 18, 3, 3, 16, 32)
    s = torch.cuda.Stream()
    t = _dev(inp)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], 32, stream=s)
        K = rfsf.rfsf_ts_gram(out, stream=s)
    s.synchronize()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], 32)
    assert np.all(block_errors(out.cpu().numpy(), want, 3, 32) <= FP32_BLOCK_TOL)
    assert gram_error(K.cpu().numpy(), oracle.gram(want)) <= GRAM_TOL


# ------------------------------------------------------------------ Gram
@pytest.mark.parametrize("Nx,Ny,C,pad", [(16, 16, 193, 0), (70, 45, 1025, 3), (1, 1, 1, 0), (129, 257, 37, 1),
                                         (300, 64, 2049, 0), (65, 130, 516, 0)])
def test_gram_against_oracle(oracle, Nx, Ny, C, pad):
    rng = np.random.default_rng(Nx + Ny + C)
    A = rng.standard_normal((Nx, C + pad)).astype(np.float32)
    B = rng.standard_normal((Ny, C + pad)).astype(np.float32)
    K = rfsf.rfsf_ts_gram(torch.from_numpy(A).cuda()[:, :C], torch.from_numpy(B).cuda()[:, :C])
    torch.cuda.synchronize()
    assert gram_error(K.cpu().numpy(), oracle.gram(A[:, :C], B[:, :C])) <= GRAM_TOL


def test_gram_unaligned_base_and_strided_output(oracle):
    rng = np.random.default_rng(9)
    A = rng.standard_normal((33, 101)).astype(np.float32)
    flat = torch.zeros(33 * 101 + 1, dtype=torch.float32, device="cuda")
    flat[1:] = torch.from_numpy(A).cuda().reshape(-1)
    Ad = flat[1:].view(33, 101)                      # base is 4 bytes off a 16-byte boundary
    Kbuf = torch.full((33, 40), -3.0, dtype=torch.float32, device="cuda")
    rfsf.rfsf_ts_gram(Ad, Ad, K=Kbuf[:, :33])
    torch.cuda.synchronize()
    assert gram_error(Kbuf[:, :33].cpu().numpy(), oracle.gram(A)) <= GRAM_TOL
    assert torch.all(Kbuf[:, 33:] == -3.0)
    assert torch.equal(Kbuf[:, :33], Kbuf[:, :33].T.contiguous())


# ------------------------------------------------------------------ degenerate tables, reproducibility
@pytest.mark.parametrize("kind", ["constant", "two_buckets", "identity"])
def test_degenerate_hash_tables(oracle, kind):
    """All coordinates in one bucket (every coordinate but two goes through a fold round of its
    own), two buckets, and a collision-free hash."""
    inp = _random_case(11, 3, 14, 3, 3, 64, 128)
    if kind == "constant":
        inp["hash"] = np.full_like(inp["hash"], 5)
    elif kind == "two_buckets":
        inp["hash"] = (np.arange(128, dtype=np.int32)[None, :] % 2 * 77).repeat(3, axis=0).astype(np.int32)
    else:
        inp["hash"] = np.arange(128, dtype=np.int32)[None, :].repeat(3, axis=0).copy()
    _check(inp, 128, oracle)


def test_results_are_bit_reproducible():
    """No atomics anywhere on the tuned path: two calls give identical bits."""
    w = wl.WORKLOADS["small"].scaled(N=96)
    inp = wl.make_inputs(w, 0)
    a = _gpu_features(inp, w.D).clone()
    b = _gpu_features(inp, w.D).clone()
    assert torch.equal(a, b)
    Ka, Kb = rfsf.rfsf_ts_gram(a).clone(), rfsf.rfsf_ts_gram(b).clone()
    torch.cuda.synchronize()
    assert torch.equal(Ka, Kb)


@pytest.mark.parametrize("N,C", [(2100, 517), (2049, 64), (4500, 100), (1000, 1025), (4501, 70), (4222, 33)])
def test_symmetric_gram_path(oracle, N, C):
    """K = Phi Phi^T with one operand: only the upper triangle is computed, the rest mirrored."""
    rng = np.random.default_rng(N + C)
    ld = (C + 3) // 4 * 4
    A = rng.standard_normal((N, ld)).astype(np.float32)
    Ad = torch.from_numpy(A).cuda()[:, :C]
    K = rfsf.rfsf_ts_gram(Ad)
    torch.cuda.synchronize()
    assert gram_error(K.cpu().numpy(), oracle.gram(A[:, :C])) <= GRAM_TOL
    assert torch.equal(K, K.T.contiguous())
    K2 = rfsf.rfsf_ts_gram(Ad, Ad.clone())                 # two operands: the general path
    torch.cuda.synchronize()
    assert gram_error(K2.cpu().numpy(), K.cpu().numpy()) <= 1e-5       # different kernels, different summation order


@pytest.mark.parametrize("N,L,d,M,F,D", [
    (4, 20, 3, 3, 40, 100),     # the paper's own bucket count: transform length 512
    (3, 15, 4, 5, 64, 200),     # 1024
    (3, 12, 2, 2, 8, 6),        # tiny: generic kernel, transform length 16
    (2, 9, 3, 4, 16, 3),        # D = 3
    (2, 30, 3, 2, 50, 1000),    # 2048
    (2, 9, 3, 5, 40, 300),      # 2048 through five levels
    (2, 7, 2, 3, 5, 1),         # a single bucket
    (2, 8, 3, 5, 50, 1000),     # the paper's largest projection size at its truncation level: 8192, buffers in global memory
    (2, 9, 2, 2, 30, 2049),     # 8192 with two levels
    (2, 6, 3, 3, 20, 1366),     # 4096 (4096 >= 3*1365+1)
])
def test_bucket_counts_that_are_no_power_of_two(oracle, N, L, d, M, F, D):
    """Circular convolution modulo D through a longer power-of-two transform: the M-fold convolution of
    sketches that occupy [0, D) is linear as long as the transform holds M*(D-1)+1 numbers; the result is
    folded modulo D at the end."""
    inp = _random_case(300 + D, N, L, d, M, F, D)
    _, _, err = _check(inp, D, oracle)
    print(f"D={D} M={M} block errors", err)


@pytest.mark.parametrize("N,L,d,M,F,D", [
    (4, 12, 3, 3, 32, 64),      # tuned kernel, several pairs per wavefront
    (3, 9, 4, 5, 64, 1024),     # one pair per wavefront
    (2, 8, 3, 4, 16, 16),       # generic kernel
    (2, 7, 2, 3, 20, 100),      # bucket count that is no power of two
    (2, 2, 3, 4, 16, 256),      # one increment: level 2 = (1/2) c_1 * c_2, levels 3, 4 vanish
    (6, 31, 5, 4, 128, 256),    # odd number of increments
    (2, 9, 3, 3, 16, 4096),     # longest power-of-two bucket count: the generic kernel's buffers move to global memory
    (2, 7, 3, 3, 20, 1500),     # 8192 with order 2
])
def test_signature_order_two(oracle, N, L, d, M, F, D):
    """A time step may be used twice in a row, with weight 1/2 (Sec. 2.1; Sec. 3.5 eq. (ts_rec), q = 2)."""
    inp = _random_case(400 + D + L, N, L, d, M, F, D)
    got = _gpu_features(inp, D, order=2).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=2)
    err = block_errors(got, want, M, D)
    print(f"order 2, D={D} M={M}: block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
    one = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D)
    if L > 2:
        assert block_errors(got, one, M, D)[1:].max() > 1e-3       # it is not the order-1 map
    with pytest.raises(binding.RfsfTsError) as e:
        _gpu_features(inp, D, order=4)
    assert e.value.code == -9


@pytest.mark.parametrize("N,L,d,M,F,D", [
    (4, 12, 3, 3, 32, 64),      # several pairs per wavefront
    (3, 9, 4, 5, 64, 1024),     # one pair per wavefront
    (2, 11, 3, 8, 16, 256),     # eight levels
    (2, 7, 2, 3, 20, 100),      # bucket count that is no power of two (transform length 512)
    (2, 2, 3, 4, 16, 256),      # one increment: level 3 = (1/6) c_1 * c_2 * c_3
    (5, 30, 5, 4, 128, 512),    # odd number of increments, two pairs per wavefront
    (2, 6, 3, 3, 40, 2048),     # a transform spanning two wavefronts
])
def test_signature_order_three(oracle, N, L, d, M, F, D):
    """A time step may be used up to three times in a row, q equal indices weighted 1/q! (Sec. 2.1; Sec. 3.5
    eq. (ts_rec), q = 1, 2, 3)."""
    inp = _random_case(500 + D + L, N, L, d, M, F, D)
    got = _gpu_features(inp, D, order=3).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=3)
    err = block_errors(got, want, M, D)
    print(f"order 3, D={D} M={M}: block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
    two = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=2)
    if M >= 3:
        assert block_errors(got, two, M, D)[2:].max() > 1e-3        # it is not the order-2 map
    if D == 64:     # 16 buckets run in a transform of 64 points (tuned kernel: order 3 there too) ...
        small = _random_case(1, 2, 6, 2, 2, 4, 16)
        got16 = _gpu_features(small, 16, order=3).cpu().numpy()
        want16 = oracle.features(small["X"], small["W"], small["hash"], small["sign"], small["lengthscale"], 16, order=3)
        assert np.all(block_errors(got16, want16, 2, 16) <= FP32_BLOCK_TOL)
        nine = _random_case(2, 2, 6, 2, 9, 4, 16)           # ... nine levels leave the tuned kernels: refused
        with pytest.raises(binding.RfsfTsError) as e:
            _gpu_features(nine, 16, order=3)
        assert e.value.code == -9


@pytest.mark.parametrize("L", [2, 3, 5, 8, 13, 21, 34])
@pytest.mark.parametrize("order", [1, 2, 3])
def test_two_pairs_per_wavefront_dealt_to_eight_wavefronts(oracle, L, order):
    """Transforms of 512 with five levels: the items, here groups of two pairs of one level, go to eight
    wavefronts in order; the lengths give last groups with one and with two pairs and last iterations with
    different numbers of items. Also as a batch of different lengths."""
    N, d, M, F, D = 4, 3, 5, 40, 512
    inp = _random_case(1200 + L, N, L, d, M, F, D)
    got = _gpu_features(inp, D, order=order).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=order)
    assert np.all(block_errors(got, want, M, D) <= FP32_BLOCK_TOL)
    lengths = np.array([L, 1, max(1, L - 1), max(1, L // 2)])
    t = _dev(inp)
    got_r = rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], D, order=order,
                                  lengths=torch.from_numpy(lengths).cuda()).cpu().numpy()
    want_r = oracle.features_ragged(inp["X"], lengths, inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D,
                                    order=order)
    assert np.all(block_errors(got_r, want_r, M, D) <= FP32_BLOCK_TOL)


@pytest.mark.parametrize("D", [100, 200, 500, 1000])
@pytest.mark.parametrize("M,F,L,order", [
    (1, 30, 9, 1),        # one level
    (2, 64, 8, 2),        # order 2, odd number of increments
    (3, 130, 12, 3),      # order 3
    (4, 50, 31, 1),       # several iterations, F < D/2 for the larger D
    (5, 700, 6, 1),       # more coordinates than buckets for most D; five levels (D = 1000: dealt to eight wavefronts)
    (6, 33, 14, 2),       # six levels
    (8, 20, 7, 1),        # eight levels
])
def test_bucket_counts_of_the_papers_experiments(oracle, D, M, F, L, order):
    """D = 100, 200, 500, 1000 (Sec. 4 of the paper uses such projection sizes) have transforms of exactly that
    length: radix-10, -5 and -2 passes, lanes beyond D/20 per transform repeating the first ones. Also as a batch
    of different lengths, and with nine levels, where the shape leaves the tuned kernel and takes the
    linear-convolution route again."""
    N, d = 3, 3
    inp = _random_case(1000 + D + L + M, N, L, d, M, F, D)
    got = _gpu_features(inp, D, order=order).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=order)
    err = block_errors(got, want, M, D)
    print(f"D={D} M={M} F={F} L={L} order {order}: block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
    lengths = np.array([L, 1, max(1, L - 1)])
    t = _dev(inp)
    got_r = rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], D, order=order,
                                  lengths=torch.from_numpy(lengths).cuda()).cpu().numpy()
    want_r = oracle.features_ragged(inp["X"], lengths, inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D,
                                    order=order)
    assert np.all(block_errors(got_r, want_r, M, D) <= FP32_BLOCK_TOL)


def test_nine_levels_of_a_hundred_buckets_take_the_linear_route(oracle):
    inp = _random_case(77, 2, 6, 2, 9, 12, 100)
    _check(inp, 100, oracle)


@pytest.mark.parametrize("N,L,d,M,F,D,order", [
    (2, 9, 3, 1, 40, 4096, 1),       # one level: a single level slot per workgroup
    (2, 8, 3, 2, 40, 4096, 2),       # two levels: level l belongs to slot l for good; odd number of increments
    (3, 12, 3, 3, 700, 4096, 1),     # three levels dealt to two slots; 1400 coordinates
    (2, 7, 2, 5, 64, 4096, 3),       # five levels, order 3
    (2, 6, 2, 8, 24, 4096, 1),       # eight levels
    (2, 5, 3, 2, 3000, 4096, 1),     # more coordinates than buckets: the staging area exceeds the transform
    (2, 9, 3, 2, 40, 4000, 1),       # 8192 points, two levels (4000 buckets)
    (2, 8, 3, 2, 300, 3000, 2),      # 8192 points, two levels, order 2
    (3, 11, 3, 5, 500, 1000, 1),     # the paper's largest projection size at its truncation level
    (2, 6, 2, 5, 500, 1000, 3),      # ... with order 3, odd number of increments
    (2, 10, 2, 8, 100, 1000, 1),     # eight levels of 1000 buckets
    (3, 13, 4, 5, 250, 500, 2),      # 500 buckets at five levels: 4096 points
])
def test_transforms_of_4096_and_8192(oracle, N, L, d, M, F, D, order):
    """Bucket counts whose transform has 4096 or 8192 points (4096 itself and non-powers of two, convolved linearly
    and folded at the end): several interleaved 1024-point transforms and a combining pass, levels dealt to two
    level slots. Also as a batch of different lengths."""
    inp = _random_case(900 + D + L + M, N, L, d, M, F, D)
    got = _gpu_features(inp, D, order=order).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=order)
    err = block_errors(got, want, M, D)
    print(f"D={D} M={M} F={F} L={L} order {order}: block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
    lengths = np.array(([L, 1, max(1, L - 1)])[:N])
    t = _dev(inp)
    got_r = rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], D, order=order,
                                  lengths=torch.from_numpy(lengths).cuda()).cpu().numpy()
    want_r = oracle.features_ragged(inp["X"], lengths, inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D,
                                    order=order)
    assert np.all(block_errors(got_r, want_r, M, D) <= FP32_BLOCK_TOL)


@pytest.mark.parametrize("L", [2, 3, 4, 5, 6, 7, 10, 17])
@pytest.mark.parametrize("M,order", [(5, 1), (6, 1), (5, 2), (6, 3)])
def test_levels_dealt_to_eight_wavefronts(oracle, L, M, order):
    """Transforms of 1024 with 5 or 6 levels: the (pair, level) items go to eight wavefronts in order, so a pair
    may be split between iterations and the last iteration has between one and eight items. The lengths cover
    every remainder of pairs * M modulo 8 for both level counts, with odd and even numbers of increments; each
    case also runs with a bucket count of 200 (M = 5: linear convolution in a transform of 1024) and as a
    batch of different lengths."""
    N, d, F, D = 6, 3, 48, 1024
    inp = _random_case(700 + L + 10 * M, N, L, d, M, F, D)
    got = _gpu_features(inp, D, order=order).cpu().numpy()
    want = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=order)
    err = block_errors(got, want, M, D)
    print(f"L={L} M={M} order {order}: block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
    lengths = np.array([L, 1, max(1, L - 1), max(1, L // 2), 2, max(1, L - 2)])
    t = _dev(inp)
    got_r = rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], D, order=order,
                                  lengths=torch.from_numpy(lengths).cuda()).cpu().numpy()
    want_r = oracle.features_ragged(inp["X"], lengths, inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D,
                                    order=order)
    assert np.all(block_errors(got_r, want_r, M, D) <= FP32_BLOCK_TOL)
    if M == 5:
        D2 = 200
        inp2 = _random_case(800 + L, N, L, d, M, F, D2)
        got2 = _gpu_features(inp2, D2, order=order).cpu().numpy()
        want2 = oracle.features(inp2["X"], inp2["W"], inp2["hash"], inp2["sign"], inp2["lengthscale"], D2, order=order)
        assert np.all(block_errors(got2, want2, M, D2) <= FP32_BLOCK_TOL)


@pytest.mark.parametrize("N,L,d,M,F,D,order", [
    (9, 33, 3, 3, 32, 64, 1),       # several pairs per wavefront
    (7, 20, 4, 5, 64, 1024, 1),     # one pair per wavefront
    (6, 17, 3, 4, 100, 2048, 1),    # a transform spanning two wavefronts
    (6, 14, 2, 3, 6, 16, 1),        # generic kernel
    (6, 19, 3, 4, 32, 256, 2),      # order 2
    (5, 12, 2, 3, 20, 100, 3),      # order 3, bucket count that is no power of two
])
def test_variable_length_batches(oracle, N, L, d, M, F, D, order):
    """Sequences of different lengths padded to L (appendix, ksig.preprocessing): row n equals the feature map of
    the first lengths[n] points alone, whatever the padding holds."""
    inp = _random_case(600 + D + L, N, L, d, M, F, D)
    rng = np.random.default_rng(L)
    lengths = rng.integers(1, L + 1, size=N)
    lengths[:4] = [L, 1, 2, L - 1]                                     # full, no increment, one, odd/even mix
    X = inp["X"].copy()
    for n, ell in enumerate(lengths):
        X[n, ell:] = 1e4 * (n + 1)                                     # padding content must not matter
    t = _dev(inp)
    got = rfsf.rfsf_ts_features(torch.from_numpy(X).cuda(), t["W"], t["hash"], t["sign"], inp["lengthscale"], D,
                                order=order, lengths=torch.from_numpy(lengths).cuda())
    torch.cuda.synchronize()
    want = oracle.features_ragged(inp["X"], lengths, inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D,
                                  order=order)
    err = block_errors(got.cpu().numpy(), want, M, D)
    print(f"variable lengths {lengths.tolist()}, D={D} M={M} order {order}: block errors", err)
    assert np.all(err <= FP32_BLOCK_TOL)
    # out-of-range entries are clamped into [1, L]
    bad = torch.from_numpy(np.array([0, -5, L + 7] + [L] * (N - 3))).cuda()
    got2 = rfsf.rfsf_ts_features(t["X"], t["W"], t["hash"], t["sign"], inp["lengthscale"], D, order=order,
                                 lengths=bad).cpu().numpy()
    full = oracle.features(inp["X"], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D, order=order)
    assert np.all(got2[:2, 1:] == 0.0) and np.all(block_errors(got2[2:], full[2:], M, D) <= FP32_BLOCK_TOL)


@pytest.mark.parametrize("N,L,d,M,F", [
    (300, 1000, 3, 2, 128),     # 2364 workgroups of eight tiles: the projection kernel takes row ranges of four tiles
    (301, 999, 3, 2, 100),      # the same with an odd sequence length (padded row space) and a partly used slab
    (5000, 100, 4, 1, 100),     # 1969 workgroups of eight tiles: ranges of two tiles over many short sequences
])
def test_projection_row_ranges_between_the_small_and_the_large_problems(oracle, N, L, d, M, F):
    """The projection kernel cuts the rows into ranges of 62, 126 or 254 increments by the size of the problem;
    the small test shapes only see the first and the full-size ones the last. Rows at both ends, at range
    boundaries and in the middle against the oracle."""
    D = 64
    inp = _random_case(N + L, N, L, d, M, F, D, step=0.05)
    got = _gpu_features(inp, D).cpu().numpy()
    sel = np.unique(np.array([0, 1, N // 7, N // 2, N // 2 + 1, N - 2, N - 1] +
                             [min(N - 1, (126 * k) // (L - 1)) for k in (1, 2, 3, 50, 777)]))
    want = oracle.features(inp["X"][sel], inp["W"], inp["hash"], inp["sign"], inp["lengthscale"], D)
    err = block_errors(got[sel], want, M, D)
    assert np.all(err <= FP32_BLOCK_TOL), err
    # every row: level 1 telescopes to the sketch of phi(x_L) - phi(x_1), so its buckets sum to the signed sum of
    # that difference; a row written to the wrong place or skipped shows up here
    lvl1 = got[:, 1:1 + D].sum(axis=1)
    X, W, sign, ls = inp["X"].astype(np.float64), inp["W"].astype(np.float64), inp["sign"].astype(np.float64), inp["lengthscale"]
    th1, th0 = X[:, -1] @ W[0] / ls, X[:, 0] @ W[0] / ls
    dphi = np.concatenate([np.cos(th1) - np.cos(th0), np.sin(th1) - np.sin(th0)], axis=1) / np.sqrt(F)
    np.testing.assert_allclose(lvl1, dphi @ sign[0], atol=2e-4)
