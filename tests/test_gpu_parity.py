"""GPU parity: the HIP library (through its C ABI binding) against the CPU oracle, element by
element, on the same seeded inputs.  Integer work (re-blocked streams) is compared bit for bit,
floating point within 1e-5 * (sum |X W| + |b|), integer-valued inputs bit for bit."""
import numpy as np
import pytest

import oracle
import paper_2510_06957_amd as tg
import synth_inputs as si
from gpu_util import assert_close, assert_exact, decode_device_form, gpu_tstgemm

pytestmark = pytest.mark.gpu

# (M, K, N): tiny and odd shapes, sizes that span several tiles with ragged tails, both kernels
SHAPES = [(1, 1, 1), (3, 37, 5), (2, 513, 65), (8, 64, 1), (5, 130, 9), (9, 37, 5), (17, 513, 65), (64, 512, 512),
          (65, 200, 130), (100, 320, 70), (129, 130, 67), (200, 1000, 100), (257, 257, 65), (300, 64, 64)]


@pytest.mark.parametrize("K,N,density", [(37, 5, 0.5), (513, 65, 0.5), (512, 512, 0.5), (1000, 130, 0.0625),
                                         (64, 9, 1.0), (130, 70, 0.0), (256, 3, 1.0), (2049, 20, 0.25)])
def test_reblocked_streams_decode_to_w(K, N, density):
    W, _, _ = si.make_inputs(1, K, N, density, "uniform", seed=200 + K + N)
    t = tg.tcsc_upload(tg.tcsc_build(W))
    Wdev, canon = decode_device_form(t)
    assert np.array_equal(Wdev, W)
    o = oracle.tcsc_build(W)
    for a, e in zip(canon, (o.col_start_pos, o.col_start_neg, o.row_index_pos, o.row_index_neg)):
        assert np.array_equal(a, e)


@pytest.mark.parametrize("M,K,N", SHAPES)
@pytest.mark.parametrize("dist", ["normal", "int8"])
def test_small_shapes(M, K, N, dist):
    W, X, b = si.make_inputs(M, K, N, 0.5, dist, seed=300 + M + K + N)
    Y, _ = gpu_tstgemm(W, X, b)
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    if dist == "int8":
        assert_exact(Y, Yd, f"{M}x{K}x{N} integer")
    else:
        assert_close(Y, Yd, A, f"{M}x{K}x{N}")


@pytest.mark.parametrize("M", [1, 4, 8, 40, 130, 256])
def test_integer_x_real_bias_is_exact(M):
    """The bias is added once, last: integer sums are exact, so one rounding decides the result."""
    W, X, _ = si.make_inputs(M, 700, 96, 0.5, "int8", seed=17)
    b = si.draw_dense(np.random.Generator(np.random.PCG64(18)), (96,), "normal")
    Y, _ = gpu_tstgemm(W, X, b)
    Yd, _, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    assert np.array_equal(Y, Yd.astype(np.float32))


@pytest.mark.parametrize("M", [3, 70])
def test_degenerate_matrices(M):
    K, N = 150, 40
    _, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=23)
    # all zero: Y = b exactly; no bias: exact zeros
    Y, h = gpu_tstgemm(np.zeros((K, N), np.int8), X, b)
    assert np.array_equal(Y, np.broadcast_to(b, Y.shape))
    Y0, _ = gpu_tstgemm(np.zeros((K, N), np.int8), X, None, handle=h)
    assert np.all(Y0 == 0)
    # all +1 / all -1 columns, one nonzero per column (a gather)
    W = np.zeros((K, N), np.int8)
    W[:, 0], W[:, 1] = 1, -1
    pick = np.random.default_rng(1).integers(0, K, size=N - 2)
    W[pick, np.arange(2, N)] = 1
    Y, _ = gpu_tstgemm(W, X, None)
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), None)
    assert_close(Y, Yd, A, "degenerate")
    assert np.array_equal(Y[:, 2:], X[:, pick])


def test_zero_weight_entries_of_x_are_never_read():
    """Gather semantics (additions and subtractions only, Sec. 2): a non-finite X entry whose weights are all zero
    must not reach Y -- also not through the padding of the index streams."""
    for M in (4, 80):
        W, X, b = si.make_inputs(M, 300, 50, 0.5, "normal", seed=29)
        W[[0, 7, 64, 299], :] = 0
        X[:, [0, 7, 64, 299]] = [np.nan, np.inf, -np.inf, np.nan]
        Y, _ = gpu_tstgemm(W, X, b)
        assert np.all(np.isfinite(Y))
        Xf = X.copy()
        Xf[:, [0, 7, 64, 299]] = 0
        Yd, A, _ = oracle.tstgemm(Xf, oracle.tcsc_build(W), b)
        assert_close(Y, Yd, A, f"nan-guard M={M}")


def test_negation_and_repeatability():
    W, X, b = si.make_inputs(96, 640, 128, 0.25, "normal", seed=31)
    Y1, h = gpu_tstgemm(W, X, None)
    Y2, _ = gpu_tstgemm(W, X, None, handle=h)
    assert np.array_equal(Y1.view(np.uint32), Y2.view(np.uint32))   # same bits on every call
    # -W swaps the two lists, which changes the fp32 summation order: equal within the tolerance, not bitwise
    Yn, _ = gpu_tstgemm(-W, X, None)
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(-W), None)
    assert_close(Yn, Yd, A, "negated W")
    assert np.all(np.abs(Yn.astype(np.float64) + Y1) <= 2e-5 * A)


@pytest.mark.parametrize("name", ["C1", "C2", "C3a", "C3b", "C4-1", "C4-8"])
@pytest.mark.parametrize("dist", [None, "int8"])
def test_benchmark_configs_full(name, dist):
    """Every element of the single-GPU benchmark configurations, in the launch configuration bench.py times."""
    W, X, b = si.make_workload(name, dist=dist)
    Y, _ = gpu_tstgemm(W, X, b)
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    if dist == "int8":
        assert_exact(Y, Yd, f"{name} integer")
    else:
        assert_close(Y, Yd, A, name)


@pytest.mark.parametrize("name", ["M64-K16384-N4096-d0.5", "M64-K4096-N4096-d0.0625", "M32-K16384-N1024-d0.25",
                                  "M8-K8192-N4096-d0.5", "M1024-K4096-N1024-d0.25"])
def test_paper_sweep_shapes_full(name):
    """Every element of the largest shapes of the paper's own sweeps (Sec. 4), one per kernel and tile height, in the
    launch configuration bench.py times; an integer-valued run bit for bit."""
    W, X, b = si.make_workload(name)
    ot = oracle.tcsc_build(W)
    Y, h = gpu_tstgemm(W, X, b)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    assert_close(Y, Yd, A, name)
    Xi = si.draw_dense(np.random.Generator(np.random.PCG64(6)), X.shape, "int8")
    Yi, _ = gpu_tstgemm(W, Xi, b, handle=h)
    assert np.array_equal(Yi, oracle.tstgemm(Xi, ot, b)[0].astype(np.float32))


@pytest.mark.parametrize("name", ["C5a", "C5b", "C5c"])
def test_prefill_configs_full(name):
    """M=4096, K=N=8192 at 50 %, 25 % and 6.25 %: EVERY element of Y, in the launch configuration bench.py times
    (16 row tiles, 128-column workgroups, no K slices), against the oracle, which goes through the rows in slabs of
    512 to bound host memory; then an integer-valued X, every element bit for bit (real-valued bias: one rounding)."""
    w = si.WORKLOADS[name]
    W, X, b = si.make_workload(name)
    ot = oracle.tcsc_build(W)
    Y, h = gpu_tstgemm(W, X, b)
    Xi = si.draw_dense(np.random.Generator(np.random.PCG64(5)), X.shape, "int8")
    Yi, _ = gpu_tstgemm(W, Xi, b, handle=h)
    for m0 in range(0, w.M, 512):
        rows = np.arange(m0, min(m0 + 512, w.M), dtype=np.int32)
        Yd, A, _ = oracle.tstgemm(X, ot, b, rows=rows)
        assert_close(Y[rows], Yd, A, f"{name} rows {m0}..{rows[-1]}")
        Ydi, _, _ = oracle.tstgemm(Xi, ot, b, rows=rows)
        assert np.array_equal(Yi[rows], Ydi.astype(np.float32)), f"{name} integer rows {m0}..{rows[-1]}"


@pytest.mark.parametrize("cols_per_wave", [1, 2, 4, 8])
@pytest.mark.parametrize("k_slices", [1, 3, 8])
def test_launch_shapes(cols_per_wave, k_slices):
    """Every launch shape of the large-M path (columns per wavefront, K slices with the reduction kernel, X packed
    and processed in slabs of one or two row tiles) gives the same, correct result; integer inputs bit for bit.
    (Eight columns per wavefront never slice K: the request for slices is ignored there.)"""
    M, K, N = 600, 700, 200
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=41)
    _, Xi, _ = si.make_inputs(M, K, N, 0.5, "int8", seed=42)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, b)
    h = None
    for slab_tiles in (0, 1, 2):
        shape = dict(cols_per_wave=cols_per_wave, k_slices=k_slices, slab_tiles=slab_tiles)
        Y, h = gpu_tstgemm(W, X, b, handle=h, **shape)
        assert_close(Y, Yd, A, f"ncw={cols_per_wave} ks={k_slices} slab={slab_tiles}")
        Yi, _ = gpu_tstgemm(W, Xi, b, handle=h, **shape)
        assert np.array_equal(Yi, Ydi.astype(np.float32))


@pytest.mark.parametrize("M,K,N,density", [(100, 300, 256, 0.1), (700, 130, 384, 0.03), (300, 200, 200, 0.5),
                                             (257, 64, 100, 0.06)])
def test_eight_columns_per_wavefront(M, K, N, density):
    """The launch shape for low densities (8 columns per wavefront, gather groups of at most 4), forced here on small
    shapes: both tile heights, a column count that is and one that is not a multiple of 128 (the latter falls back to 4
    columns), ragged N; against the oracle, integer inputs bit for bit."""
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=4242 + M)
    _, Xi, bi = si.make_inputs(M, K, N, density, "int8", seed=4243 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, bi)
    Y, h = gpu_tstgemm(W, X, b, cols_per_wave=8)
    assert_close(Y, Yd, A, "8 columns per wavefront")
    Yi, _ = gpu_tstgemm(W, Xi, bi, handle=h, cols_per_wave=8)
    assert np.array_equal(Yi, Ydi.astype(np.float32))


def test_low_density_tall_and_wide_picks_its_own_shape():
    """Tall X, wide and sparse W: rows x columns fill the chip with 128-column workgroups, so the library takes the
    low-density launch shape by itself.  Whole rows and scattered elements against the oracle; integer inputs exact."""
    M, K, N = 4096, 200, 4096
    W, X, b = si.make_inputs(M, K, N, 0.05, "uniform", seed=777)
    ot = oracle.tcsc_build(W)
    Y, h = gpu_tstgemm(W, X, b)
    rows = np.array([0, 1, 255, 256, 2047, 4095], dtype=np.int32)
    Yd, A, _ = oracle.tstgemm(X, ot, b, rows=rows)
    assert_close(Y[rows], Yd, A, "rows")
    rng = np.random.Generator(np.random.PCG64(9))
    ms, ns = rng.integers(0, M, 4096), rng.integers(0, N, 4096)
    Yp, Ap = oracle.tstgemm_points(X, ot, b, ms, ns)
    assert_close(Y[ms, ns], Yp, Ap, "points")
    Xi = si.draw_dense(np.random.Generator(np.random.PCG64(5)), X.shape, "int8")
    Yi, _ = gpu_tstgemm(W, Xi, b, handle=h)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, b, rows=rows)
    assert np.array_equal(Yi[rows], Ydi.astype(np.float32))


@pytest.mark.parametrize("cols_per_wave", [0, 1, 4])
@pytest.mark.parametrize("k_slices", [0, 1, 3, 8])
@pytest.mark.parametrize("M,K,N,density", [(64, 1100, 200, 0.5), (33, 257, 70, 0.5), (9, 2100, 40, 0.0625),
                                           (50, 600, 130, 1.0), (16, 256, 64, 0.25), (32, 1100, 100, 0.5),
                                           (20, 513, 40, 0.25), (31, 1536, 64, 1.0)])
@pytest.mark.parametrize("list_walk", [1, 2])
def test_small_tile_launch_shapes(cols_per_wave, k_slices, M, K, N, density, list_walk):
    """The path for 8 < M <= 64 (one tile of 64 rows with blocks of 256 rows of W, or of 32 rows with blocks of 512):
    lists shorter and longer than one step of the wavefront, empty slices, K below, at and above the block size, a
    last block that ends early, with and without K slices; both walks of the lists on every case."""
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=61 + M)
    _, Xi, _ = si.make_inputs(M, K, N, density, "int8", seed=62 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, b)
    shape = dict(cols_per_wave=cols_per_wave, k_slices=k_slices, list_walk=list_walk)
    Y, h = gpu_tstgemm(W, X, b, **shape)
    assert_close(Y, Yd, A, f"ncw={cols_per_wave} ks={k_slices} walk={list_walk}")
    Yi, _ = gpu_tstgemm(W, Xi, b, handle=h, **shape)
    assert np.array_equal(Yi, Ydi.astype(np.float32))


@pytest.mark.parametrize("list_walk", [1, 2])
@pytest.mark.parametrize("M,K,N,density", [(64, 700, 48, d) for d in (0.02, 0.1, 0.3, 0.7, 1.0)] +
                                          [(16, 2500, 48, d) for d in (0.02, 0.3, 1.0)] + [(32, 1300, 32, 0.6)])
def test_small_tile_slice_lengths(M, K, N, density, list_walk):
    """Slices of every length -- none, a few entries, a partly filled step alone, one to sixteen whole steps with and
    without a partly filled one in front (a column of a block of 256 / 1024 rows holds 0 .. 256 / 1024 entries of one
    sign; the random matrices make all of these lengths over their columns and blocks) -- through both walks."""
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=81 + M)
    # a few columns of one sign only and one empty column: the longest and the shortest slices there are
    W[:, 0] = 1
    W[:, 1] = -1
    W[:, 2] = 0
    _, Xi, _ = si.make_inputs(M, K, N, density, "int8", seed=82 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = gpu_tstgemm(W, X, b, list_walk=list_walk)
    assert_close(Y, Yd, A, f"{M}x{K}x{N} d={density} walk={list_walk}")
    Yi, _ = gpu_tstgemm(W, Xi, b, handle=h, list_walk=list_walk)
    assert np.array_equal(Yi, oracle.tstgemm(Xi, ot, b)[0].astype(np.float32))


@pytest.mark.parametrize("M,K,N,density", [(40, 40000, 70, 0.25), (64, 300, 20000, 0.5), (20, 70000, 33, 0.0625),
                                           (9, 513, 30000, 0.125)])
def test_small_tile_long_k_and_wide_n(M, K, N, density):
    """The small-tile path with many blocks of K per workgroup (more than eight K slices' worth) and with thousands of
    column groups."""
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=71 + M)
    _, Xi, _ = si.make_inputs(M, K, N, density, "int8", seed=72 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = gpu_tstgemm(W, X, b)
    assert_close(Y, Yd, A, f"{M}x{K}x{N}")
    Yi, _ = gpu_tstgemm(W, Xi, b, handle=h)
    assert np.array_equal(Yi, oracle.tstgemm(Xi, ot, b)[0].astype(np.float32))


def test_very_tall_x():
    """M = 70000 rows against a small matrix: hundreds of row tiles, several of them per workgroup column."""
    M, K, N = 70000, 70, 33
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=95)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = gpu_tstgemm(W, X, b)
    assert_close(Y, Yd, A, f"{M}x{K}x{N}")
    # the same through slabs of three row tiles; K is then sliced, which is another summation order: the oracle is
    # the yardstick again
    Y3, _ = gpu_tstgemm(W, X, b, handle=h, slab_tiles=3)
    assert_close(Y3, Yd, A, f"{M}x{K}x{N} in slabs")


def test_very_tall_x_wide_columns():
    """Tall X against 256 columns: enough (row tile, 128-column group) pairs for the shape with 8 columns per
    wavefront to be taken by itself; the same forced through slabs of three row tiles."""
    M, K, N = 70000, 70, 256
    W, X, b = si.make_inputs(M, K, N, 0.3, "normal", seed=96)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = gpu_tstgemm(W, X, b)
    assert_close(Y, Yd, A, f"{M}x{K}x{N}")
    Y3, _ = gpu_tstgemm(W, X, b, handle=h, cols_per_wave=8, slab_tiles=3)
    assert_close(Y3, Yd, A, f"{M}x{K}x{N} in slabs, 8 columns per wavefront")


@pytest.mark.parametrize("M", [3, 40, 130, 300])
def test_very_long_k(M):
    """K = 100000 (1563 K-blocks, 391 list cuts, several LDS chunks of the decode kernel) with a handful of columns:
    every path with far more blocks of K per workgroup than any benchmark shape has."""
    K, N = 100000, 70
    W, X, b = si.make_inputs(M, K, N, 0.25, "normal", seed=91 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = gpu_tstgemm(W, X, b)
    assert_close(Y, Yd, A, f"{M}x{K}x{N}")
    Xi = si.draw_dense(np.random.Generator(np.random.PCG64(92)), X.shape, "int8")
    Yi, _ = gpu_tstgemm(W, Xi, b, handle=h)
    assert np.array_equal(Yi, oracle.tstgemm(Xi, ot, b)[0].astype(np.float32))


@pytest.mark.parametrize("M,K,N", [(70, 130, 67), (300, 516, 100), (6, 130, 40), (40, 130, 67)])
def test_unaligned_operands(M, K, N):
    """X, b and Y that start 4 bytes off a 16-byte boundary (views into larger tensors): the element-wise paths."""
    import torch
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=43)
    t = tg.tcsc_upload(tg.tcsc_build(W))
    Xbuf = torch.zeros(M * K + 1, dtype=torch.float32, device="cuda")
    bbuf = torch.zeros(N + 1, dtype=torch.float32, device="cuda")
    Ybuf = torch.full((M * N + 1,), float("nan"), dtype=torch.float32, device="cuda")
    Xd, bd, Yd_ = Xbuf[1:].view(M, K), bbuf[1:], Ybuf[1:].view(M, N)
    assert Xd.data_ptr() % 16 == 4
    Xd.copy_(torch.from_numpy(X))
    bd.copy_(torch.from_numpy(b))
    tg.tstgemm(Xd, t, bd, Yd_)
    torch.cuda.synchronize()
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    assert_close(Yd_.cpu().numpy(), Yd, A, f"unaligned {M}x{K}x{N}")


def test_measurement_probes_run():
    """The three probe kernels of the library run to completion and report the bytes they moved (what bench.py divides
    by their time): LDS reads, a streaming read, and the tile exchange by itself on a buffer of one and of many pieces."""
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert tg.tstgemm_probe_lds_read(3) == 2 * cus * 1024 * 16 * 8 * 3
    buf = torch.zeros((1 << 20) + 40, dtype=torch.uint8, device="cuda")
    assert tg.tstgemm_probe_stream_read(buf[:1 << 20]) == 1 << 20
    assert tg.tstgemm_probe_tile_copy(buf[:65536], 5) == 2 * cus * 65536 * 5
    assert tg.tstgemm_probe_tile_copy(buf, 7) == 2 * cus * 65536 * 7          # 16 whole pieces; the 40 bytes behind them are not read
    torch.cuda.synchronize()


def test_profile_events_bracket_the_main_kernel():
    import torch
    W, X, b = si.make_workload("C1")
    t = tg.tcsc_upload(tg.tcsc_build(W))
    Xd, bd = torch.from_numpy(X).cuda(), torch.from_numpy(b).cuda()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); e1.record()
    torch.cuda.synchronize()
    Y = tg.tstgemm(Xd, t, bd, events=(e0, e1))
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    assert 0.0 < ms < 50.0
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    assert_close(Y.cpu().numpy(), Yd, A, "C1 with events")


@pytest.mark.parametrize("M,K,N", [(1, 300, 70), (8, 513, 65), (40, 700, 130), (40, 2100, 130), (20, 1100, 70),
                                   (200, 640, 96), (300, 1000, 200)])
@pytest.mark.parametrize("per_column", [False, True])
def test_prelu_epilogue(M, K, N, per_column):
    """The fused PReLU (after the bias add) in the decode kernel, the small-tile and large-M kernels and the split-K
    reduction kernel, against the oracle's; integer inputs with power-of-two slopes bit for bit."""
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=61 + M)
    rng = np.random.default_rng(62)
    alpha = rng.uniform(-1.5, 2.5, N).astype(np.float32) if per_column else np.array([0.25], np.float32)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Yp, Ap = oracle.prelu(Yd, A, alpha)
    Y, h = gpu_tstgemm(W, X, b, alpha=alpha)
    assert (Yd < 0).any() and (Yd > 0).any()
    assert_close(Y, Yp, Ap, f"prelu {M}x{K}x{N}")
    # exact: integer X and b, slopes that are powers of two
    _, Xi, bi = si.make_inputs(M, K, N, 0.5, "int8", seed=63 + M)
    a2 = (2.0 ** rng.integers(-3, 3, N)).astype(np.float32) * rng.choice([-1.0, 1.0], N).astype(np.float32) \
        if per_column else np.array([0.5], np.float32)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, bi)
    Ypi, _ = oracle.prelu(Ydi, None, a2)
    Yi, _ = gpu_tstgemm(W, Xi, bi, handle=h, alpha=a2)
    assert_exact(Yi, Ypi, f"prelu integer {M}x{K}x{N}")


@pytest.mark.parametrize("per_column", [False, True])
def test_prelu_in_the_eight_column_shape(per_column):
    """The fused PReLU in the output path of the large-M kernel's shape with 8 columns per wavefront (vector stores of
    two pieces of four columns, and the single stores of a ragged last column group)."""
    M, K, N = 300, 150, 380   # n_pad = 384 = 3 x 128
    W, X, b = si.make_inputs(M, K, N, 0.2, "normal", seed=91)
    rng = np.random.default_rng(92)
    alpha = rng.uniform(-1.5, 2.5, N).astype(np.float32) if per_column else np.array([0.25], np.float32)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Yp, Ap = oracle.prelu(Yd, A, alpha)
    _, Xi, bi = si.make_inputs(M, K, N, 0.2, "int8", seed=93)
    a2 = (2.0 ** rng.integers(-3, 3, N)).astype(np.float32) if per_column else np.array([0.5], np.float32)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, bi)
    Ypi, _ = oracle.prelu(Ydi, None, a2)
    Y, h = gpu_tstgemm(W, X, b, alpha=alpha, cols_per_wave=8)
    assert_close(Y, Yp, Ap, "prelu, 8 columns per wavefront")
    Yi, _ = gpu_tstgemm(W, Xi, bi, handle=h, alpha=a2, cols_per_wave=8)
    assert_exact(Yi, Ypi, "prelu integer, 8 columns per wavefront")


def test_prelu_rejects_bad_slopes():
    import torch
    W, X, b = si.make_inputs(4, 64, 8, 0.5, "normal", seed=64)
    t = tg.tcsc_upload(tg.tcsc_build(W))
    with pytest.raises(ValueError):
        tg.tstgemm(torch.from_numpy(X).cuda(), t, alpha=torch.zeros(3, device="cuda"))
    lib = tg.binding._load()
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.empty((4, 8), device="cuda")
    assert lib.tstgemm_prelu(Xd.data_ptr(), t.handle, None, None, 1, Yd.data_ptr(), 4, 64, 8, None) == -1
    a = torch.zeros(8, device="cuda")
    assert lib.tstgemm_prelu(Xd.data_ptr(), t.handle, None, a.data_ptr(), 3, Yd.data_ptr(), 4, 64, 8, None) == -1


@pytest.mark.parametrize("M,K,N", [(8, 4799, 40), (8, 4800, 40), (8, 8229, 70), (5, 20000, 33), (1, 40001, 20),
                                   (2, 77000, 9)])
def test_decode_k_chunks(M, K, N):
    """M <= 8 with more of X than the LDS holds: K is taken in chunks, each list is consumed chunk by chunk (at the
    chunk border a round of 256 indices is split between two chunks); real inputs within tolerance, integer inputs
    bit for bit."""
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=71 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = gpu_tstgemm(W, X, b)
    assert_close(Y, Yd, A, f"decode chunks {M}x{K}x{N}")
    _, Xi, bi = si.make_inputs(M, K, N, 0.5, "int8", seed=72 + M)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, bi)
    Yi, _ = gpu_tstgemm(W, Xi, bi, handle=h)
    assert_exact(Yi, Ydi, f"decode chunks integer {M}x{K}x{N}")


@pytest.mark.parametrize("M", [4, 40, 300])
def test_calls_can_be_captured_in_a_hip_graph(M):
    """tstgemm() enqueues kernels only (no allocation, no host synchronisation, no memset), so a stream capture
    records it; every replay, with new contents of X in the same buffer and eager work in between, must give
    the eager result bit for bit."""
    import torch
    K, N = 700, 200
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=81 + M)
    t = tg.tcsc_upload(tg.tcsc_build(W))
    Xd = torch.from_numpy(X).cuda()
    bd = torch.from_numpy(b).cuda()
    Yg = torch.empty((M, N), dtype=torch.float32, device="cuda")
    tg.tstgemm(Xd, t, bd, Yg)                       # first call outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            tg.tstgemm(Xd, t, bd, Yg, stream=side)
    torch.cuda.synchronize()
    rng = np.random.default_rng(82)
    for rep in range(4):
        Xn = rng.standard_normal((M, K)).astype(np.float32)
        Xd.copy_(torch.from_numpy(Xn).cuda())
        Yg.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        Ye = tg.tstgemm(Xd, t, bd)                  # eager, same inputs
        torch.cuda.synchronize()
        assert torch.equal(Yg, Ye), f"replay {rep}"
        Yd, A, _ = oracle.tstgemm(Xn, oracle.tcsc_build(W), b)
        assert_close(Yg.cpu().numpy(), Yd, A, f"graph replay {rep}")


def test_handles_share_one_workspace_and_streams_run_side_by_side():
    """Matrices uploaded without a workspace of their own: two of them go through ONE caller-supplied workspace on one
    stream, call after call, while a third runs on a second stream with a workspace of its own; every result against
    the oracle, integer inputs bit for bit.  The shapes take the large-M path (with K slices), the small-tile path and
    the large-M path again."""
    import torch
    shapes = [(256, 1024, 512), (40, 2100, 130), (300, 700, 200)]
    forms = tg.FORM_ROWSETS | tg.FORM_CUTS
    problems = []
    for i, (M, K, N) in enumerate(shapes):
        W, X, b = si.make_inputs(M, K, N, 0.5, "int8" if i == 1 else "normal", seed=880 + i)
        t = tg.tcsc_upload(tg.tcsc_build(W), forms=forms)
        assert tg.tcsc_layout(t).workspace_bytes == 0 and tg.tcsc_device_bytes(t) < 8 << 20
        Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
        problems.append((t, torch.from_numpy(X).cuda(), torch.from_numpy(b).cuda(), Yd, A))
    need = [tg.tstgemm_workspace_bytes(*s) for s in shapes]
    shared = torch.empty(max(need[0][1], need[1][1]), dtype=torch.uint8, device="cuda")
    own = torch.empty(need[2][1], dtype=torch.uint8, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = [[], [], []]
    for rep in range(3):
        for i in (0, 1):
            t, Xd, bd, _, _ = problems[i]
            outs[i].append(tg.tstgemm(Xd, t, bd, stream=s1, workspace=shared))
        t, Xd, bd, _, _ = problems[2]
        outs[2].append(tg.tstgemm(Xd, t, bd, stream=s2, workspace=own))
    torch.cuda.synchronize()
    for i, (t, Xd, bd, Yd, A) in enumerate(problems):
        for Y in outs[i]:
            if i == 1:
                assert_exact(Y.cpu().numpy(), Yd, f"problem {i}")
            else:
                assert_close(Y.cpu().numpy(), Yd, A, f"problem {i}")
            assert torch.equal(Y, outs[i][0])
    # no workspace at all, one below the minimum, a form that was not uploaded
    t, Xd, bd, _, _ = problems[0]
    with pytest.raises(tg.TstgemmError) as err:
        tg.tstgemm(Xd, t, bd)
    assert err.value.code == -8
    with pytest.raises(tg.TstgemmError) as err:
        tg.tstgemm(Xd, t, bd, workspace=shared[:need[0][0] - 256])
    assert err.value.code == -8
    with pytest.raises(tg.TstgemmError) as err:
        tg.tstgemm_signed(Xd[:4].contiguous(), t, bd)
    assert err.value.code == -7
    # the minimum is enough (K is then not sliced; another summation order, the oracle decides)
    Ymin = tg.tstgemm(Xd, t, bd, workspace=shared[:need[0][0]])
    torch.cuda.synchronize()
    assert_close(Ymin.cpu().numpy(), problems[0][3], problems[0][4], "minimum workspace")


@pytest.mark.parametrize("forms,M,code", [(0, 4, 0), (0, 40, -7), (0, 100, -7), (2, 40, -8), (2 | 32, 40, 0),
                                          (1 | 32, 100, 0), (1 | 32, 40, -7), (4, 4, 0), (16 | 32, 4, 0)])
def test_calls_need_their_form(forms, M, code):
    """tstgemm() on a handle uploaded with a subset of the device forms: the paths whose form (or workspace) is there
    give the oracle's result, the others an error code and no launch."""
    import torch
    K, N = 300, 70
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=890 + M)
    t = tg.tcsc_upload(tg.tcsc_build(W), forms=forms)
    Xd, bd = torch.from_numpy(X).cuda(), torch.from_numpy(b).cuda()
    fn = tg.tstgemm_packed if forms & 16 else tg.tstgemm
    if code:
        with pytest.raises(tg.TstgemmError) as err:
            fn(Xd, t, bd)
        assert err.value.code == code
        return
    Y = fn(Xd, t, bd)
    torch.cuda.synchronize()
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    assert_close(Y.cpu().numpy(), Yd, A, f"forms={forms} M={M}")


def test_random_shapes_and_densities():
    """Eighty seeded random problems (M, K, N, density, with or without bias, any kernel): real inputs within the
    tolerance, integer inputs bit for bit."""
    rng = np.random.default_rng(4711)
    for case in range(80):
        M = int(rng.choice([rng.integers(1, 9), rng.integers(9, 65), rng.integers(65, 400)]))
        K = int(rng.choice([rng.integers(1, 70), rng.integers(70, 700), rng.integers(700, 5000)]))
        N = int(rng.choice([rng.integers(1, 20), rng.integers(20, 300)]))
        density = float(rng.choice([0.02, 0.125, 0.5, 0.9]))
        W, X, b = si.make_inputs(M, K, N, density, "normal", seed=5000 + case)
        if case % 4 == 0:
            b = None
        ot = oracle.tcsc_build(W)
        Yd, A, _ = oracle.tstgemm(X, ot, b)
        Y, h = gpu_tstgemm(W, X, b)
        assert_close(Y, Yd, A, f"case {case}: {M}x{K}x{N} d={density}")
        Xi = si.draw_dense(np.random.Generator(np.random.PCG64(6000 + case)), X.shape, "int8")
        Yi, _ = gpu_tstgemm(W, Xi, b, handle=h)
        assert np.array_equal(Yi, oracle.tstgemm(Xi, ot, b)[0].astype(np.float32)), f"case {case}: {M}x{K}x{N}"
        if M <= 8:
            import torch
            Xd = torch.from_numpy(Xi).cuda()
            bd = None if b is None else torch.from_numpy(b).cuda()
            for fn in (tg.tstgemm_signed, tg.tstgemm_packed):
                Yv = fn(Xd, h, bd)
                torch.cuda.synchronize()
                assert np.array_equal(Yv.cpu().numpy(), Yi), f"case {case} {fn.__name__}: {M}x{K}x{N}"


@pytest.mark.parametrize("M,K,N", [(1, 300, 70), (8, 513, 65), (3, 4096, 200), (8, 8229, 70), (1, 30000, 40),
                                   (5, 65535, 33), (2, 65536, 20), (4, 70000, 9)])
def test_decode_list_widths(M, K, N):
    """The small-M kernel on the padded 16-bit copy of the lists (K <= 65535, X whole in the LDS) and on the 32-bit TCSC
    arrays: both within tolerance of the oracle, integer inputs bit for bit; K in chunks or beyond 16 bits takes the
    32-bit arrays either way."""
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=97 + M)
    _, Xi, _ = si.make_inputs(M, K, N, 0.5, "int8", seed=98 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Ydi = oracle.tstgemm(Xi, ot, b)[0].astype(np.float32)
    Y, h = gpu_tstgemm(W, X, b)
    assert tg.tcsc_layout(h).has_lists16 == (1 if K <= 65535 else 0)
    assert_close(Y, Yd, A, f"{M}x{K}x{N}")
    assert np.array_equal(gpu_tstgemm(W, Xi, b, handle=h)[0], Ydi)
    Yw, _ = gpu_tstgemm(W, X, b, handle=h, wide_lists=True)
    Ywi, _ = gpu_tstgemm(W, Xi, b, handle=h, wide_lists=True)
    assert_close(Yw, Yd, A, f"{M}x{K}x{N}, 32-bit lists")
    assert np.array_equal(Ywi, Ydi)


@pytest.mark.parametrize("M", [1, 2])
@pytest.mark.parametrize("K,N", [(300, 9000), (300, 8192), (257, 33000), (4096, 70), (64, 11008)])
def test_decode_whole_columns_and_dealt_lists(M, K, N):
    """One or two rows of X on the 16-bit lists: the launch either gives every wavefront whole columns or deals the
    lists of a run of columns to the wavefronts of a workgroup, depending on how well whole columns fill the chip
    (on 256 compute units: 8192 and 70 columns whole, 9000, 11008 and 33000 dealt, the last with more columns per
    workgroup than it keeps sums for at a time).  PReLU and the bias go through the same epilogue in both."""
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=131 + M + N)
    _, Xi, _ = si.make_inputs(M, K, N, 0.5, "int8", seed=132 + M + N)
    W[:, 3] = 0          # an empty column
    W[:, 4] = 1          # a column without a -1 list
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = gpu_tstgemm(W, X, b)
    assert_close(Y, Yd, A, f"{M}x{K}x{N}")
    assert np.array_equal(gpu_tstgemm(W, Xi, b, handle=h)[0], oracle.tstgemm(Xi, ot, b)[0].astype(np.float32))
    alpha = np.linspace(-0.5, 1.5, N).astype(np.float32)
    Ya, _ = gpu_tstgemm(W, X, b, handle=h, alpha=alpha)
    Yp, Ap = oracle.prelu(Yd, A, alpha)
    assert_close(Ya, Yp, Ap, f"{M}x{K}x{N} PReLU")
