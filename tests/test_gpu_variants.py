"""GPU parity of the two small-M variants that read the paper's other encodings of W (Sec. 3): tstgemm_signed
(inverted index) and tstgemm_packed (value compression), through the C ABI binding, against the oracle's
routines for those encodings; the device forms themselves are compared bit for bit."""
import numpy as np
import pytest

import oracle
import paper_2510_06957_amd as tg
import synth_inputs as si
from gpu_util import assert_close, assert_exact

pytestmark = pytest.mark.gpu


def run(fn, W, X, b, handle=None, **options):
    import torch
    if handle is None:
        handle = tg.tcsc_upload(tg.tcsc_build(W))
    Xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
    bd = None if b is None else torch.from_numpy(np.ascontiguousarray(b)).cuda()
    Yd = torch.full((X.shape[0], W.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
    fn(Xd, handle, bd, Yd, **options)
    torch.cuda.synchronize()
    return Yd.cpu().numpy(), handle


def device_section(t, off, count, dtype):
    import torch
    torch.cuda.synchronize()
    off0 = t.device_base - t.device_buffer.data_ptr()
    raw = t.device_buffer.cpu().numpy()
    start = off0 + off
    return raw[start:start + count * np.dtype(dtype).itemsize].view(dtype)


@pytest.mark.parametrize("K,N,density", [(37, 5, 0.5), (513, 65, 0.5), (512, 512, 0.5), (1000, 130, 0.0625),
                                         (64, 9, 1.0), (130, 70, 0.0), (81, 3, 1.0), (2049, 20, 0.25)])
def test_device_forms_match_the_oracle(K, N, density):
    W, _, _ = si.make_inputs(1, K, N, density, "uniform", seed=400 + K + N)
    t = tg.tcsc_upload(tg.tcsc_build(W))
    lay = tg.tcsc_layout(t)
    ot = oracle.tcsc_build(W)
    _, oidx = oracle.signed_build(ot)
    assert np.array_equal(device_section(t, lay.off_signed_index, lay.nnz_pos + lay.nnz_neg, np.int32), oidx)
    # padded 16-bit lists: column n's list at [col_start16[n], col_start16[n + 1]), a multiple of 8 long, the pad is K
    assert lay.has_lists16 == 1
    for cs, ri, off_cs, off_ri, nnz16 in ((ot.col_start_pos, ot.row_index_pos, lay.off_col_start16_pos, lay.off_row_index16_pos, lay.nnz16_pos),
                                          (ot.col_start_neg, ot.row_index_neg, lay.off_col_start16_neg, lay.off_row_index16_neg, lay.nnz16_neg)):
        cs16 = device_section(t, off_cs, N + 1, np.int32)
        ri16 = device_section(t, off_ri, nnz16, np.uint16)
        assert cs16[0] == 0 and cs16[N] == nnz16 and not (cs16 % 8).any()
        for n in range(N):
            col = ri[cs[n]:cs[n + 1]]
            got = ri16[cs16[n]:cs16[n + 1]]
            assert got.size == -(-col.size // 8) * 8
            # the order inside a list is the library's (chosen for the LDS banks): the same rows, each once, and the pad
            assert np.array_equal(np.sort(got[got != K]), col) and np.count_nonzero(got == K) == got.size - col.size
    # packed[chunk][column][16]: group g of column n is byte [g // 16][n][g % 16]; padding groups and columns are 0
    dev = device_section(t, lay.off_packed, lay.n_chunks5 * lay.n_pad * 16, np.uint8).reshape(lay.n_chunks5, lay.n_pad, 16)
    codes = oracle.pack5(W)                                       # [N][G]
    G = codes.shape[1]
    assert lay.n_chunks5 == -(-G // 16)
    expect = np.zeros((lay.n_pad, lay.n_chunks5 * 16), np.uint8)
    expect[:N, :G] = codes
    assert np.array_equal(dev.transpose(1, 0, 2).reshape(lay.n_pad, -1), expect)


SHAPES = [(1, 1, 1), (3, 37, 5), (2, 513, 65), (8, 64, 1), (5, 130, 9), (8, 700, 96), (7, 1000, 200), (4, 81, 130),
          (1, 4096, 300), (8, 4100, 70)]


@pytest.mark.parametrize("M,K,N", SHAPES)
@pytest.mark.parametrize("variant", ["signed", "packed"])
def test_variant_parity(variant, M, K, N):
    fn = tg.tstgemm_signed if variant == "signed" else tg.tstgemm_packed
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=500 + M + K + N)
    ot = oracle.tcsc_build(W)
    if variant == "signed":
        Yd, A = oracle.tstgemm_signed(X, *oracle.signed_build(ot), b, K)
    else:
        Yd, A = oracle.tstgemm_packed(X, oracle.pack5(W), b, K)
    Y, h = run(fn, W, X, b)
    assert_close(Y, Yd, A, f"{variant} {M}x{K}x{N}")
    # integer inputs: exact in any order, and the bias is added once, last
    _, Xi, _ = si.make_inputs(M, K, N, 0.5, "int8", seed=501 + M)
    Ydi, _, _ = oracle.tstgemm(Xi, ot, b)
    Yi, _ = run(fn, W, Xi, b, handle=h)
    assert np.array_equal(Yi, Ydi.astype(np.float32))
    Y0, _ = run(fn, W, Xi, None, handle=h)
    assert_exact(Y0, oracle.tstgemm(Xi, ot, None)[0], f"{variant} no bias")


@pytest.mark.parametrize("variant", ["signed", "packed"])
@pytest.mark.parametrize("M,K,N,density", [(8, 8229, 70, 0.5), (5, 20000, 33, 0.25), (1, 40001, 20, 0.5),
                                           (2, 30000, 40, 0.0625), (8, 3041, 9000, 0.5), (3, 500, 16500, 0.25)])
def test_variant_long_k_and_wide_n(variant, M, K, N, density):
    """K beyond what the LDS holds of X (chunks of the decode kernel, segments of the packed kernel) and N wide enough
    for every columns-per-workgroup choice of the packed kernel."""
    fn = tg.tstgemm_signed if variant == "signed" else tg.tstgemm_packed
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=520 + M + N)
    _, Xi, _ = si.make_inputs(M, K, N, density, "int8", seed=521 + M)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = run(fn, W, X, b)
    assert_close(Y, Yd, A, f"{variant} {M}x{K}x{N}")
    Yi, _ = run(fn, W, Xi, b, handle=h)
    assert np.array_equal(Yi, oracle.tstgemm(Xi, ot, b)[0].astype(np.float32))


@pytest.mark.parametrize("k_parts", [0, 1, 2, 3, 8])
@pytest.mark.parametrize("M,K,N", [(8, 4100, 70), (2, 6000, 200), (5, 1300, 64)])
def test_packed_k_parts(k_parts, M, K, N):
    """The packed kernel with K dealt to several workgroups per column group (sums combined by the reduction kernel)
    and without, also where K is too short for the number of parts asked for."""
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=560 + M)
    _, Xi, _ = si.make_inputs(M, K, N, 0.5, "int8", seed=561 + M)
    ot = oracle.tcsc_build(W)
    Yd, A = oracle.tstgemm_packed(X, oracle.pack5(W), b, K)
    Y, h = run(tg.tstgemm_packed, W, X, b, k_slices=k_parts)
    assert_close(Y, Yd, A, f"k_parts={k_parts}")
    Yi, _ = run(tg.tstgemm_packed, W, Xi, b, handle=h, k_slices=k_parts)
    assert np.array_equal(Yi, oracle.tstgemm(Xi, ot, b)[0].astype(np.float32))


def test_lists16_order_spreads_rows_over_the_bank_groups():
    """The padded 16-bit lists are stored so that the sixteen lanes that gather together (lanes 16 j .. 16 j + 15 of a
    round of 512 entries, same slot of their 8) get rows that differ modulo 16: on a benchmark-sized random column most
    whole groups must be free of repeats (a class of rows with fewer members than there are groups leaves holes that other
    classes fill: about one group in eight has one repeat; in ascending order about one group in a thousand has none)."""
    K, N = 4096, 24
    W, _, _ = si.make_inputs(1, K, N, 0.5, "uniform", seed=470)
    t = tg.tcsc_upload(tg.tcsc_build(W))
    lay = tg.tcsc_layout(t)
    cs16 = device_section(t, lay.off_col_start16_pos, N + 1, np.int32)
    ri16 = device_section(t, lay.off_row_index16_pos, lay.nnz16_pos, np.uint16)
    whole = clean = 0
    for n in range(N):
        col = ri16[cs16[n]:cs16[n + 1]].astype(np.int64)
        for r in range(col.size // 512):
            rnd = col[r * 512:(r + 1) * 512].reshape(64, 8)            # [lane][slot]
            for j in range(4):
                for e in range(8):
                    rows = rnd[16 * j:16 * j + 16, e]
                    whole += 1
                    clean += np.unique(rows % 16).size == 16 and not (rows == K).any()
    assert whole >= N * 8 and clean >= 0.8 * whole, (clean, whole)


def test_variant_degenerate_matrices():
    K, N, M = 150, 40, 3
    _, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=530)
    for fn in (tg.tstgemm_signed, tg.tstgemm_packed):
        Y, h = run(fn, np.zeros((K, N), np.int8), X, b)
        assert np.array_equal(Y, np.broadcast_to(b, Y.shape))
        ones = np.ones((K, N), np.int8)
        Xi = si.make_inputs(M, K, N, 0.5, "int8", seed=531)[1]
        Y1, _ = run(fn, ones, Xi, None)
        assert np.array_equal(Y1, np.broadcast_to(Xi.sum(axis=1, keepdims=True), Y1.shape))
        Ym, _ = run(fn, -ones, Xi, None)
        assert np.array_equal(Ym, -Y1)


def test_signed_never_reads_zero_weight_entries():
    """The inverted-index path is still a gather: X entries under zero weights do not reach Y.  (The packed path
    multiplies every entry and documents that X must be finite.)"""
    M, K, N = 4, 300, 50
    W, X, b = si.make_inputs(M, K, N, 0.25, "normal", seed=540)
    W[::7] = 0                           # rows no column uses
    unused = ~W.any(axis=1)
    assert unused.any()
    Xn = X.copy()
    Xn[:, unused] = np.nan
    Y, h = run(tg.tstgemm_signed, W, X, b)
    Yn, _ = run(tg.tstgemm_signed, W, Xn, b, handle=h)
    assert np.array_equal(Y, Yn)


@pytest.mark.parametrize("name", ["C4-1", "C4-8"])
@pytest.mark.parametrize("variant", ["signed", "packed"])
def test_variant_decode_configs_full(variant, name):
    fn = tg.tstgemm_signed if variant == "signed" else tg.tstgemm_packed
    W, X, b = si.make_workload(name)
    ot = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, ot, b)
    Y, h = run(fn, W, X, b)
    assert_close(Y, Yd, A, f"{variant} {name}")
    Y2, _ = run(fn, W, X, b, handle=h)
    assert np.array_equal(Y, Y2)          # repeatable


def test_variants_reject_large_m():
    import torch
    W, X, b = si.make_inputs(9, 64, 8, 0.5, "normal", seed=550)
    t = tg.tcsc_upload(tg.tcsc_build(W))
    for fn in (tg.tstgemm_signed, tg.tstgemm_packed):
        with pytest.raises(tg.TstgemmError):
            fn(torch.from_numpy(X).cuda(), t)
