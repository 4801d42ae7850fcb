"""Helpers of the GPU parity tests: run the HIP path through its binding, compare with the oracle."""
import numpy as np

import oracle
import paper_2510_06957_amd as tg

REL_TOL = 1e-5   # |Y_gpu - Y_oracle| <= REL_TOL * (sum_k |X[m,k] W[k,n]| + |b[n]|), per element


def gpu_tstgemm(W, X, b, handle=None, alpha=None, **options):
    """Y (numpy float32) from the HIP library for host inputs; returns (Y, handle).  alpha: PReLU slopes or None;
    options: per-call options of the binding's tstgemm() (launch shape, workspace, list width)."""
    import torch
    if handle is None:
        handle = tg.tcsc_upload(tg.tcsc_build(W))
    Xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
    bd = None if b is None else torch.from_numpy(np.ascontiguousarray(b)).cuda()
    Yd = torch.full((X.shape[0], W.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
    ad = None if alpha is None else torch.from_numpy(np.ascontiguousarray(np.atleast_1d(alpha), dtype=np.float32)).cuda()
    tg.tstgemm(Xd, handle, bd, Yd, alpha=ad, **options)
    torch.cuda.synchronize()
    return Yd.cpu().numpy(), handle


def assert_close(Y, Yd, A, what=""):
    err = np.abs(Y.astype(np.float64) - Yd)
    bad = ~(err <= REL_TOL * A)
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, err / np.maximum(A, 1e-300), 0)), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} elements outside tolerance; worst at {i}: "
                             f"gpu={Y[i]!r} oracle={Yd[i]!r} bound={A[i]!r}")


def assert_exact(Y, Yd, what=""):
    expect = Yd.astype(np.float32)
    assert np.array_equal(expect.astype(np.float64), Yd), "oracle result not representable in fp32"
    bad = Y != expect
    if bad.any():
        i = np.unravel_index(np.argmax(bad), bad.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} elements differ; first at {i}: "
                             f"gpu={Y[i]!r} oracle={expect[i]!r}")


def decode_device_form(t):
    """Dense W rebuilt from the K-blocked device form (64-bit row sets), plus the four
    canonical arrays as they sit in the device buffer.  Written against the layout documented in
    include/tstgemm.h, independent of the library's own code."""
    import torch
    lay = tg.tcsc_layout(t)
    torch.cuda.synchronize()
    off0 = t.device_base - t.device_buffer.data_ptr()
    raw = t.device_buffer.cpu().numpy()[off0:off0 + lay.total_bytes]

    def view(off, count, dtype):
        return raw[off:off + count * np.dtype(dtype).itemsize].view(dtype)

    canon = (view(lay.off_col_start_pos, lay.N + 1, np.int32), view(lay.off_col_start_neg, lay.N + 1, np.int32),
             view(lay.off_row_index_pos, lay.nnz_pos, np.int32), view(lay.off_row_index_neg, lay.nnz_neg, np.int32))
    masks = view(lay.off_masks, lay.n_kblocks * lay.n_pad * 2, np.uint64).reshape(lay.n_kblocks, lay.n_pad, 2)
    assert lay.k_block == 64
    assert not masks[:, lay.N:, :].any()                      # padding columns are empty
    assert not (masks[:, :, 0] & masks[:, :, 1]).any()        # a row is +1 or -1, never both
    W = np.zeros((lay.n_kblocks * 64, lay.N), np.int8)
    for r in range(64):
        bit = np.uint64(1) << np.uint64(r)
        W[r::64][(masks[:, :lay.N, 0] & bit) != 0] = 1
        W[r::64][(masks[:, :lay.N, 1] & bit) != 0] = -1
    assert not W[lay.K:].any()                                # no row at or beyond K
    W = W[:lay.K]
    # list cuts: entry [c][n] = number of the first entry of column n's list whose row is >= 256 c (plain search here)
    assert lay.n_cuts == -(-lay.K // 256)
    cuts = view(lay.off_list_cuts, (lay.n_cuts + 1) * lay.n_pad * 2, np.int32).reshape(lay.n_cuts + 1, lay.n_pad, 2)
    assert not cuts[:, lay.N:, :].any()
    for sign, (cs, ri) in enumerate(((canon[0], canon[2]), (canon[1], canon[3]))):
        for n in range(lay.N):
            col = ri[cs[n]:cs[n + 1]]
            expect = cs[n] + np.searchsorted(col, 256 * np.arange(lay.n_cuts + 1), side="left")
            assert np.array_equal(cuts[:, n, sign], expect), (sign, n)
            assert cuts[lay.n_cuts, n, sign] == cs[n + 1]
    return W, canon
