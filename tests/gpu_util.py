"""Helpers of the GPU parity tests: run the HIP path through its binding, compare with the oracle."""
import numpy as np

import oracle
import paper_2510_06957_amd as tg

REL_TOL = 1e-5   # |Y_gpu - Y_oracle| <= REL_TOL * (sum_k |X[m,k] W[k,n]| + |b[n]|), per element


def gpu_tstgemm(W, X, b, handle=None):
    """Y (numpy float32) from the HIP library for host inputs; returns (Y, handle)."""
    import torch
    if handle is None:
        handle = tg.tcsc_upload(tg.tcsc_build(W))
    Xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
    bd = None if b is None else torch.from_numpy(np.ascontiguousarray(b)).cuda()
    Yd = torch.full((X.shape[0], W.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
    tg.tstgemm(Xd, handle, bd, Yd)
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
    """Dense W rebuilt from the K-blocked device streams (seg_count, col_ptr, stream), plus the four
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
    seg = view(lay.off_seg_count, lay.n_kblocks * lay.n_pad, np.int32).reshape(lay.n_kblocks, lay.n_pad)
    seg_ptr = view(lay.off_seg_ptr, lay.n_kblocks * lay.n_pad, np.uint32).reshape(lay.n_kblocks, lay.n_pad)
    stream = view(lay.off_stream, lay.stream_len, np.int32)
    W = np.zeros((lay.K, lay.N), np.int8)
    C = lay.chunk

    def read_list(pos, count):
        full = count // C * C
        vals = list(stream[pos:pos + full])
        r = count - full
        if r:
            ch = stream[pos + full:pos + full + C]
            if r & 4:
                vals += list(ch[0:4])
            if r & 2:
                vals += list(ch[4:6])
            if r & 1:
                vals.append(ch[6])
        return np.array(vals, dtype=np.int64), pos + (count + C - 1) // C * C

    pos = 0   # lists are stored K-block after K-block, column after column, without gaps
    for kb in range(lay.n_kblocks):
        for n in range(lay.n_pad):
            c = int(seg[kb, n])
            cp, cn = c & 0xffff, (c >> 16) & 0xffff
            assert int(seg_ptr[kb, n]) * C == pos
            if n >= lay.N:
                assert c == 0
                continue
            for count, sign in ((cp, 1), (cn, -1)):
                rows, pos = read_list(pos, count)
                assert rows.size == 0 or (rows.min() >= 0 and rows.max() < lay.k_block and np.all(np.diff(rows) > 0))
                assert np.all(W[kb * lay.k_block + rows, n] == 0)
                W[kb * lay.k_block + rows, n] = sign
    assert pos == lay.stream_len
    return W, canon
