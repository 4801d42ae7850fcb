"""tstgemm_noalloc(): the entry point whose workspace is a static device array of the library, through the C ABI,
against tstgemm_ex() with a caller-supplied workspace of the same size (same kernels, same launch shapes: bit for
bit) and against the oracle; two calls in a row, the second with a smaller input, so that whatever the first call
left in the shared array is there when the second runs."""
import numpy as np
import pytest

import oracle
import paper_2510_06957_amd as tg
import synth_inputs as si
from gpu_util import assert_close

pytestmark = pytest.mark.gpu


def _both(W, X, b, forms):
    """(Y of tstgemm_noalloc, Y of tstgemm_ex with a workspace of the static array's size), numpy."""
    import torch
    t = tg.tcsc_upload(tg.tcsc_build(W), forms=forms)     # no workspace inside the handle
    assert tg.tcsc_layout(t).workspace_bytes == 0
    Xd, bd = torch.from_numpy(X).cuda(), torch.from_numpy(b).cuda()
    Y1 = torch.full((X.shape[0], W.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
    tg.tstgemm_noalloc(Xd, t, bd, Y1)
    torch.cuda.synchronize()
    ws = torch.empty(tg.NOALLOC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    Y2 = tg.tstgemm(Xd, t, bd, workspace=ws)
    torch.cuda.synchronize()
    return Y1.cpu().numpy(), Y2.cpu().numpy()


@pytest.mark.parametrize("first,second", [((256, 2048, 1024), (130, 700, 200)),      # large-M path, K sliced; then smaller
                                          ((64, 4096, 512), (20, 1100, 70)),         # small-tile path
                                          ((1000, 640, 384), (8, 513, 65))])         # several row tiles; then M <= 8
def test_noalloc_matches_the_workspace_entry_point(first, second):
    forms = tg.FORM_ROWSETS | tg.FORM_CUTS | tg.FORM_LISTS16
    for i, (M, K, N) in enumerate((first, second)):
        W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=990 + i + M)
        Y1, Y2 = _both(W, X, b, forms)
        assert np.array_equal(Y1.view(np.uint32), Y2.view(np.uint32)), f"{M}x{K}x{N}: differs from tstgemm_ex"
        Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
        assert_close(Y1, Yd, A, f"noalloc {M}x{K}x{N}")
        _, Xi, _ = si.make_inputs(M, K, N, 0.5, "int8", seed=991 + i + M)
        Yi, _ = _both(W, Xi, b, forms)
        assert np.array_equal(Yi, oracle.tstgemm(Xi, oracle.tcsc_build(W), b)[0].astype(np.float32)), \
            f"noalloc integer {M}x{K}x{N}"


def test_noalloc_in_slabs():
    """More row tiles than the static array holds at once (M = 3000 rows over K = 16384: 12 tiles of 16 MiB): the call
    goes through X in slabs, as tstgemm_ex() does with a workspace of that size."""
    M, K, N = 3000, 16384, 70
    W, X, b = si.make_inputs(M, K, N, 0.25, "normal", seed=995)
    Y1, Y2 = _both(W, X, b, tg.FORM_ROWSETS)
    assert np.array_equal(Y1.view(np.uint32), Y2.view(np.uint32))
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    assert_close(Y1, Yd, A, "noalloc in slabs")


def test_noalloc_under_graph_capture():
    """What the entry point is for: a stream capture records it (kernels only, nothing allocated, the array's address
    looked up by the call before the capture); every replay, with new contents of X and eager work in between, gives
    the eager result bit for bit."""
    import torch
    M, K, N = 256, 1024, 512
    W, X, b = si.make_inputs(M, K, N, 0.5, "normal", seed=997)
    t = tg.tcsc_upload(tg.tcsc_build(W), forms=tg.FORM_ROWSETS)
    Xd, bd = torch.from_numpy(X).cuda(), torch.from_numpy(b).cuda()
    Yg = torch.empty((M, N), dtype=torch.float32, device="cuda")
    Ye = torch.empty_like(Yg)
    tg.tstgemm_noalloc(Xd, t, bd, Yg)              # first call on the device: outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            tg.tstgemm_noalloc(Xd, t, bd, Yg, stream=side)
    torch.cuda.synchronize()
    rng = np.random.default_rng(998)
    for rep in range(3):
        Xn = rng.standard_normal((M, K)).astype(np.float32)
        Xd.copy_(torch.from_numpy(Xn).cuda())
        Yg.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        tg.tstgemm_noalloc(Xd, t, bd, Ye)
        torch.cuda.synchronize()
        assert torch.equal(Yg, Ye), f"replay {rep}"
        Yd, A, _ = oracle.tstgemm(Xn, oracle.tcsc_build(W), b)
        assert_close(Yg.cpu().numpy(), Yd, A, f"noalloc graph replay {rep}")


def test_noalloc_rejects_what_does_not_fit():
    """One row tile over K must fit the static array: K = 200000 at M = 100 needs 128 x 200000 x 4 bytes."""
    import torch
    K, N, M = 200000, 2, 100
    assert tg.tstgemm_workspace_bytes(M, K, N)[0] > tg.NOALLOC_SCRATCH_BYTES
    W = np.zeros((K, N), np.int8)
    W[::7, 0], W[::5, 1] = 1, -1
    t = tg.tcsc_upload(tg.tcsc_build(W), forms=tg.FORM_ROWSETS)
    Xd = torch.ones((M, K), dtype=torch.float32, device="cuda")
    Yd = torch.full((M, N), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(tg.TstgemmError) as err:
        tg.tstgemm_noalloc(Xd, t, None, Yd)
    assert err.value.code == -9 and "static" in str(err.value)
    torch.cuda.synchronize()
    assert torch.all(Yd == 7.0)                    # nothing was launched
    lib = tg.binding._load()
    assert lib.tstgemm_noalloc(Xd.data_ptr(), t.handle, None, Yd.data_ptr(), M, K + 1, N, None) == -1
    assert lib.tstgemm_noalloc(None, t.handle, None, Yd.data_ptr(), M, K, N, None) == -1
    # the same matrix with few enough rows of X for the small-tile path fits (a tile of 16 rows) -- but that path's
    # form was not uploaded: the error is the ordinary one, not a launch
    with pytest.raises(tg.TstgemmError) as err:
        tg.tstgemm_noalloc(Xd[:16].contiguous(), t, None, Yd[:16].contiguous())
    assert err.value.code == -7
