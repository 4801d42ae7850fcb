"""ctypes binding of libtstgemm.so -- same names as the C entry points in include/tstgemm.h.

Nothing is computed here.  If the shared library has not been built the first call raises:
there is no fallback path.
"""
from __future__ import annotations

import ctypes
import pathlib

import numpy as np

_HERE = pathlib.Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libtstgemm.so"
_lib = None


class TstgemmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {tcsc_strerror(code)} (code {code})")


class TcscLayout(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("N", ctypes.c_int32), ("n_pad", ctypes.c_int32), ("k_block", ctypes.c_int32),
                ("n_kblocks", ctypes.c_int32), ("n_cuts", ctypes.c_int32),
                ("n_chunks5", ctypes.c_int32), ("has_lists16", ctypes.c_int32),
                ("nnz_pos", ctypes.c_int64), ("nnz_neg", ctypes.c_int64),
                ("nnz16_pos", ctypes.c_int64), ("nnz16_neg", ctypes.c_int64),
                ("off_col_start_pos", ctypes.c_size_t), ("off_col_start_neg", ctypes.c_size_t),
                ("off_row_index_pos", ctypes.c_size_t), ("off_row_index_neg", ctypes.c_size_t),
                ("off_masks", ctypes.c_size_t), ("off_list_cuts", ctypes.c_size_t),
                ("off_col_start16_pos", ctypes.c_size_t), ("off_col_start16_neg", ctypes.c_size_t),
                ("off_row_index16_pos", ctypes.c_size_t), ("off_row_index16_neg", ctypes.c_size_t),
                ("off_signed_index", ctypes.c_size_t), ("off_packed", ctypes.c_size_t), ("off_workspace", ctypes.c_size_t),
                ("workspace_bytes", ctypes.c_size_t), ("total_bytes", ctypes.c_size_t), ("forms", ctypes.c_uint32)]


class TstgemmOpts(ctypes.Structure):
    """tstgemm_opts_t of include/tstgemm.h."""
    _fields_ = [("struct_size", ctypes.c_size_t), ("encoding", ctypes.c_int), ("alpha_count", ctypes.c_int),
                ("alpha", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("cols_per_wave", ctypes.c_int), ("k_slices", ctypes.c_int), ("slab_tiles", ctypes.c_int),
                ("list_walk", ctypes.c_int), ("decode_wide_lists", ctypes.c_int), ("event_before", ctypes.c_void_p), ("event_after", ctypes.c_void_p)]


# TCSC_FORM_* of include/tstgemm.h
FORM_ROWSETS, FORM_CUTS, FORM_LISTS16, FORM_SIGNED, FORM_PACKED, FORM_WORKSPACE, FORM_ALL = 1, 2, 4, 8, 16, 32, 63


def library_path() -> pathlib.Path:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2510_06957_amd.build` "
                           "(there is no fallback implementation)")
    # PyTorch ships its own copy of the HIP runtime.  Device pointers and streams are only valid inside the
    # runtime that created them, so torch must be in the process first: the loader then resolves this library's
    # libamdhip64 dependency to the copy torch already mapped instead of opening a second runtime.
    import torch  # noqa: F401
    lib = ctypes.CDLL(str(_LIB_PATH))
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.tcsc_build.argtypes = [vp, ci, ci, ctypes.POINTER(vp)]
    lib.tcsc_from_arrays.argtypes = [vp, vp, vp, vp, ci, ci, ctypes.POINTER(vp)]
    lib.tcsc_to_dense.argtypes = [vp, vp]
    lib.tcsc_dims.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_int64),
                              ctypes.POINTER(ctypes.c_int64)]
    lib.tcsc_arrays.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp)]
    lib.tcsc_device_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
    lib.tcsc_layout.argtypes = [vp, ctypes.POINTER(TcscLayout)]
    lib.tcsc_upload.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.tstgemm.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
    lib.tstgemm_prelu.argtypes = [vp, vp, vp, vp, ci, vp, ci, ci, ci, vp]
    lib.tstgemm_signed.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
    lib.tstgemm_packed.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
    lib.tcsc_signed_arrays.argtypes = [vp, vp, vp]
    lib.tcsc_packed_codes.argtypes = [vp, vp]
    lib.tcsc_destroy.argtypes = [vp]
    lib.tcsc_destroy.restype = None
    lib.tcsc_strerror.argtypes = [ci]
    lib.tcsc_strerror.restype = ctypes.c_char_p
    lib.tstgemm_noalloc.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
    lib.tstgemm_ex.argtypes = [vp, vp, vp, vp, ci, ci, ci, ctypes.POINTER(TstgemmOpts), vp]
    lib.tstgemm_workspace_bytes.argtypes = [ci, ci, ci, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
    lib.tcsc_select_forms.argtypes = [vp, ctypes.c_uint32]
    lib.tstgemm_probe_lds_read.argtypes = [ci, ctypes.POINTER(ctypes.c_int64), vp]
    lib.tstgemm_probe_lds_read.restype = ci
    lib.tstgemm_probe_stream_read.argtypes = [vp, ctypes.c_size_t, vp]
    lib.tstgemm_probe_stream_read.restype = ci
    lib.tstgemm_probe_tile_copy.argtypes = [vp, ctypes.c_size_t, ci, ctypes.POINTER(ctypes.c_int64), vp]
    lib.tstgemm_probe_tile_copy.restype = ci
    for name in ("tcsc_build", "tcsc_from_arrays", "tcsc_to_dense", "tcsc_dims", "tcsc_arrays", "tcsc_device_bytes",
                 "tcsc_layout", "tcsc_upload", "tstgemm", "tstgemm_prelu", "tstgemm_signed", "tstgemm_packed",
                 "tcsc_signed_arrays", "tcsc_packed_codes", "tstgemm_ex", "tstgemm_workspace_bytes", "tcsc_select_forms",
                 "tstgemm_noalloc"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def tcsc_strerror(code: int) -> str:
    return _load().tcsc_strerror(int(code)).decode()


def _check(code: int, where: str):
    if code != 0:
        raise TstgemmError(code, where)


def _np_ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


class Tcsc:
    """Owner of a tcsc_t handle (and, once uploaded, of the torch tensor backing its device form)."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)
        self.device_buffer = None
        self.K, self.N, self.nnz_pos, self.nnz_neg = tcsc_dims(self)

    @property
    def nnz(self) -> int:
        return self.nnz_pos + self.nnz_neg

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("tcsc handle already destroyed")
        return self._h

    def __del__(self):
        try:
            tcsc_destroy(self)
        except Exception:
            pass


def tcsc_build(W: np.ndarray) -> Tcsc:
    """TCSC handle from a dense ternary matrix (host, K x N, values in {-1,0,+1})."""
    W = np.ascontiguousarray(W, dtype=np.int8)
    if W.ndim != 2:
        raise ValueError("W must be a K x N matrix")
    out = ctypes.c_void_p()
    _check(_load().tcsc_build(_np_ptr(W), W.shape[0], W.shape[1], ctypes.byref(out)), "tcsc_build")
    return Tcsc(out.value)


def tcsc_from_arrays(col_start_pos, col_start_neg, row_index_pos, row_index_neg, K: int, N: int) -> Tcsc:
    arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in (col_start_pos, col_start_neg, row_index_pos,
                                                               row_index_neg)]
    if arrs[0].size != N + 1 or arrs[1].size != N + 1:
        raise ValueError("col_start arrays need N + 1 entries")
    if arrs[0].size and (arrs[2].size < arrs[0][-1] or arrs[3].size < arrs[1][-1]):
        raise ValueError("row_index arrays shorter than col_start[N]")
    out = ctypes.c_void_p()
    _check(_load().tcsc_from_arrays(*[_np_ptr(a) for a in arrs], int(K), int(N), ctypes.byref(out)),
           "tcsc_from_arrays")
    return Tcsc(out.value)


def tcsc_to_dense(t: Tcsc) -> np.ndarray:
    W = np.empty((t.K, t.N), np.int8)
    _check(_load().tcsc_to_dense(t.handle, _np_ptr(W)), "tcsc_to_dense")
    return W


def tcsc_dims(t: Tcsc):
    K, N = ctypes.c_int(), ctypes.c_int()
    p, q = ctypes.c_int64(), ctypes.c_int64()
    _check(_load().tcsc_dims(t.handle, ctypes.byref(K), ctypes.byref(N), ctypes.byref(p), ctypes.byref(q)),
           "tcsc_dims")
    return K.value, N.value, p.value, q.value


def tcsc_arrays(t: Tcsc):
    """Copies of the handle's four host arrays (col_start_pos, col_start_neg, row_index_pos, row_index_neg)."""
    ptrs = [ctypes.c_void_p() for _ in range(4)]
    _check(_load().tcsc_arrays(t.handle, *[ctypes.byref(p) for p in ptrs]), "tcsc_arrays")
    sizes = [t.N + 1, t.N + 1, t.nnz_pos, t.nnz_neg]
    out = []
    for p, n in zip(ptrs, sizes):
        if n == 0:
            out.append(np.empty(0, np.int32))
        else:
            out.append(np.ctypeslib.as_array(ctypes.cast(p, ctypes.POINTER(ctypes.c_int32)), shape=(n,)).copy())
    return tuple(out)


def tcsc_device_bytes(t: Tcsc) -> int:
    n = ctypes.c_size_t()
    _check(_load().tcsc_device_bytes(t.handle, ctypes.byref(n)), "tcsc_device_bytes")
    return n.value


def tcsc_layout(t: Tcsc) -> TcscLayout:
    lay = TcscLayout()
    _check(_load().tcsc_layout(t.handle, ctypes.byref(lay)), "tcsc_layout")
    return lay


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def tcsc_select_forms(t: Tcsc, forms: int):
    """Which device forms the next tcsc_upload() builds (FORM_* bits; a new handle has FORM_ALL)."""
    _check(_load().tcsc_select_forms(t.handle, int(forms)), "tcsc_select_forms")


def tstgemm_workspace_bytes(M: int, K: int, N: int):
    """(min_bytes, best_bytes) of scratch memory for a call with these dimensions."""
    lo, hi = ctypes.c_size_t(), ctypes.c_size_t()
    _check(_load().tstgemm_workspace_bytes(int(M), int(K), int(N), ctypes.byref(lo), ctypes.byref(hi)),
           "tstgemm_workspace_bytes")
    return lo.value, hi.value


def tcsc_upload(t: Tcsc, device="cuda:0", stream=None, forms=None) -> Tcsc:
    """Allocate the device buffer with torch and run the upload + GPU re-blocking pass into it.  forms: FORM_* bits
    to select first (None: leave the handle's choice, all forms for a new handle)."""
    import torch
    dev = torch.device(device)
    if forms is not None:
        tcsc_select_forms(t, forms)
    with torch.cuda.device(dev):
        buf = torch.empty(tcsc_device_bytes(t) + 256, dtype=torch.uint8, device=dev)
        base = (buf.data_ptr() + 255) // 256 * 256
        _check(_load().tcsc_upload(t.handle, base, tcsc_device_bytes(t), _stream_ptr(stream)), "tcsc_upload")
    t.device_buffer = buf
    t.device_base = base
    t.device_index = buf.device.index
    return t


def _gemm_args(X, t: Tcsc, b, Y):
    """Checks shared by the tstgemm* wrappers; returns (M, K, N, b_ptr, Y)."""
    import torch
    f32 = torch.float32
    if not (X.is_cuda and X.dtype == f32 and X.dim() == 2 and X.is_contiguous()):
        raise ValueError("X must be a contiguous float32 CUDA matrix")
    M, K = X.shape
    N = t.N
    dev = X.device.index
    if dev != getattr(t, "device_index", dev) or dev != torch.cuda.current_device():
        raise ValueError("X, the uploaded handle and the current device must be the same GPU")
    if b is None:
        b_ptr = None
    elif b.is_cuda and b.dtype == f32 and b.is_contiguous() and b.numel() == N and b.device.index == dev:
        b_ptr = b.data_ptr()
    else:
        raise ValueError("b must be a contiguous float32 CUDA vector of length N on X's device")
    if Y is None:
        Y = torch.empty((M, N), dtype=f32, device=X.device)
    elif not (Y.is_cuda and Y.dtype == f32 and Y.dim() == 2 and Y.shape[0] == M and Y.shape[1] == N
              and Y.is_contiguous() and Y.device.index == dev):
        raise ValueError("Y must be a contiguous float32 CUDA matrix of shape [M, N] on X's device")
    return M, K, N, b_ptr, Y


def _opts(X, N, encoding=0, alpha=None, workspace=None, cols_per_wave=0, k_slices=0, slab_tiles=0, wide_lists=False,
          events=None, list_walk=0):
    """tstgemm_opts_t from keyword arguments, or None when every one has its default (argument marshalling only).
    workspace: a CUDA tensor on X's device; events: a pair of torch.cuda.Event(enable_timing=True) objects that have
    been recorded once (so that their native handles exist)."""
    import torch
    if (encoding == 0 and alpha is None and workspace is None and not cols_per_wave and not k_slices and not slab_tiles
            and not wide_lists and events is None and not list_walk):
        return None
    o = TstgemmOpts()
    o.struct_size = ctypes.sizeof(TstgemmOpts)
    o.encoding = encoding
    if alpha is not None:
        if not (alpha.is_cuda and alpha.dtype == torch.float32 and alpha.is_contiguous() and alpha.numel() in (1, N)
                and alpha.device.index == X.device.index):
            raise ValueError("alpha must be a contiguous float32 CUDA tensor with 1 or N entries on X's device")
        o.alpha, o.alpha_count = alpha.data_ptr(), alpha.numel()
    if workspace is not None:
        if not (workspace.is_cuda and workspace.is_contiguous() and workspace.device.index == X.device.index):
            raise ValueError("workspace must be a contiguous CUDA tensor on X's device")
        o.workspace, o.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    o.cols_per_wave, o.k_slices, o.slab_tiles = int(cols_per_wave), int(k_slices), int(slab_tiles)
    o.list_walk = int(list_walk)
    o.decode_wide_lists = int(bool(wide_lists))
    if events is not None:
        o.event_before, o.event_after = events[0].cuda_event, events[1].cuda_event
    return o


def tstgemm(X, t: Tcsc, b=None, Y=None, stream=None, alpha=None, **options):
    """Y = X W + b on the GPU, or Y = PReLU(X W + b) when `alpha` is given (tstgemm_prelu of the C ABI).
    X: cuda float32 [M, K] contiguous; b: cuda float32 [N] or None; alpha: cuda float32 with 1 or N entries.
    options (tstgemm_ex of the C ABI): workspace=, cols_per_wave=, k_slices=, slab_tiles=, list_walk=, wide_lists=, events=.

    Launches on `stream` (default: torch's current stream) of the current device, which must be the device the
    handle was uploaded to and the one holding X, b, alpha and Y."""
    M, K, N, b_ptr, Y = _gemm_args(X, t, b, Y)
    o = _opts(X, N, 0, alpha, **options)
    if o is None:
        rc = _load().tstgemm(X.data_ptr(), t.handle, b_ptr, Y.data_ptr(), M, K, N, _stream_ptr(stream))
    elif not options:
        rc = _load().tstgemm_prelu(X.data_ptr(), t.handle, b_ptr, o.alpha, o.alpha_count, Y.data_ptr(), M, K, N,
                                   _stream_ptr(stream))
    else:
        rc = _load().tstgemm_ex(X.data_ptr(), t.handle, b_ptr, Y.data_ptr(), M, K, N, ctypes.byref(o), _stream_ptr(stream))
    if rc != 0:
        raise TstgemmError(rc, "tstgemm")
    return Y


def _variant(name, encoding, X, t, b, Y, stream, options):
    M, K, N, b_ptr, Y = _gemm_args(X, t, b, Y)
    if options:
        o = _opts(X, N, encoding, None, **options)
        rc = _load().tstgemm_ex(X.data_ptr(), t.handle, b_ptr, Y.data_ptr(), M, K, N, ctypes.byref(o), _stream_ptr(stream))
    else:
        rc = getattr(_load(), name)(X.data_ptr(), t.handle, b_ptr, Y.data_ptr(), M, K, N, _stream_ptr(stream))
    if rc != 0:
        raise TstgemmError(rc, name)
    return Y


NOALLOC_SCRATCH_BYTES = 64 << 20   # TSTGEMM_NOALLOC_SCRATCH_BYTES of include/tstgemm.h


def tstgemm_noalloc(X, t: Tcsc, b, Y, stream=None):
    """Y = X W + b through the library's static scratch buffer (tstgemm_noalloc of the C ABI).  Y must be given: this
    wrapper allocates nothing either."""
    if Y is None:
        raise ValueError("tstgemm_noalloc needs an output tensor")
    M, K, N, b_ptr, Y = _gemm_args(X, t, b, Y)
    rc = _load().tstgemm_noalloc(X.data_ptr(), t.handle, b_ptr, Y.data_ptr(), M, K, N, _stream_ptr(stream))
    if rc != 0:
        raise TstgemmError(rc, "tstgemm_noalloc")
    return Y


def tstgemm_signed(X, t: Tcsc, b=None, Y=None, stream=None, **options):
    """Y = X W + b for M <= 8 from the inverted-index form of the uploaded matrix (tstgemm_signed of the C ABI)."""
    return _variant("tstgemm_signed", 1, X, t, b, Y, stream, options)


def tstgemm_packed(X, t: Tcsc, b=None, Y=None, stream=None, **options):
    """Y = X W + b for M <= 8 from the value-compression form of the uploaded matrix (tstgemm_packed of the C ABI);
    X must be finite."""
    return _variant("tstgemm_packed", 2, X, t, b, Y, stream, options)


def tcsc_signed_arrays(t: Tcsc):
    """(col_start, index) of the inverted-index encoding: int32 arrays of N + 1 and nnz entries (host)."""
    col_start = np.empty(t.N + 1, np.int32)
    index = np.empty(max(t.nnz, 1), np.int32)
    _check(_load().tcsc_signed_arrays(t.handle, _np_ptr(col_start), _np_ptr(index)), "tcsc_signed_arrays")
    return col_start, index[:t.nnz]


def tcsc_packed_codes(t: Tcsc) -> np.ndarray:
    """The value-compression encoding: uint8 [N, ceil(K / 5)] (host)."""
    codes = np.empty((t.N, (t.K + 4) // 5), np.uint8)
    _check(_load().tcsc_packed_codes(t.handle, _np_ptr(codes)), "tcsc_packed_codes")
    return codes


def tstgemm_probe_lds_read(iters: int, stream=None) -> int:
    """Enqueue the LDS-read probe kernel; returns the bytes its wavefronts read together."""
    n = ctypes.c_int64()
    _check(_load().tstgemm_probe_lds_read(int(iters), ctypes.byref(n), _stream_ptr(stream)), "tstgemm_probe_lds_read")
    return n.value


def tstgemm_probe_stream_read(buf, stream=None) -> int:
    """Enqueue the streaming-read probe kernel over a CUDA tensor; returns the bytes it reads."""
    nbytes = buf.numel() * buf.element_size()
    _check(_load().tstgemm_probe_stream_read(buf.data_ptr(), nbytes, _stream_ptr(stream)), "tstgemm_probe_stream_read")
    return nbytes // 16 * 16


def tstgemm_probe_tile_copy(buf, iters: int, stream=None) -> int:
    """Enqueue the tile-copy probe kernel over a CUDA tensor (at least 64 KiB); returns the bytes its workgroups copy
    into their LDS together."""
    n = ctypes.c_int64()
    nbytes = buf.numel() * buf.element_size()
    _check(_load().tstgemm_probe_tile_copy(buf.data_ptr(), nbytes, int(iters), ctypes.byref(n), _stream_ptr(stream)),
           "tstgemm_probe_tile_copy")
    return n.value


def tcsc_destroy(t: Tcsc):
    if getattr(t, "_h", None) is not None:
        _load().tcsc_destroy(t._h)
        t._h = None
        t.device_buffer = None
