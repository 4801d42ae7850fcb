"""CPU oracle for the sparse ternary GEMM Y = X W + b -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around oracle/tstgemm_oracle.c and oracle/variants_oracle.c (see those files
for what they follow in the paper).  Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product package never does.  It imports nothing from the product package.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(str(path))
        lib.oracle_tstgemm_rows.restype = ctypes.c_int
        lib.oracle_tstgemm_points.restype = ctypes.c_int
        lib.oracle_tcsc_build.restype = ctypes.c_int
        lib.oracle_tcsc_count.restype = ctypes.c_int
        lib.oracle_tcsc_to_dense.restype = ctypes.c_int
        lib.oracle_prelu.restype = ctypes.c_int
        for name in ("oracle_signed_build", "oracle_signed_to_dense", "oracle_tstgemm_signed", "oracle_pack5",
                     "oracle_unpack5", "oracle_tstgemm_packed"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class Tcsc:
    """The four TCSC arrays of Sec. 2 (int32, 0-based) plus the shape of W."""
    col_start_pos: np.ndarray
    col_start_neg: np.ndarray
    row_index_pos: np.ndarray
    row_index_neg: np.ndarray
    K: int
    N: int

    @property
    def nnz(self) -> int:
        return int(self.row_index_pos.size + self.row_index_neg.size)

    def negated(self) -> "Tcsc":
        """TCSC of -W: the two sign lists trade places."""
        return Tcsc(self.col_start_neg, self.col_start_pos, self.row_index_neg, self.row_index_pos, self.K, self.N)


def tcsc_build(W: np.ndarray) -> Tcsc:
    W = np.ascontiguousarray(W, dtype=np.int8)
    K, N = W.shape
    lib = _load()
    p, q = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = lib.oracle_tcsc_count(_p(W), K, N, ctypes.byref(p), ctypes.byref(q))
    if rc:
        raise ValueError(f"oracle_tcsc_count failed ({rc}): W must hold only -1, 0, +1")
    csp = np.empty(N + 1, np.int32)
    csn = np.empty(N + 1, np.int32)
    rip = np.empty(p.value, np.int32)
    rin = np.empty(q.value, np.int32)
    rc = lib.oracle_tcsc_build(_p(W), K, N, _p(csp), _p(csn), _p(rip), _p(rin))
    if rc:
        raise ValueError(f"oracle_tcsc_build failed ({rc})")
    return Tcsc(csp, csn, rip, rin, K, N)


def tcsc_to_dense(t: Tcsc) -> np.ndarray:
    W = np.empty((t.K, t.N), np.int8)
    rc = _load().oracle_tcsc_to_dense(_p(t.col_start_pos), _p(t.col_start_neg), _p(t.row_index_pos),
                                      _p(t.row_index_neg), t.K, t.N, _p(W))
    if rc:
        raise ValueError(f"oracle_tcsc_to_dense failed ({rc})")
    return W


def tstgemm(X: np.ndarray, t: Tcsc, b: np.ndarray | None, rows=None, threads: int = 0):
    """(Yd, A, threads_used): all rows of Y, or the rows listed in `rows`, in float64."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    M, K = X.shape
    if K != t.K:
        raise ValueError("X has the wrong number of columns")
    if b is not None:
        b = np.ascontiguousarray(b, dtype=np.float32)
        if b.shape != (t.N,):
            raise ValueError("b has the wrong length")
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        if rows.size and (rows.min() < 0 or rows.max() >= M):
            raise ValueError("row out of range")
    n_rows = M if rows is None else int(rows.size)
    Yd = np.empty((n_rows, t.N), np.float64)
    A = np.empty((n_rows, t.N), np.float64)
    used = _load().oracle_tstgemm_rows(_p(X), _p(t.col_start_pos), _p(t.col_start_neg), _p(t.row_index_pos),
                                       _p(t.row_index_neg), _p(b), _p(rows), n_rows, M, K, t.N, _p(Yd), _p(A),
                                       int(threads))
    if used < 0:
        raise ValueError(f"oracle_tstgemm_rows failed ({used})")
    return Yd, A, used


def tstgemm_points(X: np.ndarray, t: Tcsc, b: np.ndarray | None, ms, ns):
    """(Yd, A) for the sampled elements (ms[i], ns[i])."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    M, K = X.shape
    if K != t.K:
        raise ValueError("X has the wrong number of columns")
    if b is not None:
        b = np.ascontiguousarray(b, dtype=np.float32)
    ms = np.ascontiguousarray(ms, dtype=np.int32)
    ns = np.ascontiguousarray(ns, dtype=np.int32)
    Yd = np.empty(ms.size, np.float64)
    A = np.empty(ms.size, np.float64)
    rc = _load().oracle_tstgemm_points(_p(X), _p(t.col_start_pos), _p(t.col_start_neg), _p(t.row_index_pos),
                                       _p(t.row_index_neg), _p(b), _p(ms), _p(ns), ctypes.c_int64(ms.size),
                                       M, K, t.N, _p(Yd), _p(A))
    if rc:
        raise ValueError(f"oracle_tstgemm_points failed ({rc})")
    return Yd, A


def prelu(Yd: np.ndarray, A: np.ndarray | None, alpha) -> tuple[np.ndarray, np.ndarray | None]:
    """PReLU of a finished Y (rows x N, float64): copies of (Yd, A) with v <= 0 replaced by alpha * v and the
    tolerance scale multiplied by max(1, |alpha|).  alpha: one slope, or one per column."""
    Yd = np.array(Yd, dtype=np.float64, order="C", copy=True)
    if Yd.ndim != 2:
        raise ValueError("Yd must be a matrix")
    A = None if A is None else np.array(A, dtype=np.float64, order="C", copy=True)
    alpha = np.ascontiguousarray(np.atleast_1d(alpha), dtype=np.float32)
    if alpha.size not in (1, Yd.shape[1]):
        raise ValueError("alpha must have 1 or N entries")
    rc = _load().oracle_prelu(_p(Yd), _p(A), Yd.shape[0], Yd.shape[1], _p(alpha), int(alpha.size))
    if rc:
        raise ValueError(f"oracle_prelu failed ({rc})")
    return Yd, A


# ---------------------------------------------------------------------------------------------------------------
# The two alternative encodings of W (Sec. 3, "Inverted Index" and "Value Compression"); see variants_oracle.c.

def signed_build(t: Tcsc) -> tuple[np.ndarray, np.ndarray]:
    """(col_start, index): the two lists of every column merged, +1 in row i stored as i, -1 as ~i."""
    col_start = np.empty(t.N + 1, np.int32)
    index = np.empty(t.nnz, np.int32)
    rc = _load().oracle_signed_build(_p(t.col_start_pos), _p(t.col_start_neg), _p(t.row_index_pos),
                                     _p(t.row_index_neg), t.N, _p(col_start), _p(index))
    if rc:
        raise ValueError(f"oracle_signed_build failed ({rc})")
    return col_start, index


def signed_to_dense(col_start: np.ndarray, index: np.ndarray, K: int) -> np.ndarray:
    col_start = np.ascontiguousarray(col_start, dtype=np.int32)
    index = np.ascontiguousarray(index, dtype=np.int32)
    N = col_start.size - 1
    W = np.empty((K, N), np.int8)
    rc = _load().oracle_signed_to_dense(_p(col_start), _p(index), K, N, _p(W))
    if rc:
        raise ValueError(f"oracle_signed_to_dense failed ({rc})")
    return W


def _xb(X, b, K, N):
    X = np.ascontiguousarray(X, dtype=np.float32)
    if X.ndim != 2 or X.shape[1] != K:
        raise ValueError("X has the wrong shape")
    if b is not None:
        b = np.ascontiguousarray(b, dtype=np.float32)
        if b.shape != (N,):
            raise ValueError("b has the wrong length")
    return X, b


def tstgemm_signed(X, col_start, index, b, K: int):
    """(Yd, A) of Y = X W + b with W given as merged signed lists."""
    col_start = np.ascontiguousarray(col_start, dtype=np.int32)
    index = np.ascontiguousarray(index, dtype=np.int32)
    N = col_start.size - 1
    X, b = _xb(X, b, K, N)
    M = X.shape[0]
    Yd = np.empty((M, N), np.float64)
    A = np.empty((M, N), np.float64)
    rc = _load().oracle_tstgemm_signed(_p(X), _p(col_start), _p(index), _p(b), M, K, N, _p(Yd), _p(A))
    if rc:
        raise ValueError(f"oracle_tstgemm_signed failed ({rc})")
    return Yd, A


def pack5(W: np.ndarray) -> np.ndarray:
    """codes[n][g]: five consecutive rows of column n as one base-3 number (uint8, N x ceil(K/5))."""
    W = np.ascontiguousarray(W, dtype=np.int8)
    K, N = W.shape
    codes = np.empty((N, (K + 4) // 5), np.uint8)
    rc = _load().oracle_pack5(_p(W), K, N, _p(codes))
    if rc:
        raise ValueError(f"oracle_pack5 failed ({rc})")
    return codes


def unpack5(codes: np.ndarray, K: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, G = codes.shape
    if G != (K + 4) // 5:
        raise ValueError("codes has the wrong number of groups")
    W = np.empty((K, N), np.int8)
    rc = _load().oracle_unpack5(_p(codes), K, N, _p(W))
    if rc:
        raise ValueError(f"oracle_unpack5 failed ({rc})")
    return W


def tstgemm_packed(X, codes, b, K: int):
    """(Yd, A) of Y = X W + b with W given as base-3 codes."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, G = codes.shape
    if G != (K + 4) // 5:
        raise ValueError("codes has the wrong number of groups")
    X, b = _xb(X, b, K, N)
    M = X.shape[0]
    Yd = np.empty((M, N), np.float64)
    A = np.empty((M, N), np.float64)
    rc = _load().oracle_tstgemm_packed(_p(X), _p(codes), _p(b), M, K, N, _p(Yd), _p(A))
    if rc:
        raise ValueError(f"oracle_tstgemm_packed failed ({rc})")
    return Yd, A
