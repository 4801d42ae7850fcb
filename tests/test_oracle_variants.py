"""Pins for the oracle of the two alternative encodings of W (Sec. 3 of the paper, "Inverted Index" and "Value
Compression"): hand-worked values, closed forms, round trips through the dense matrix, a library dense product
and the TCSC oracle's result.  No GPU, no product code."""
import itertools
import json

import numpy as np
import pytest

import oracle
import synth_inputs as si

SHAPES = [(1, 1, 1), (3, 37, 5), (2, 513, 65), (7, 64, 1), (5, 4, 9), (4, 131, 33)]


def dense_reference(X, W, b):
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    return Xd @ Wd + b.astype(np.float64), np.abs(Xd) @ np.abs(Wd) + np.abs(b.astype(np.float64))


# ------------------------------------------------------------------------------------------------ inverted index

def test_signed_worked_example(golden_dir):
    g = json.loads((golden_dir / "worked_example.json").read_text())
    W = np.array(g["W"], np.int8)
    cs, idx = oracle.signed_build(oracle.tcsc_build(W))
    assert cs.tolist() == g["signed_col_start"]
    assert idx.tolist() == g["signed_index"]
    Yd, A = oracle.tstgemm_signed(np.array(g["X"], np.float32), cs, idx, np.array(g["b"], np.float32), g["K"])
    assert Yd.tolist() == g["Y"] and A.tolist() == g["A"]
    assert np.array_equal(oracle.signed_to_dense(cs, idx, g["K"]), W)


@pytest.mark.parametrize("M,K,N", SHAPES)
@pytest.mark.parametrize("density", [0.5, 0.0625, 1.0])
def test_signed_stream_properties(M, K, N, density):
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=900 + K + N)
    t = oracle.tcsc_build(W)
    cs, idx = oracle.signed_build(t)
    # one pointer array whose steps are the column counts of both signs together
    assert np.array_equal(cs, t.col_start_pos + t.col_start_neg)
    assert idx.size == t.nnz and int((idx < 0).sum()) == t.row_index_neg.size
    rows = np.where(idx < 0, -idx.astype(np.int64) - 1, idx)        # ~i = -i - 1
    for n in range(N):
        col = rows[cs[n]:cs[n + 1]]
        assert np.all(np.diff(col) > 0)                             # ascending rows inside a column
        sign = np.where(idx[cs[n]:cs[n + 1]] < 0, -1, 1)
        assert np.array_equal(W[col, n], sign)                      # the sign travels with the entry
        assert np.count_nonzero(W[:, n]) == col.size
    assert np.array_equal(oracle.signed_to_dense(cs, idx, K), W)
    Yd, A = oracle.tstgemm_signed(X, cs, idx, b, K)
    Yref, Aref = dense_reference(X, W, b)
    assert np.allclose(Yd, Yref, rtol=0, atol=1e-12 * max(1.0, Aref.max()))
    assert np.allclose(A, Aref, rtol=1e-13, atol=0)
    # integer inputs: every order of summation gives the same, exact sum as the TCSC oracle
    _, Xi, bi = si.make_inputs(M, K, N, density, "int8", seed=901 + K)
    assert np.array_equal(oracle.tstgemm_signed(Xi, cs, idx, bi, K)[0], oracle.tstgemm(Xi, t, bi)[0])


def test_signed_zero_row_keeps_its_sign():
    """Row 0 is where i and ~i differ from i and -i: -1 in row 0 must be stored as -1, not as 0."""
    W = np.array([[-1, 1], [1, -1]], np.int8)
    cs, idx = oracle.signed_build(oracle.tcsc_build(W))
    assert cs.tolist() == [0, 2, 4] and idx.tolist() == [-1, 1, 0, -2]
    X = np.array([[3.0, 5.0]], np.float32)
    Yd, _ = oracle.tstgemm_signed(X, cs, idx, None, 2)
    assert Yd.tolist() == [[2.0, -2.0]]


# ------------------------------------------------------------------------------------------- value compression

def test_packed_worked_example(golden_dir):
    g = json.loads((golden_dir / "worked_example.json").read_text())
    W = np.array(g["W"], np.int8)
    codes = oracle.pack5(W)
    assert codes.tolist() == g["packed_codes"]
    Yd, A = oracle.tstgemm_packed(np.array(g["X"], np.float32), codes, np.array(g["b"], np.float32), g["K"])
    assert Yd.tolist() == g["Y"] and A.tolist() == g["A"]
    col = np.array(g["packed_k7_column"], np.int8).reshape(7, 1)
    c7 = oracle.pack5(col)
    assert c7.tolist() == g["packed_k7_codes"]
    assert np.array_equal(oracle.unpack5(c7, 7), col)


def test_packed_codes_are_base3_numbers():
    """All 243 five-tuples as columns: code = sum of digit * 3^(4 - row) with digits 0, 1, 2 for 0, +1, -1; the
    codes are exactly 0..242, each once (3^5 = 243 of the 256 byte values, 5.08 % unused)."""
    tuples = np.array(list(itertools.product((0, 1, -1), repeat=5)), np.int8)      # 243 x 5
    codes = oracle.pack5(np.ascontiguousarray(tuples.T))[:, 0].astype(np.int64)
    digits = np.where(tuples == -1, 2, tuples).astype(np.int64)
    assert np.array_equal(codes, digits @ np.array([81, 27, 9, 3, 1]))
    assert sorted(codes.tolist()) == list(range(243))
    assert abs((256 - 243) / 256 - 0.0508) < 5e-5
    assert np.array_equal(oracle.unpack5(codes.astype(np.uint8).reshape(243, 1), 5), tuples.T)


@pytest.mark.parametrize("M,K,N", SHAPES)
@pytest.mark.parametrize("density", [0.5, 0.0625, 1.0])
def test_packed_properties(M, K, N, density):
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=950 + K + N)
    codes = oracle.pack5(W)
    assert codes.shape == (N, -(-K // 5)) and codes.max(initial=0) <= 242
    assert np.array_equal(oracle.unpack5(codes, K), W)
    # an all-zero group has code 0; a matrix of zeros is all code 0
    zero_groups = [(n, g) for n in range(N) for g in range(codes.shape[1]) if not W[5 * g:5 * g + 5, n].any()]
    assert all(codes[n, g] == 0 for n, g in zero_groups)
    assert int((codes == 0).sum()) == len(zero_groups)
    Yd, A = oracle.tstgemm_packed(X, codes, b, K)
    Yref, Aref = dense_reference(X, W, b)
    assert np.allclose(Yd, Yref, rtol=0, atol=1e-12 * max(1.0, Aref.max()))
    assert np.allclose(A, Aref, rtol=1e-13, atol=0)
    _, Xi, bi = si.make_inputs(M, K, N, density, "int8", seed=951 + K)
    assert np.array_equal(oracle.tstgemm_packed(Xi, codes, bi, K)[0], oracle.tstgemm(Xi, oracle.tcsc_build(W), bi)[0])


def test_packed_rejects_bad_codes_and_skips_zero_weights():
    with pytest.raises(ValueError):
        oracle.unpack5(np.array([[243]], np.uint8), 5)
    with pytest.raises(ValueError):
        oracle.unpack5(np.array([[1]], np.uint8), 4)      # digit of a padding row (row 4 of K = 4) is not zero
    with pytest.raises(ValueError):
        oracle.pack5(np.array([[2]], np.int8))
    # zero weights never read X: a NaN under them does not reach Y
    W = np.array([[1], [0], [-1]], np.int8)
    X = np.array([[2.0, np.nan, 0.5]], np.float32)
    Yd, _ = oracle.tstgemm_packed(X, oracle.pack5(W), None, 3)
    assert Yd.tolist() == [[1.5]]
    cs, idx = oracle.signed_build(oracle.tcsc_build(W))
    assert oracle.tstgemm_signed(X, cs, idx, None, 3)[0].tolist() == [[1.5]]
