"""Pins for the CPU oracle: everything here checks oracle/ against something that is not
oracle/ -- hand-worked values, a library dense product, a library CSC builder, closed forms
and invariants of Eq. 1.  No GPU, no product code."""
import json

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import synth_inputs as si

ODD_SHAPES = [(1, 1, 1), (3, 37, 5), (2, 513, 65), (7, 64, 1), (5, 1, 9), (4, 130, 33)]


def dense_reference(X, W, b):
    """Eq. 1 through numpy's float64 matrix product (finite X, so the product equals the gather sum)."""
    Xd = X.astype(np.float64)
    Wd = W.astype(np.float64)
    Y = Xd @ Wd + (0.0 if b is None else b.astype(np.float64))
    A = np.abs(Xd) @ np.abs(Wd) + (0.0 if b is None else np.abs(b.astype(np.float64)))
    return Y, A


def test_worked_example(golden_dir):
    g = json.loads((golden_dir / "worked_example.json").read_text())
    W = np.array(g["W"], np.int8)
    t = oracle.tcsc_build(W)
    assert t.col_start_pos.tolist() == g["col_start_pos"]
    assert t.col_start_neg.tolist() == g["col_start_neg"]
    assert t.row_index_pos.tolist() == g["row_index_pos"]
    assert t.row_index_neg.tolist() == g["row_index_neg"]
    Yd, A, _ = oracle.tstgemm(np.array(g["X"], np.float32), t, np.array(g["b"], np.float32))
    assert Yd.tolist() == g["Y"]          # all values are exact binary fractions
    assert A.tolist() == g["A"]


@pytest.mark.parametrize("M,K,N", ODD_SHAPES)
@pytest.mark.parametrize("density", [0.5, 0.125, 1.0])
def test_brute_force_dense(M, K, N, density):
    W, X, b = si.make_inputs(M, K, N, density, "normal", seed=7 + M + K + N)
    t = oracle.tcsc_build(W)
    Yd, A, _ = oracle.tstgemm(X, t, b)
    Yref, Aref = dense_reference(X, W, b)
    assert np.all(np.abs(Yd - Yref) <= 1e-12 * Aref + 1e-300)
    assert np.all(np.abs(A - Aref) <= 1e-12 * Aref + 1e-300)


@pytest.mark.parametrize("K,N,density", [(37, 5, 0.5), (512, 512, 0.5), (300, 70, 0.0625), (64, 9, 1.0), (16, 4, 0.0)])
def test_format_matches_library_csc(K, N, density):
    """The +1 / -1 lists are exactly the CSC index structure of (W==1) / (W==-1)."""
    W, _, _ = si.make_inputs(1, K, N, density, "uniform", seed=11)
    t = oracle.tcsc_build(W)
    for mask, cs, ri in [(W == 1, t.col_start_pos, t.row_index_pos), (W == -1, t.col_start_neg, t.row_index_neg)]:
        c = sp.csc_matrix(mask.astype(np.int8))
        c.sort_indices()
        assert cs.dtype == np.int32 and ri.dtype == np.int32
        assert np.array_equal(cs, c.indptr)
        assert np.array_equal(ri, c.indices)
    # structure stated in Sec. 2 / Sec. 3: N+1 pointers, start at 0, end at nnz, ascending rows in a column
    assert t.col_start_pos[0] == 0 and t.col_start_pos[-1] == t.row_index_pos.size
    assert t.col_start_neg[0] == 0 and t.col_start_neg[-1] == t.row_index_neg.size
    assert t.nnz == int(np.count_nonzero(W))
    for cs, ri in [(t.col_start_pos, t.row_index_pos), (t.col_start_neg, t.row_index_neg)]:
        assert np.all(np.diff(cs) >= 0)
        for j in range(N):
            seg = ri[cs[j]:cs[j + 1]]
            assert np.all(np.diff(seg) > 0)
            assert seg.size == 0 or (seg[0] >= 0 and seg[-1] < K)


def test_round_trip_and_bad_values():
    W, _, _ = si.make_inputs(1, 129, 31, 0.5, "uniform", seed=3)
    assert np.array_equal(oracle.tcsc_to_dense(oracle.tcsc_build(W)), W)
    bad = W.copy()
    bad[5, 7] = 2
    with pytest.raises(ValueError):
        oracle.tcsc_build(bad)


def test_zero_weights_give_bias():
    _, X, b = si.make_inputs(6, 40, 11, 0.5, "normal", seed=5)
    t = oracle.tcsc_build(np.zeros((40, 11), np.int8))
    Yd, A, _ = oracle.tstgemm(X, t, b)
    assert np.array_equal(Yd, np.broadcast_to(b.astype(np.float64), Yd.shape))
    assert np.array_equal(A, np.broadcast_to(np.abs(b.astype(np.float64)), A.shape))
    Y0, _, _ = oracle.tstgemm(X, t, None)
    assert np.all(Y0 == 0.0)


def test_negated_weights_negate_the_product():
    W, X, b = si.make_inputs(5, 200, 17, 0.5, "normal", seed=9)
    t = oracle.tcsc_build(W)
    Yp, Ap, _ = oracle.tstgemm(X, t, None)
    Yn, An, _ = oracle.tstgemm(X, t.negated(), None)
    assert np.array_equal(Yn, -Yp)
    assert np.array_equal(An, Ap) or np.allclose(An, Ap, rtol=1e-15)
    assert np.array_equal(oracle.tcsc_to_dense(t.negated()), -W)
    # and the sign convention itself: a single +1 adds, a single -1 subtracts
    E = np.zeros((3, 2), np.int8)
    E[1, 0], E[2, 1] = 1, -1
    x = np.array([[10.0, 20.0, 30.0]], np.float32)
    Y, _, _ = oracle.tstgemm(x, oracle.tcsc_build(E), np.array([1.0, 2.0], np.float32))
    assert Y.tolist() == [[21.0, -28.0]]


def test_one_plus_one_per_column_is_a_gather():
    rng = np.random.default_rng(21)
    K, N, M = 50, 23, 4
    pick = rng.integers(0, K, size=N)
    W = np.zeros((K, N), np.int8)
    W[pick, np.arange(N)] = 1
    X = rng.standard_normal((M, K), dtype=np.float32)
    Y, _, _ = oracle.tstgemm(X, oracle.tcsc_build(W), None)
    assert np.array_equal(Y, X[:, pick].astype(np.float64))


def test_all_ones_is_row_sum():
    rng = np.random.default_rng(22)
    K, N, M = 33, 6, 5
    X = rng.integers(-8, 9, size=(M, K)).astype(np.float32)
    b = rng.integers(-8, 9, size=N).astype(np.float32)
    Y, _, _ = oracle.tstgemm(X, oracle.tcsc_build(np.ones((K, N), np.int8)), b)
    expect = X.astype(np.int64).sum(axis=1)[:, None] + b.astype(np.int64)[None, :]
    assert np.array_equal(Y, expect.astype(np.float64))


def test_integer_inputs_are_exact():
    W, X, b = si.make_inputs(9, 700, 40, 0.5, "int8", seed=31)
    Y, _, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    expect = X.astype(np.int64) @ W.astype(np.int64) + b.astype(np.int64)
    assert np.array_equal(Y, expect.astype(np.float64))


def test_row_permutation_column_independence_and_row_subset():
    W, X, b = si.make_inputs(8, 150, 20, 0.25, "normal", seed=41)
    t = oracle.tcsc_build(W)
    Y, A, _ = oracle.tstgemm(X, t, b)
    perm = np.random.default_rng(0).permutation(8)
    Yp, _, _ = oracle.tstgemm(X[perm], t, b)
    assert np.array_equal(Yp, Y[perm])
    W2 = W.copy()
    W2[:, 3] = -W2[:, 3]
    Y2, _, _ = oracle.tstgemm(X, oracle.tcsc_build(W2), b)
    keep = np.arange(20) != 3
    assert np.array_equal(Y2[:, keep], Y[:, keep]) and not np.array_equal(Y2[:, 3], Y[:, 3])
    rows = np.array([5, 0, 5, 7], np.int32)
    Yr, Ar, _ = oracle.tstgemm(X, t, b, rows=rows)
    assert np.array_equal(Yr, Y[rows]) and np.array_equal(Ar, A[rows])
    ms = np.array([0, 7, 3], np.int32)
    ns = np.array([19, 0, 3], np.int32)
    Ypt, Apt = oracle.tstgemm_points(X, t, b, ms, ns)
    assert np.array_equal(Ypt, Y[ms, ns]) and np.array_equal(Apt, A[ms, ns])


def test_thread_count_does_not_change_results():
    W, X, b = si.make_inputs(16, 256, 48, 0.5, "normal", seed=51)
    t = oracle.tcsc_build(W)
    Y1, _, used1 = oracle.tstgemm(X, t, b, threads=1)
    Y4, _, used4 = oracle.tstgemm(X, t, b, threads=4)
    assert used1 == 1 and used4 == 4
    assert np.array_equal(Y1, Y4)


def test_generator_statistics():
    """E[nnz] = d K N and P(+1) = P(-1): the recipe the workloads are drawn with."""
    K, N, d = 1024, 512, 0.5
    W, X, b = si.make_inputs(4, K, N, d, "uniform", seed=1002)
    n = K * N
    sd = np.sqrt(n * d * (1 - d))
    assert abs(np.count_nonzero(W) - d * n) < 5 * sd
    assert abs(int((W == 1).sum()) - int((W == -1).sum())) < 5 * np.sqrt(n * d)
    assert X.dtype == np.float32 and b.dtype == np.float32 and W.dtype == np.int8
    assert X.min() >= -1 and X.max() < 1
    W2, X2, b2 = si.make_inputs(4, K, N, d, "uniform", seed=1002)
    assert np.array_equal(W, W2) and np.array_equal(X, X2) and np.array_equal(b, b2)


def test_prelu_worked_example(golden_dir):
    g = json.loads((golden_dir / "worked_example.json").read_text())
    t = oracle.tcsc_build(np.array(g["W"], np.int8))
    Yd, A, _ = oracle.tstgemm(np.array(g["X"], np.float32), t, np.array(g["b"], np.float32))
    Yp, Ap = oracle.prelu(Yd, A, g["alpha_per_column"])
    assert Yp.tolist() == g["Y_prelu_per_column"]
    assert Ap.tolist() == (np.array(g["A"]) * np.maximum(1.0, np.abs(g["alpha_per_column"]))).tolist()
    Ys, As = oracle.prelu(Yd, A, g["alpha_scalar"])
    assert Ys.tolist() == g["Y_prelu_scalar"]
    assert As.tolist() == g["A"]


def test_prelu_special_slopes_and_library():
    """Slope 1 is the identity, slope 0 is max(v, 0), slope -1 is |v|; arbitrary per-column slopes against torch's
    CPU prelu in float64."""
    import torch
    W, X, b = si.make_inputs(6, 70, 9, 0.5, "normal", seed=55)
    Yd, A, _ = oracle.tstgemm(X, oracle.tcsc_build(W), b)
    assert (Yd < 0).any() and (Yd > 0).any()
    assert np.array_equal(oracle.prelu(Yd, A, 1.0)[0], Yd)
    assert np.array_equal(oracle.prelu(Yd, A, 0.0)[0], np.maximum(Yd, 0.0))
    assert np.array_equal(oracle.prelu(Yd, A, -1.0)[0], np.abs(Yd))
    alpha = np.linspace(-2.0, 3.0, 9).astype(np.float32)
    Yp, Ap = oracle.prelu(Yd, A, alpha)
    ref = torch.nn.functional.prelu(torch.from_numpy(Yd), torch.from_numpy(alpha.astype(np.float64))).numpy()
    assert np.array_equal(Yp, ref)
    assert np.array_equal(Ap, A * np.maximum(1.0, np.abs(alpha.astype(np.float64))))
    same = np.full(9, 0.3, np.float32)
    assert np.array_equal(oracle.prelu(Yd, A, same)[0], oracle.prelu(Yd, A, np.float32(0.3))[0])
    # the inputs are left alone
    Y0 = Yd.copy()
    oracle.prelu(Yd, A, alpha)
    assert np.array_equal(Yd, Y0)
