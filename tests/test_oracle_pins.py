"""Pins for the CPU oracle: every oracle function is checked against something other than
itself -- hand-worked examples, brute force in pure Python on tiny inputs, closed forms,
invariants and finite differences -- chosen so that a dropped term, a wrong sign or index, or a
transposed operand fails at least one test.  The paper prints no numeric example, so there are
no paper-printed goldens; the hand-worked example lives in tests/golden/.
"""
import json
import math
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------------------------
# helpers written without the oracle
# ------------------------------------------------------------------------------------------------

def py_entry_set(n, src, dst, symmetrise, self_loops):
    s = set()
    for u, v in zip(src.tolist(), dst.tolist()):
        if u == v:
            continue
        s.add((u, v))
        if symmetrise:
            s.add((v, u))
    if self_loops:
        for i in range(n):
            s.add((i, i))
    return s


def py_dense(A: "oracle.Csr"):
    D = [[0.0] * A.n for _ in range(A.n)]
    for i in range(A.n):
        for k in range(int(A.rowptr[i]), int(A.rowptr[i + 1])):
            D[i][int(A.colidx[k])] = float(A.val[k])
    return D


def py_matmul(A, B):
    M, K, N = len(A), len(B), len(B[0])
    return [[math.fsum(A[i][k] * B[k][j] for k in range(K)) for j in range(N)] for i in range(M)]


def small_graph(n=40, m=90, seed=3):
    src, dst = synth.erdos_renyi(n, m, seed)
    return n, src, dst


# ------------------------------------------------------------------------------------------------
# graph construction ("Graph Neural Networks": self-connections, D^-1/2 (A+I) D^-1/2)
# ------------------------------------------------------------------------------------------------

def test_csr_hand_worked_example():
    # tests/golden/five_vertex_graph.json was worked by hand from the definition.
    with open(os.path.join(GOLDEN, "five_vertex_graph.json")) as fh:
        g = json.load(fh)
    A = oracle.build_csr(g["n"], np.array(g["src"], np.int32), np.array(g["dst"], np.int32))
    assert A.rowptr.tolist() == g["rowptr"]
    assert A.colidx.tolist() == g["colidx"]
    assert A.deg.tolist() == g["deg"]
    want = [1.0 / math.sqrt(a * b) for a, b in g["val_degree_products"]]
    np.testing.assert_array_equal(A.val, np.array(want, np.float64).astype(np.float32))


@pytest.mark.parametrize("symmetrise", [True, False])
@pytest.mark.parametrize("self_loops", [True, False])
def test_csr_matches_python_set(symmetrise, self_loops):
    n, src, dst = small_graph()
    src = np.concatenate([src, src[:7], np.array([2, 5], np.int32)])     # duplicates and input loops
    dst = np.concatenate([dst, dst[:7], np.array([2, 5], np.int32)])
    A = oracle.build_csr(n, src, dst, symmetrise, self_loops, norm="none")
    want = sorted(py_entry_set(n, src, dst, symmetrise, self_loops))
    got = [(i, int(A.colidx[k])) for i in range(n) for k in range(int(A.rowptr[i]), int(A.rowptr[i + 1]))]
    assert got == want
    assert np.all(A.val == 1.0)


def test_csr_invariants():
    n, src, dst = small_graph(200, 900, 5)
    A = oracle.build_csr(n, src, dst)
    assert A.rowptr[0] == 0 and A.rowptr[-1] == A.colidx.shape[0] == A.val.shape[0]
    assert np.all(np.diff(A.rowptr) >= 1)
    for i in range(n):
        cols = A.colidx[A.rowptr[i]:A.rowptr[i + 1]]
        assert np.all(np.diff(cols) > 0)
        assert i in cols.tolist()
    assert int(A.deg.sum()) == A.nnz
    D = np.array(py_dense(A))
    assert np.array_equal(D != 0, (D != 0).T)
    assert np.array_equal(D, D.T)          # value symmetry is exact by construction


def test_csr_rejects_out_of_range():
    with pytest.raises(ValueError):
        oracle.build_csr(4, np.array([0, 4], np.int32), np.array([1, 2], np.int32))


def test_transpose_of_symmetric_is_identical():
    n, src, dst = small_graph(150, 600, 7)
    A = oracle.build_csr(n, src, dst)
    At = oracle.build_csr(n, src, dst, transpose=True)
    for a, b in [(A.rowptr, At.rowptr), (A.colidx, At.colidx), (A.val, At.val), (A.deg, At.deg)]:
        np.testing.assert_array_equal(a, b)


def test_transpose_of_directed_matches_dense_transpose():
    n, src, dst = small_graph(60, 200, 9)
    A = oracle.build_csr(n, src, dst, symmetrise=False)
    At = oracle.build_csr(n, src, dst, symmetrise=False, transpose=True)
    D, Dt = np.array(py_dense(A)), np.array(py_dense(At))
    assert not np.array_equal(D, D.T)
    np.testing.assert_array_equal(Dt, D.T)
    np.testing.assert_array_equal(A.deg, At.deg)     # degrees are those of the untransposed matrix
    # transposing twice: swap the roles of src and dst
    Att = oracle.build_csr(n, dst, src, symmetrise=False, transpose=True, norm="none")
    np.testing.assert_array_equal(Att.rowptr, A.rowptr)
    np.testing.assert_array_equal(Att.colidx, A.colidx)


def test_normalisation_closed_forms():
    # ring: every modified degree is 3, so every stored value is 1/3
    n = 17
    A = oracle.build_csr(n, *synth.ring(n))
    assert np.all(A.deg == 3)
    np.testing.assert_array_equal(A.val, np.full(A.nnz, np.float32(1.0 / 3.0)))
    # star: centre degree n, leaves degree 2
    n = 33
    A = oracle.build_csr(n, *synth.star(n))
    assert A.deg[0] == n and np.all(A.deg[1:] == 2)
    D = np.array(py_dense(A))
    assert D[0, 0] == np.float32(1.0 / n)
    assert np.all(D[0, 1:] == np.float32(1.0 / math.sqrt(2.0 * n)))
    assert np.all(np.diag(D)[1:] == np.float32(0.5))


def test_symmetric_normalisation_of_a_vertex_without_entries_is_zero():
    """Directed graph without self-connections: vertex 2 has incoming edges only, so its row is empty and
    D^-1/2 (a pseudo-inverse there) scales by 0: the stored values that touch it are 0, as are the
    per-vertex factors of the value-free product, and the two forms of the product agree."""
    src = np.array([0, 0, 1], np.int32)
    dst = np.array([1, 2, 2], np.int32)
    A = oracle.build_csr(3, src, dst, symmetrise=False, self_loops=False, norm="sym")
    assert A.deg.tolist() == [2, 1, 0] and A.colidx.tolist() == [1, 2, 2]
    assert A.val.tolist() == [np.float32(1 / math.sqrt(2.0)), 0.0, 0.0]
    s = oracle.inv_sqrt_degrees(A)
    assert s.tolist() == [np.float32(1 / math.sqrt(2.0)), 1.0, 0.0]
    X = synth.normal_features(3, 4, 5).astype(np.float64)
    np.testing.assert_allclose(oracle.spmm_pattern(A, oracle.scale_rows(X, s), s), oracle.spmm(A, X), rtol=1e-7)
    assert np.all(np.isfinite(oracle.spmm(A, X)))


def test_normalised_matrix_has_sqrt_degree_eigenvector():
    # D^-1/2 (A+I) D^-1/2 sqrt(d) = D^-1/2 (A+I) 1 = D^-1/2 d = sqrt(d)
    n, src, dst = small_graph(300, 2000, 11)
    A = oracle.build_csr(n, src, dst)
    x = np.sqrt(A.deg.astype(np.float64))[:, None]
    y = oracle.spmm(A, x)
    np.testing.assert_allclose(y, x, rtol=1e-6)


def test_row_slice_and_transpose_pins():
    """Block rows of the 1D algorithm: the slice's product is the matching rows of the full product;
    transposing twice gives the matrix back; the transposed slice matches the dense transpose."""
    n, src, dst = small_graph(60, 240, 29)
    A = oracle.build_csr(n, src, dst, symmetrise=False)
    S = oracle.slice_rows(A, 13, 41)
    assert (S.n, S.n_cols) == (28, n)
    D = np.array(py_dense(A))
    X = synth.normal_features(n, 4, 6).astype(np.float64)
    np.testing.assert_array_equal(oracle.spmm(S, X), oracle.spmm(A, X)[13:41])
    St = oracle.transpose(S)
    assert (St.n, St.n_cols) == (n, 28)
    Dt = np.zeros((n, 28))
    for i in range(n):
        for k in range(int(St.rowptr[i]), int(St.rowptr[i + 1])):
            Dt[i, St.colidx[k]] = St.val[k]
    np.testing.assert_array_equal(Dt, D[13:41].T)
    Stt = oracle.transpose(St)
    for a, b in [(Stt.rowptr, S.rowptr), (Stt.colidx, S.colidx), (Stt.val, S.val)]:
        np.testing.assert_array_equal(a, b)
    At = oracle.build_csr(n, src, dst, symmetrise=False, transpose=True)      # independent construction
    T = oracle.transpose(A)
    for a, b in [(T.rowptr, At.rowptr), (T.colidx, At.colidx), (T.val, At.val)]:
        np.testing.assert_array_equal(a, b)


def test_row_normalisation_pins():
    """D^-1 (A+I) on a directed graph: every row sums to one, the values are 1/d_i by hand, and the
    transposed structure carries the transposed values."""
    n, src, dst = small_graph(70, 260, 27)
    A = oracle.build_csr(n, src, dst, symmetrise=False, norm="row")
    At = oracle.build_csr(n, src, dst, symmetrise=False, norm="row", transpose=True)
    D, Dt = np.array(py_dense(A)), np.array(py_dense(At))
    np.testing.assert_array_equal(Dt, D.T)
    for i in range(n):
        row = D[i][D[i] != 0]
        assert len(row) == A.deg[i]
        assert np.all(row == np.float32(1.0 / A.deg[i]))
    ones = np.ones((n, 2), np.float64)
    np.testing.assert_allclose(oracle.spmm(A, ones), ones, rtol=1e-6)
    assert not np.allclose(oracle.spmm(At, ones), ones, rtol=1e-3)     # column sums are not one


# ------------------------------------------------------------------------------------------------
# SpMM
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_spmm_brute_force_dense(dtype):
    n, src, dst = small_graph(36, 100, 13)
    A = oracle.build_csr(n, src, dst, symmetrise=False)      # unsymmetric: catches a transposed operand
    X = synth.uniform_features(n, 5, 1).astype(dtype)
    want = np.array(py_matmul(py_dense(A), X.astype(np.float64).tolist()))
    got = oracle.spmm(A, X)
    assert got.dtype == dtype
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-7 if dtype == np.float32 else 1e-15)
    if dtype == np.float32:     # double accumulation, one rounding: equals the rounded exact sum
        np.testing.assert_array_equal(got, want.astype(np.float32))


def test_spmm_identity_returns_operand_bitwise():
    n = 50
    A = oracle.build_csr(n, np.zeros(0, np.int32), np.zeros(0, np.int32))   # only self loops, deg 1
    assert np.all(A.val == 1.0) and A.nnz == n
    X = synth.normal_features(n, 7, 2)
    np.testing.assert_array_equal(oracle.spmm(A, X), X)


def test_spmm_ones_gives_integer_degrees():
    n, src, dst = synth.make_graph(synth.scaled(3, 64))
    A = oracle.build_csr(n, src, dst, norm="none")
    Z = oracle.spmm(A, np.ones((n, 3), np.float32))
    np.testing.assert_array_equal(Z, np.repeat(A.deg.astype(np.float32)[:, None], 3, axis=1))
    assert A.deg.max() > 64      # the skewed generator does make heavy rows


def test_spmm_unit_vector_extracts_column():
    n, src, dst = small_graph(30, 80, 17)
    A = oracle.build_csr(n, src, dst, symmetrise=False)
    D = np.array(py_dense(A))
    for j in (0, 7, 29):
        e = np.zeros((n, 1), np.float64)
        e[j] = 1.0
        np.testing.assert_array_equal(oracle.spmm(A, e)[:, 0], D[:, j])


def test_spmm_linearity_and_leading_dimension():
    n, src, dst = small_graph(64, 300, 19)
    A = oracle.build_csr(n, src, dst)
    X = synth.normal_features(n, 6, 3).astype(np.float64)
    Y = synth.normal_features(n, 6, 4).astype(np.float64)
    lhs = oracle.spmm(A, 2.0 * X - 3.0 * Y)
    rhs = 2.0 * oracle.spmm(A, X) - 3.0 * oracle.spmm(A, Y)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-13)
    wide = np.concatenate([X, Y], axis=1)            # a view with ld = 12 > f = 6
    np.testing.assert_array_equal(oracle.spmm(A, wide[:, :6]), oracle.spmm(A, X))


def test_spmm_rows_equals_rows_of_full_product():
    n, src, dst = small_graph(80, 400, 21)
    A = oracle.build_csr(n, src, dst)
    X = synth.normal_features(n, 9, 5)
    rows = np.array([79, 0, 13, 13, 42])
    np.testing.assert_array_equal(oracle.spmm_rows(A, X, rows), oracle.spmm(A, X)[rows])


# value-free form for the symmetric normalisation: D^-1/2 (A+I) D^-1/2 X = D^-1/2 ((A+I) (D^-1/2 X))

def test_pattern_product_brute_force_and_unit_cases():
    n, src, dst = small_graph(36, 100, 23)
    A = oracle.build_csr(n, src, dst, symmetrise=False)          # unsymmetric pattern
    entries = py_entry_set(n, src, dst, False, True)
    X = synth.normal_features(n, 4, 6).astype(np.float64)
    rs = (np.arange(n) % 5 + 1).astype(np.float32) / 4           # exactly representable scales
    want = [[float(rs[i]) * math.fsum(X[j, c] for (r, j) in entries if r == i) for c in range(4)] for i in range(n)]
    np.testing.assert_allclose(oracle.spmm_pattern(A, X, rs), np.array(want), rtol=1e-14, atol=1e-14)
    # no scale, operand of ones: the integer row lengths, whatever the stored values are
    ones = np.ones((n, 2), np.float32)
    np.testing.assert_array_equal(oracle.spmm_pattern(A, ones), np.repeat(A.deg.astype(np.float32)[:, None], 2, axis=1))
    # scale_rows and the inverse square roots against their definitions
    s = oracle.inv_sqrt_degrees(A)
    np.testing.assert_array_equal(s, np.array([np.float32(1.0 / math.sqrt(int(d))) for d in A.deg]))
    Y = oracle.scale_rows(X, rs)
    np.testing.assert_array_equal(Y, X * rs.astype(np.float64)[:, None])


@pytest.mark.parametrize("directed", [False, True])
def test_pattern_product_equals_normalised_product(directed):
    """The factorised form gives the product with the normalised matrix: in the double build the two
    differ only by the float roundings of val_ij and s_i (a few 2^-24 relative per term)."""
    n, src, dst = synth.make_graph(synth.scaled(3, 128))
    A = oracle.build_csr(n, src, dst, symmetrise=not directed)
    At = oracle.build_csr(n, src, dst, symmetrise=not directed, transpose=True)
    X = np.abs(synth.normal_features(n, 3, 8).astype(np.float64)) + 0.1      # positive: no cancellation
    s = oracle.inv_sqrt_degrees(A)
    for M in (A, At):
        got = oracle.spmm_pattern(M, oracle.scale_rows(X, s), s)
        want = oracle.spmm(M, X)
        np.testing.assert_allclose(got, want, rtol=4e-7, atol=0)
    # closed form on a ring: every row holds two neighbours and the loop, so all degrees are 3
    src, dst = synth.ring(12)
    R = oracle.build_csr(12, src, dst)
    x = np.arange(12, dtype=np.float64)[:, None]
    sr = oracle.inv_sqrt_degrees(R)
    got = oracle.spmm_pattern(R, oracle.scale_rows(x, sr), sr)[:, 0]
    want = np.array([(x[(i - 1) % 12, 0] + x[i, 0] + x[(i + 1) % 12, 0]) * float(sr[0]) ** 2 for i in range(12)])
    np.testing.assert_allclose(got, want, rtol=1e-15)


# ------------------------------------------------------------------------------------------------
# dense products
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_gemm_against_python_triple_loop(ta, tb):
    rng = np.random.default_rng(5)
    M, K, N = 7, 5, 4
    A = rng.integers(-4, 5, size=(K, M) if ta else (M, K)).astype(np.float64)
    B = rng.integers(-4, 5, size=(N, K) if tb else (K, N)).astype(np.float64)
    opA = [[A[k][i] if ta else A[i][k] for k in range(K)] for i in range(M)]
    opB = [[B[j][k] if tb else B[k][j] for j in range(N)] for k in range(K)]
    want = np.array(py_matmul(opA, opB))
    np.testing.assert_array_equal(oracle.gemm(A, B, ta, tb), want)          # small integers: exact
    np.testing.assert_array_equal(oracle.gemm(A.astype(np.float32), B.astype(np.float32), ta, tb),
                                  want.astype(np.float32))


def test_gemm_identity_weight_returns_operand():
    H = synth.normal_features(23, 6, 6)
    np.testing.assert_array_equal(oracle.gemm(H, np.eye(6, dtype=np.float32)), H)


# ------------------------------------------------------------------------------------------------
# activation, loss
# ------------------------------------------------------------------------------------------------

def test_relu_and_mask_values():
    z = np.array([[-1.5, -0.0, 0.0, 1e-30, 2.0]], np.float32)
    g = np.array([[10.0, 20.0, 30.0, 40.0, 50.0]], np.float32)
    np.testing.assert_array_equal(oracle.relu(z), np.array([[0, 0, 0, 1e-30, 2.0]], np.float32))
    np.testing.assert_array_equal(oracle.relu_mask(g, z), np.array([[0, 0, 0, 40.0, 50.0]], np.float32))


def test_softmax_nll_closed_forms():
    n, Cn = 12, 7
    y = synth.labels(n, Cn, 1)
    loss, G = oracle.softmax_nll(np.full((n, Cn), 3.25, np.float64), y)
    assert abs(loss - math.log(Cn)) < 1e-15
    want = np.full((n, Cn), 1.0 / Cn)
    want[np.arange(n), y] -= 1.0
    np.testing.assert_allclose(G, want / n, rtol=1e-14)
    # a confidently right and a confidently wrong row
    Z = np.array([[50.0, 0.0], [0.0, 50.0]])
    loss, _ = oracle.softmax_nll(Z, np.array([0, 0], np.int32))
    assert abs(loss - 0.5 * 50.0) < 1e-12


def test_softmax_nll_invariants_and_python_reference():
    n, Cn = 9, 5
    Z = synth.normal_features(n, Cn, 8).astype(np.float64) * 3.0
    y = synth.labels(n, Cn, 2)
    loss, G = oracle.softmax_nll(Z, y)
    ref = 0.0
    for i in range(n):
        lse = math.log(math.fsum(math.exp(v) for v in Z[i].tolist()))
        ref -= Z[i, y[i]] - lse
        p = [math.exp(v - lse) for v in Z[i].tolist()]
        assert abs(math.fsum(p) - 1.0) < 1e-12
        for j in range(Cn):
            assert abs(G[i, j] - (p[j] - (1.0 if j == y[i] else 0.0)) / n) < 1e-15
    assert abs(loss - ref / n) < 1e-13
    np.testing.assert_allclose(G.sum(axis=1), 0.0, atol=1e-15)
    shifted, Gs = oracle.softmax_nll(Z + 1000.0, y)           # shift invariance, no overflow
    assert abs(shifted - loss) < 1e-10
    np.testing.assert_allclose(Gs, G, atol=1e-12)


def test_softmax_nll_gradient_by_finite_differences():
    n, Cn = 6, 4
    Z = synth.normal_features(n, Cn, 9).astype(np.float64)
    y = synth.labels(n, Cn, 3)
    _, G = oracle.softmax_nll(Z, y)
    eps = 1e-6
    for i in range(n):
        for j in range(Cn):
            Zp, Zm = Z.copy(), Z.copy()
            Zp[i, j] += eps
            Zm[i, j] -= eps
            fd = (oracle.softmax_nll(Zp, y, False)[0] - oracle.softmax_nll(Zm, y, False)[0]) / (2 * eps)
            assert abs(fd - G[i, j]) < 1e-9


def test_softmax_nll_training_split():
    """Negative labels mark vertices outside the training split: the loss is the mean over the others,
    their gradient rows are zero, and the rest equals the unmasked computation on the subset."""
    n, Cn = 11, 4
    Z = synth.normal_features(n, Cn, 21).astype(np.float64) * 2.0
    y = synth.labels(n, Cn, 5)
    ym = y.copy()
    out_of_split = np.array([0, 3, 4, 9])
    ym[out_of_split] = -1
    keep = np.setdiff1d(np.arange(n), out_of_split)
    loss_m, G_m = oracle.softmax_nll(Z, ym)
    loss_s, G_s = oracle.softmax_nll(Z[keep], y[keep])
    assert abs(loss_m - loss_s) < 1e-14
    np.testing.assert_array_equal(G_m[out_of_split], 0.0)
    np.testing.assert_allclose(G_m[keep], G_s, rtol=1e-14)
    ref = -sum(Z[i, y[i]] - math.log(math.fsum(math.exp(v) for v in Z[i].tolist())) for i in keep.tolist()) / len(keep)
    assert abs(loss_m - ref) < 1e-13
    eps = 1e-6
    for (i, j) in [(0, 1), (1, 2), (9, 0), (10, 3)]:
        Zp, Zm = Z.copy(), Z.copy()
        Zp[i, j] += eps
        Zm[i, j] -= eps
        fd = (oracle.softmax_nll(Zp, ym, False)[0] - oracle.softmax_nll(Zm, ym, False)[0]) / (2 * eps)
        assert abs(fd - G_m[i, j]) < 1e-9


def test_sgd_step():
    W = np.array([[1.0, -2.0]], np.float64)
    Y = np.array([[0.5, 4.0]], np.float64)
    np.testing.assert_array_equal(oracle.sgd(W, Y, 0.1), np.array([[0.95, -2.4]]))
    np.testing.assert_array_equal(W, np.array([[1.0, -2.0]]))


# ------------------------------------------------------------------------------------------------
# forward / backward (Equations 1-3)
# ------------------------------------------------------------------------------------------------

def tiny_problem(directed, dims=(5, 4, 3, 3), n=24, seed=4):
    src, dst = synth.erdos_renyi(n, 60, seed)
    kw = dict(symmetrise=not directed)
    A = oracle.build_csr(n, src, dst, **kw)
    At = oracle.build_csr(n, src, dst, transpose=True, **kw)
    H0 = synth.normal_features(n, dims[0], seed).astype(np.float64)
    y = synth.labels(n, dims[-1], seed)
    Ws = [w.astype(np.float64) * 2.0 for w in synth.glorot_weights(dims, seed)]
    return A, At, H0, y, Ws


def test_forward_matches_dense_python():
    A, At, H0, y, Ws = tiny_problem(directed=True, dims=(4, 3, 2))
    Zs, Hs = oracle.forward(At, H0, Ws)
    D = np.array(py_dense(A))                     # A itself; the formula needs A^T
    H = H0
    for l, W in enumerate(Ws):
        Z = np.array(py_matmul(D.T.tolist(), py_matmul(H.tolist(), W.tolist())))
        np.testing.assert_allclose(Zs[l], Z, rtol=1e-13, atol=1e-14)
        H = np.maximum(Z, 0.0) if l + 1 < len(Ws) else Z
        np.testing.assert_allclose(Hs[l + 1], H, rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("directed", [False, True])
def test_weight_gradients_by_central_differences(directed):
    """Equation 3 (with Equations 1 and 2 feeding it) against d loss / d W, every element of every
    weight matrix.  The directed case fails if A and A^T are swapped anywhere."""
    A, At, H0, y, Ws = tiny_problem(directed)
    out = oracle.epoch(A, At, H0, y, Ws)
    eps = 1e-5
    for l, W in enumerate(Ws):
        for i in range(W.shape[0]):
            for j in range(W.shape[1]):
                Wp = [w.copy() for w in Ws]
                Wm = [w.copy() for w in Ws]
                Wp[l][i, j] += eps
                Wm[l][i, j] -= eps
                fd = (oracle.loss_only(At, H0, y, Wp) - oracle.loss_only(At, H0, y, Wm)) / (2 * eps)
                an = out["Y"][l][i, j]
                assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (l, i, j, fd, an)
    assert all(np.abs(Y).max() > 1e-4 for Y in out["Y"])     # the check is not vacuous


def test_backward_recurrence_matches_dense_python():
    A, At, H0, y, Ws = tiny_problem(directed=True, dims=(4, 3, 2))
    out = oracle.epoch(A, At, H0, y, Ws)
    D = np.array(py_dense(A))
    G1 = out["G"][1]
    S = np.array(py_matmul(D.tolist(), G1.tolist()))
    Y1 = np.array(py_matmul(out["H"][1].T.tolist(), S.tolist()))
    G0 = np.array(py_matmul(S.tolist(), Ws[1].T.tolist())) * (out["Z"][0] > 0)
    np.testing.assert_allclose(out["Y"][1], Y1, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(out["G"][0], G0, rtol=1e-12, atol=1e-15)


def test_backward_with_imposed_sign_pattern_matches_dense_python():
    """Equation 2 with sigma' taken from a sign pattern the caller imposes (what the GPU parity tests do with
    the GPU's own pre-activations): the same dense recurrence with that pattern; the forward pass, the loss
    and the last layer's gradient do not depend on it; the oracle's own Z as the pattern changes nothing."""
    A, At, H0, y, Ws = tiny_problem(directed=True, dims=(4, 3, 3, 2))
    base = oracle.epoch(A, At, H0, y, Ws)
    same = oracle.epoch(A, At, H0, y, Ws, sign_from=[base["Z"][0], base["H"][2]])   # H = ReLU(Z): same signs
    for l in range(3):
        np.testing.assert_array_equal(same["Y"][l], base["Y"][l])
    P = [synth.normal_features(A.n, 3, 77).astype(np.float64), None]                 # layer 1 imposed, layer 2 own
    assert ((P[0] > 0) != (base["Z"][0] > 0)).sum() > 10
    out = oracle.epoch(A, At, H0, y, Ws, sign_from=P)
    assert out["loss"] == base["loss"]
    for l in range(3):
        np.testing.assert_array_equal(out["Z"][l], base["Z"][l])
    np.testing.assert_array_equal(out["G"][2], base["G"][2])
    np.testing.assert_array_equal(out["G"][1], base["G"][1])
    np.testing.assert_array_equal(out["Y"][1], base["Y"][1])
    D = np.array(py_dense(A))
    S = np.array(py_matmul(D.tolist(), base["G"][1].tolist()))
    G0 = np.array(py_matmul(S.tolist(), Ws[1].T.tolist())) * (P[0] > 0)
    np.testing.assert_allclose(out["G"][0], G0, rtol=1e-12, atol=1e-15)
    S0 = np.array(py_matmul(D.tolist(), G0.tolist()))
    np.testing.assert_allclose(out["Y"][0], np.array(py_matmul(H0.T.tolist(), S0.tolist())), rtol=1e-12, atol=1e-15)
    assert np.abs(out["Y"][0] - base["Y"][0]).max() > 1e-6                           # the pattern is really used


def test_layer_backward_bias_gradient():
    A, At, H0, y, Ws = tiny_problem(False, dims=(4, 3))
    G = synth.normal_features(A.n, 3, 12).astype(np.float64)
    _, _, _, db = oracle.layer_backward(A, H0, None, Ws[0], G)
    np.testing.assert_allclose(db, [math.fsum(G[:, j].tolist()) for j in range(3)], rtol=1e-13)
    b = np.array([0.5, -1.0, 2.0])
    Z0, _ = oracle.layer_forward(At, H0, Ws[0], "none")
    Zb, Hb = oracle.layer_forward(At, H0, Ws[0], "relu", bias=b)
    np.testing.assert_allclose(Zb, Z0 + b[None, :], rtol=1e-15)
    np.testing.assert_array_equal(Hb, np.maximum(Zb, 0))


def test_sgd_epoch_reduces_loss():
    A, At, H0, y, Ws = tiny_problem(False)
    first = oracle.epoch(A, At, H0, y, Ws, lr=0.5)
    second = oracle.epoch(A, At, H0, y, first["W"], lr=0.0)
    assert second["loss"] < first["loss"]
    for W, Y, Wn in zip(Ws, first["Y"], first["W"]):
        np.testing.assert_allclose(Wn, W - 0.5 * Y, rtol=1e-15)


def test_config1_loss_near_log_classes_at_init():
    w = synth.CONFIGS[1]
    n, src, dst = synth.make_graph(w)
    A = oracle.build_csr(n, src, dst)
    H0, y, Ws = synth.make_model_inputs(w)
    out = oracle.epoch(A, A, H0, y, Ws)
    assert abs(out["loss"] - math.log(8)) < 0.1
    assert A.nnz == int(A.deg.sum()) and 60_000 < A.nnz < 72_000


def test_float_build_rounds_once():
    """The float build equals the double build rounded to float, for each primitive."""
    n, src, dst = small_graph(50, 300, 23)
    A = oracle.build_csr(n, src, dst)
    X = synth.normal_features(n, 8, 10)
    np.testing.assert_array_equal(oracle.spmm(A, X), oracle.spmm(A, X.astype(np.float64)).astype(np.float32))
    W = synth.glorot_weights((8, 5), 1)[0]
    np.testing.assert_array_equal(oracle.gemm(X, W), oracle.gemm(X.astype(np.float64), W.astype(np.float64)).astype(np.float32))
