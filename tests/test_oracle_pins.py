"""Pins for the fp64 CPU checker (``oracle/``): it is compared with things other than itself.

* exact rational brute force on tiny dense operands (non-symmetric, empty row, full row/column),
* a hand-worked 3 x 3 product and the 3 x 3 grid fixture under ``tests/golden``,
* operands whose product is known bit for bit (identity, permutation, diagonal, unit vectors),
* closed forms (row-stochastic operand, grid operator row sums and sine eigenvectors, powers),
* a library CSR product (scipy) in float64.

A dropped term, a wrong sign, a transposed operand or an off-by-one in the row pointers fails
at least one of these.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2307_05740_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_csr(rng, n, density, full_row=None, full_col=None, empty_row=None):
    M = (rng.random((n, n)) < density)
    if full_row is not None:
        M[full_row, :] = True
    if full_col is not None:
        M[:, full_col] = True
    if empty_row is not None:
        M[empty_row, :] = False
    V = np.where(M, rng.uniform(-1, 1, (n, n)), 0.0).astype(np.float32)
    rowptr = np.zeros(n + 1, np.int64)
    cols, vals = [], []
    for i in range(n):
        for j in range(n):
            if M[i, j]:
                cols.append(j)
                vals.append(V[i, j])
        rowptr[i + 1] = len(cols)
    return rowptr, np.array(cols, np.int32), np.array(vals, np.float32), V


def exact_product(V, X):
    """Y and |A||X| in exact rational arithmetic from the dense fp32 arrays."""
    n, k = X.shape
    Y = [[Fraction(0)] * k for _ in range(n)]
    B = [[Fraction(0)] * k for _ in range(n)]
    for i in range(n):
        for j in range(n):
            a = Fraction(float(V[i, j]))
            if a == 0:
                continue
            for c in range(k):
                x = Fraction(float(X[j, c]))
                Y[i][c] += a * x
                B[i][c] += abs(a) * abs(x)
    return Y, B


@pytest.mark.parametrize("n,k,density,seed", [(7, 3, 0.4, 1), (33, 5, 0.15, 2), (64, 4, 0.3, 3)])
def test_brute_force_exact_rational(n, k, density, seed):
    rng = np.random.default_rng(seed)
    rowptr, colidx, vals, V = random_csr(rng, n, density, full_row=1, full_col=2, empty_row=n - 1)
    X = rng.standard_normal((n, k)).astype(np.float32)
    Y, B = oracle.spmm(rowptr, colidx, vals, X)
    Ye, Be = exact_product(V, X)
    u = 2.0 ** -53
    for i in range(n):
        for c in range(k):
            # fp64 recursive summation of m exactly-representable products: error <= m*u*B
            assert abs(Fraction(Y[i, c]) - Ye[i][c]) <= Fraction(n * u) * Be[i][c]
            assert abs(Fraction(B[i, c]) - Be[i][c]) <= Fraction(n * u) * Be[i][c]
    assert np.all(Y[n - 1] == 0) and np.all(B[n - 1] == 0)      # the empty row


def test_transposed_operand_is_detected():
    """The brute force distinguishes A from its transpose (operand is not symmetric)."""
    rng = np.random.default_rng(11)
    rowptr, colidx, vals, V = random_csr(rng, 16, 0.3)
    X = rng.standard_normal((16, 2)).astype(np.float32)
    Y, _ = oracle.spmm(rowptr, colidx, vals, X)
    assert np.allclose(Y, V.astype(np.float64) @ X.astype(np.float64), rtol=0, atol=1e-12)
    assert not np.allclose(Y, V.T.astype(np.float64) @ X.astype(np.float64), atol=1e-3)


def test_golden_hand_3x3():
    rec = {}
    for line in open(os.path.join(GOLDEN, "hand_3x3_product.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *nums = line.split()
        rec[name] = np.array([float(t) for t in nums])
    X = rec["X"].reshape(3, 2).astype(np.float32)
    Y, B = oracle.spmm(rec["A_rowptr"].astype(np.int64), rec["A_colidx"].astype(np.int32),
                       rec["A_vals"].astype(np.float32), X)
    assert np.array_equal(Y, rec["Y"].reshape(3, 2))
    assert np.array_equal(B, rec["B"].reshape(3, 2))


def test_golden_grid3_times_ones():
    want = np.loadtxt(os.path.join(GOLDEN, "grid3_times_ones.txt")).reshape(9, 1)
    rp, ci = synth.grid5_pattern(3)
    Y, B = oracle.spmm(rp, ci, synth.fill_grid5(rp, ci), np.ones((9, 1), np.float32))
    assert np.array_equal(Y, want)
    assert np.array_equal(B, 8.0 - want)          # |A| row sums: 4 + number of neighbours


def test_identity_permutation_diagonal_bitwise():
    rng = np.random.default_rng(5)
    n, k = 50, 6
    X = rng.standard_normal((n, k)).astype(np.float32)
    rp = np.arange(n + 1, dtype=np.int64)
    ones = np.ones(n, np.float32)
    Y, B = oracle.spmm(rp, np.arange(n, dtype=np.int32), ones, X)
    assert np.array_equal(Y, X.astype(np.float64)) and np.array_equal(B, np.abs(X, dtype=np.float64))
    perm = rng.permutation(n).astype(np.int32)
    Y, _ = oracle.spmm(rp, perm, ones, X)               # row i holds a 1 in column perm[i]
    assert np.array_equal(Y, X[perm].astype(np.float64))
    d = rng.uniform(-2, 2, n).astype(np.float32)
    Y, _ = oracle.spmm(rp, np.arange(n, dtype=np.int32), d, X)
    assert np.array_equal(Y, d.astype(np.float64)[:, None] * X.astype(np.float64))  # exact in fp64


def test_unit_vector_columns_give_columns_of_A():
    rng = np.random.default_rng(6)
    n = 24
    rowptr, colidx, vals, V = random_csr(rng, n, 0.25)
    Y, _ = oracle.spmm(rowptr, colidx, vals, np.eye(n, dtype=np.float32))
    assert np.array_equal(Y, V.astype(np.float64))


def test_row_stochastic_times_ones():
    rp, ci = synth.rmat_pattern(10, 8 << 10, seed=3)
    vals = synth.fill_row_normalized(rp)
    n = rp.shape[0] - 1
    nonempty = np.diff(rp) > 0
    Y, B = oracle.spmm(rp, ci, vals, np.ones((n, 2), np.float32))
    assert np.allclose(Y[nonempty], 1.0, rtol=0, atol=2e-7) and np.all(Y[~nonempty] == 0)
    assert np.array_equal(Y, B)                      # all terms are non-negative
    Xl, El = oracle.spmm_iter(rp, ci, vals, np.ones((n, 2), np.float32), 4)
    reach = Xl[:, 0] != 0                            # rows whose walks never hit an empty row
    assert np.allclose(Xl[reach & nonempty], 1.0, rtol=0, atol=1e-6)


@pytest.mark.parametrize("N,p,q", [(8, 1, 1), (12, 2, 5), (17, 17, 3)])
def test_grid_operator_sine_eigenvectors_and_powers(N, p, q):
    rp, ci = synth.grid5_pattern(N)
    vals = synth.fill_grid5(rp, ci)
    xs = np.arange(1, N + 1)
    v = np.outer(np.sin(np.pi * q * xs / (N + 1)), np.sin(np.pi * p * xs / (N + 1))).reshape(-1, 1)
    lam = 4 - 2 * np.cos(np.pi * p / (N + 1)) - 2 * np.cos(np.pi * q / (N + 1))
    v32 = v.astype(np.float32)
    Y, B = oracle.spmm(rp, ci, vals, v32)
    # v32 differs from the eigenvector by fp32 rounding only: residual <= |A| * 2^-24 per term
    assert np.all(np.abs(Y - lam * v32.astype(np.float64)) <= 2.0 ** -23 * (B + 1e-30) + 1e-12)
    for l in (0, 1, 2, 5):
        Xl, El = oracle.spmm_iter(rp, ci, vals, v32, l)
        assert np.all(np.abs(Xl - lam ** l * v32.astype(np.float64)) <= 2.0 ** -22 * El + 1e-12), l
        assert np.all(El >= np.abs(Xl) - 1e-12)


def test_library_csr_product_and_iterates():
    w = synth.make_config(0)                          # R-MAT scale 12, uniform values
    X = w.make_x()
    A = sp.csr_matrix((w.vals.astype(np.float64), w.colidx, w.rowptr), shape=(w.n, w.n))
    Y, B = oracle.spmm(w.rowptr, w.colidx, w.vals, X)
    Ylib = A @ X.astype(np.float64)
    Blib = abs(A) @ np.abs(X.astype(np.float64))
    assert np.all(np.abs(Y - Ylib) <= 1e-13 * Blib)
    assert np.all(np.abs(B - Blib) <= 1e-13 * Blib)
    Xl, El = oracle.spmm_iter(w.rowptr, w.colidx, w.vals, X, 3)
    assert np.all(np.abs(Xl - A @ (A @ Ylib)) <= 1e-12 * (abs(A) @ (abs(A) @ Blib)))
    assert np.all(np.abs(El - abs(A) @ (abs(A) @ Blib)) <= 1e-12 * El)


def test_row_selection_and_column_slice_agree_with_full():
    w = synth.make_config(0)
    X = w.make_x()
    Y, B = oracle.spmm(w.rowptr, w.colidx, w.vals, X)
    rows = np.array([0, 5, 4095, 17, 17], np.int64)
    Ys, Bs = oracle.spmm(w.rowptr, w.colidx, w.vals, X, rows=rows, c0=3, kc=7)
    assert np.array_equal(Ys, Y[rows, 3:10]) and np.array_equal(Bs, B[rows, 3:10])
    X0, E0 = oracle.spmm_iter(w.rowptr, w.colidx, w.vals, X, 0)
    assert np.array_equal(X0, X.astype(np.float64)) and np.array_equal(E0, np.abs(X0))
    X1, E1 = oracle.spmm_iter(w.rowptr, w.colidx, w.vals, X, 1)
    assert np.array_equal(X1, Y) and np.array_equal(E1, B)


def test_linearity_and_symmetry_identities():
    w = synth.make_config(0, shrink=2)
    X = w.make_x()
    A = (w.rowptr, w.colidx, w.vals)
    Y, B = oracle.spmm(*A, X)
    X2 = synth.normal_matrix(w.n, w.k, seed=99)
    Y2, B2 = oracle.spmm(*A, X2)
    # the pattern is symmetric but the values are not: use A + A^T through both products
    M = sp.csr_matrix((w.vals.astype(np.float64), w.colidx, w.rowptr), shape=(w.n, w.n))
    lhs = np.sum(X2.astype(np.float64) * Y)                 # <X2, A X>
    rhs = np.sum((M.T @ X2.astype(np.float64)) * X)         # <A^T X2, X>
    assert abs(lhs - rhs) <= 1e-10 * np.sum(B * np.abs(X2))
    Xs = (2.0 * X + X2).astype(np.float32)                  # exact? no: rounded, so use the bound
    Ys, Bs = oracle.spmm(*A, Xs)
    assert np.all(np.abs(Ys - (2 * Y + Y2)) <= 2.0 ** -22 * (2 * B + B2) + 1e-30)


# ---------------------------------------------------------------------------------------------
# sampled dense-dense product  S(i,j) = A(i,j) * sum_r U(i,r) V(j,r)
# ---------------------------------------------------------------------------------------------
def test_sddmm_exact_rational_brute_force():
    rng = np.random.default_rng(31)
    n, k = 19, 5
    rowptr, colidx, vals, Vd = random_csr(rng, n, 0.3, full_row=2, full_col=3, empty_row=7)
    U = rng.standard_normal((n, k)).astype(np.float32)
    W = rng.standard_normal((n, k)).astype(np.float32)
    S, B = oracle.sddmm(rowptr, colidx, vals, U, W)
    u = 2.0 ** -53
    p = 0
    for i in range(n):
        for j in range(n):
            if Vd[i, j] == 0 and not (rowptr[i] <= p < rowptr[i + 1] and colidx[p] == j):
                continue
            dot = sum(Fraction(float(U[i, r])) * Fraction(float(W[j, r])) for r in range(k))
            adot = sum(abs(Fraction(float(U[i, r])) * Fraction(float(W[j, r]))) for r in range(k))
            a = Fraction(float(vals[p]))
            assert colidx[p] == j
            assert abs(Fraction(S[p]) - a * dot) <= Fraction((k + 2) * u) * abs(a) * adot
            assert abs(Fraction(B[p]) - abs(a) * adot) <= Fraction((k + 2) * u) * abs(a) * adot
            p += 1
    assert p == rowptr[-1]


def test_sddmm_hand_worked_and_transposition():
    # A = [[0, 2], [-1, 0.5]], U = [[1, 2], [3, 4]], V = [[5, 6], [7, 8]]
    # U V^T = [[17, 23], [39, 53]]  ->  S = [2*23, -1*39, 0.5*53] = [46, -39, 26.5]
    rowptr = np.array([0, 1, 3], np.int64)
    colidx = np.array([1, 0, 1], np.int32)
    vals = np.array([2, -1, 0.5], np.float32)
    U = np.array([[1, 2], [3, 4]], np.float32)
    V = np.array([[5, 6], [7, 8]], np.float32)
    S, B = oracle.sddmm(rowptr, colidx, vals, U, V)
    assert np.array_equal(S, [46.0, -39.0, 26.5]) and np.array_equal(B, [46.0, 39.0, 26.5])
    St, _ = oracle.sddmm(rowptr, colidx, vals, V, U)          # swapping U and V is a different product
    # V U^T = (U V^T)^T = [[17, 39], [23, 53]]
    assert np.array_equal(St, [2 * 39.0, -1 * 23.0, 0.5 * 53.0])


def test_sddmm_closed_forms_and_library():
    w = synth.make_config(0, shrink=2)
    n, k = w.n, 7
    A = sp.csr_matrix((w.vals.astype(np.float64), w.colidx, w.rowptr), shape=(n, n))
    ones = np.ones((n, k), np.float32)
    S, B = oracle.sddmm(w.rowptr, w.colidx, w.vals, ones, ones)
    assert np.array_equal(S, k * w.vals.astype(np.float64)) and np.array_equal(B, k * np.abs(w.vals, dtype=np.float64))
    U = synth.normal_matrix(n, k, seed=5)
    V = synth.normal_matrix(n, k, seed=6)
    S, B = oracle.sddmm(w.rowptr, w.colidx, w.vals, U, V)
    D = U.astype(np.float64) @ V.astype(np.float64).T
    rows = np.repeat(np.arange(n), np.diff(w.rowptr))
    want = w.vals.astype(np.float64) * D[rows, w.colidx]
    assert np.all(np.abs(S - want) <= 1e-13 * B)
    assert np.allclose(A.multiply(D).tocsr().data, S, rtol=0, atol=1e-12)     # library: elementwise product
    # identity operand with U = V: squared row norms; unit-vector factors pick single products
    rp = np.arange(n + 1, dtype=np.int64)
    Sd, _ = oracle.sddmm(rp, np.arange(n, dtype=np.int32), np.ones(n, np.float32), U, U)
    assert np.allclose(Sd, np.sum(U.astype(np.float64) ** 2, axis=1), rtol=1e-15)
    E = np.zeros((n, k), np.float32); E[:, 2] = 1
    S2, _ = oracle.sddmm(w.rowptr, w.colidx, w.vals, U, E)                    # S = a_ij * U[i, 2]
    assert np.array_equal(S2, w.vals.astype(np.float64) * U[rows, 2].astype(np.float64))
    # consistency with the product kernel: row sums of S equal (A .* (U V^T)) 1 = diag-free identity
    Y, _ = oracle.spmm(w.rowptr, w.colidx, w.vals, V)                         # A V
    lhs = np.add.reduceat(np.concatenate([S, [0.0]]), np.minimum(w.rowptr[:-1], len(S)))[:n]
    lhs[np.diff(w.rowptr) == 0] = 0.0
    assert np.all(np.abs(lhs - np.sum(U.astype(np.float64) * Y, axis=1)) <= 1e-11 * (1 + np.abs(lhs)))


# ---------------------------------------------------------------------------------------------
# order-3 MTTKRP  A(i,a) = sum_{j,k} T(i,j,k) B(j,a) C(k,a)
# ---------------------------------------------------------------------------------------------
def random_tensor(rng, dims, density):
    I, J, K = dims
    M = rng.random(dims) < density
    i, j, k = np.nonzero(M)                                   # sorted by (i, j, k)
    v = rng.uniform(-1, 1, len(i)).astype(np.float32)
    return i.astype(np.int32), j.astype(np.int32), k.astype(np.int32), v


def test_mttkrp_golden_hand_2x2x2():
    rec = {}
    for line in open(os.path.join(GOLDEN, "hand_2x2x2_mttkrp.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *nums = line.split()
        rec[name] = np.array([float(t) for t in nums])
    A, E = oracle.mttkrp((2, 2, 2), rec["T_i"], rec["T_j"], rec["T_k"], rec["T_v"],
                         rec["B"].reshape(2, 2).astype(np.float32), rec["C"].reshape(2, 2).astype(np.float32))
    assert np.array_equal(A, rec["A"].reshape(2, 2)) and np.array_equal(E, rec["E"].reshape(2, 2))


def test_mttkrp_exact_rational_brute_force():
    rng = np.random.default_rng(41)
    dims, R = (4, 5, 3), 3
    i, j, k, v = random_tensor(rng, dims, 0.4)
    B = rng.standard_normal((dims[1], R)).astype(np.float32)
    C = rng.standard_normal((dims[2], R)).astype(np.float32)
    A, E = oracle.mttkrp(dims, i, j, k, v, B, C)
    u = 2.0 ** -53
    for ii in range(dims[0]):
        for a in range(R):
            s = Fraction(0); e = Fraction(0)
            for p in range(len(v)):
                if i[p] == ii:
                    t = Fraction(float(v[p])) * Fraction(float(B[j[p], a])) * Fraction(float(C[k[p], a]))
                    s += t; e += abs(t)
            m = dims[1] * dims[2]
            assert abs(Fraction(A[ii, a]) - s) <= Fraction((m + 3) * u) * e
            assert abs(Fraction(E[ii, a]) - e) <= Fraction((m + 3) * u) * e


def test_mttkrp_library_contraction_and_pairwise_form():
    rng = np.random.default_rng(42)
    dims, R = (13, 9, 11), 6
    i, j, k, v = random_tensor(rng, dims, 0.2)
    B = rng.standard_normal((dims[1], R)).astype(np.float32)
    C = rng.standard_normal((dims[2], R)).astype(np.float32)
    A, E = oracle.mttkrp(dims, i, j, k, v, B, C)
    T = np.zeros(dims); T[i, j, k] = v
    want = np.einsum("ijk,ja,ka->ia", T, B.astype(np.float64), C.astype(np.float64))
    assert np.all(np.abs(A - want) <= 1e-13 * E + 1e-300)
    assert np.all(np.abs(E - np.einsum("ijk,ja,ka->ia", np.abs(T), np.abs(B, dtype=np.float64), np.abs(C, dtype=np.float64))) <= 1e-13 * E)
    # the pairwise (factorized) evaluation gives the same result: X(i,j,a) = sum_k T C, A = sum_j X B
    X = np.einsum("ijk,ka->ija", T, C.astype(np.float64))
    assert np.all(np.abs(A - np.einsum("ija,ja->ia", X, B.astype(np.float64))) <= 1e-13 * E + 1e-300)
    # the entry order of the list does not matter beyond rounding (unsorted lists run on one thread)
    perm = rng.permutation(len(v))
    A2, E2 = oracle.mttkrp(dims, i[perm], j[perm], k[perm], v[perm], B, C)
    assert np.all(np.abs(A2 - A) <= 1e-13 * E + 1e-300)


def test_mttkrp_closed_forms():
    rng = np.random.default_rng(43)
    I, J, K, R = 6, 7, 5, 4
    B = rng.standard_normal((J, R)).astype(np.float32)
    C = rng.standard_normal((K, R)).astype(np.float32)
    # all-ones dense tensor: A(i,a) = (sum_j B(j,a)) (sum_k C(k,a))
    ii, jj, kk = np.meshgrid(np.arange(I), np.arange(J), np.arange(K), indexing="ij")
    A, _ = oracle.mttkrp((I, J, K), ii.ravel(), jj.ravel(), kk.ravel(), np.ones(I * J * K, np.float32), B, C)
    want = B.astype(np.float64).sum(0) * C.astype(np.float64).sum(0)
    assert np.allclose(A, np.broadcast_to(want, (I, R)), rtol=1e-12, atol=1e-12)
    # indicator factors: B = ones, C = identity (K = R) -> A(i,a) = sum_j T(i,j,a), exactly
    i, j, k, v = random_tensor(rng, (I, J, R), 0.5)
    A, E = oracle.mttkrp((I, J, R), i, j, k, v, np.ones((J, R), np.float32), np.eye(R, dtype=np.float32))
    T = np.zeros((I, J, R)); T[i, j, k] = v
    assert np.allclose(A, T.sum(1), rtol=0, atol=1e-15) and np.allclose(E, np.abs(T).sum(1), rtol=0, atol=1e-15)


def test_mttkrp_reduces_to_the_matrix_product_when_K_is_1():
    """K = 1 and C = ones: A = T_(IxJ) . B, the order-2 kernel -- checked against the other checker."""
    w = synth.make_config(0, shrink=3)
    rows = np.repeat(np.arange(w.n), np.diff(w.rowptr)).astype(np.int32)
    B = synth.normal_matrix(w.n, 5, seed=9)
    A, E = oracle.mttkrp((w.n, w.n, 1), rows, w.colidx, np.zeros(w.nnz, np.int32), w.vals, B, np.ones((1, 5), np.float32))
    Y, Bd = oracle.spmm(w.rowptr, w.colidx, w.vals, B)
    assert np.array_equal(A, Y) and np.array_equal(E, Bd)


def test_mttkrp_swapping_modes_and_factors():
    rng = np.random.default_rng(44)
    dims, R = (5, 6, 6), 3
    i, j, k, v = random_tensor(rng, dims, 0.3)
    B = rng.standard_normal((6, R)).astype(np.float32)
    C = rng.standard_normal((6, R)).astype(np.float32)
    A, E = oracle.mttkrp(dims, i, j, k, v, B, C)
    A_sw, _ = oracle.mttkrp(dims, i, k, j, v, C, B)          # swap the roles of j and k consistently
    assert np.all(np.abs(A_sw - A) <= 1e-13 * E + 1e-300)
    A_bad, _ = oracle.mttkrp(dims, i, j, k, v, C, B)         # factors swapped, indices not
    assert not np.allclose(A_bad, A, atol=1e-3)
    with pytest.raises(RuntimeError):
        oracle.mttkrp(dims, i, j, k + 1, v, B, C)            # an index out of range


def test_tensor_generator_is_seeded_sorted_and_deduplicated():
    a = synth.make_tensor_config(0, shrink=5)
    b = synth.make_tensor_config(0, shrink=5)
    assert all(np.array_equal(x, y) for x, y in zip((a.i, a.j, a.k, a.vals), (b.i, b.j, b.k, b.vals)))
    key = (a.i.astype(np.int64) * a.dims[1] + a.j) * a.dims[2] + a.k
    assert np.all(np.diff(key) > 0)
    assert 0.9e-3 < a.nnz / np.prod([float(d) for d in a.dims]) < 1.1e-3
    assert np.all(np.abs(a.vals) <= 1) and abs(float(a.vals.mean())) < 0.05
    s = synth.make_tensor_config(1, shrink=5)
    sl = np.bincount(s.i, minlength=s.dims[0])
    assert sl.max() > 50 * max(1.0, sl.mean()) and (sl == 0).sum() > 0.3 * s.dims[0]   # hub slices, empty slices
