"""Pins for the dense CPU oracle (Eq. 1, Eq. 2, transpose of Section III).

The paper prints no worked numeric product, so the oracle is pinned by what the
definitions fix: hand-expanded sums, exact integer arithmetic, identities, closed
forms, and an independent library routine.  A dropped term, a swapped index or a
transposed operand fails at least one of these.
"""
import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import inputs as I


def test_nt_1x1x1_and_hand_expanded_2x3x4():
    assert oracle.nt_ref(np.array([[3.0]], np.float32), np.array([[-2.0]], np.float32))[0, 0] == -6.0
    A = np.array([[1, 2, 3, 4], [5, 6, 7, 8]], np.float32)                   # 2 x 4
    B = np.array([[1, 0, -1, 2], [3, 1, 0, -2], [0.5, 0.25, 2, 1]], np.float32)  # 3 x 4
    C = oracle.nt_ref(A, B)
    want = [[1 * 1 + 2 * 0 + 3 * -1 + 4 * 2, 1 * 3 + 2 * 1 + 3 * 0 + 4 * -2, 1 * .5 + 2 * .25 + 3 * 2 + 4 * 1],
            [5 * 1 + 6 * 0 + 7 * -1 + 8 * 2, 5 * 3 + 6 * 1 + 7 * 0 + 8 * -2, 5 * .5 + 6 * .25 + 7 * 2 + 8 * 1]]
    assert C.tolist() == want
    # not symmetric in its operands: NT(B, A) is the 3 x 2 transpose
    assert oracle.nt_ref(B, A).tolist() == np.array(want).T.tolist()


def test_nn_hand_expanded_2x3x2():
    A = np.array([[1, 2], [3, 4]], np.float32)           # 2 x 2
    B = np.array([[5, 6, 7], [8, 9, 10]], np.float32)    # 2 x 3 (k x n)
    want = [[1 * 5 + 2 * 8, 1 * 6 + 2 * 9, 1 * 7 + 2 * 10], [3 * 5 + 4 * 8, 3 * 6 + 4 * 9, 3 * 7 + 4 * 10]]
    assert oracle.nn_ref(A, B).tolist() == want


@pytest.mark.parametrize("m,n,k", [(7, 5, 9), (33, 65, 130), (1, 17, 1), (64, 1, 300)])
def test_integer_inputs_match_exact_integer_arithmetic(m, n, k):
    A = I.small_integers(11, 0, m, k)
    B = I.small_integers(11, 1, n, k)
    exact_nt = A.astype(np.int64) @ B.astype(np.int64).T
    assert np.array_equal(oracle.nt_ref(A, B), exact_nt.astype(np.float64))
    Bt = I.small_integers(11, 2, k, n)
    exact_nn = A.astype(np.int64) @ Bt.astype(np.int64)
    assert np.array_equal(oracle.nn_ref(A, Bt), exact_nn.astype(np.float64))


def test_transposed_product_identity_is_bit_exact():
    # (A B^T)^T = B A^T: same products, same order of summation -> identical doubles
    A, B = I.nt_operands(37, 29, 101, 5)
    assert np.array_equal(oracle.nt_ref(A, B).T, oracle.nt_ref(B, A))


def test_nt_equals_nn_of_transposed_b_bit_exact():
    # the TNN claim (Section III): NT(A, B) = NN(A, transpose(B))
    A, B = I.nt_operands(40, 23, 77, 6, dist="normal")
    C, S = oracle.nt_ref(A, B, with_bound=True)
    C2, S2 = oracle.tnn_ref(A, B, with_bound=True)
    assert np.array_equal(C, C2) and np.array_equal(S, S2)


def test_identity_and_permutation():
    A = I.uniform_pm1(7, 0, 19, 12)
    eye = np.eye(12, dtype=np.float32)
    assert np.array_equal(oracle.nt_ref(A, eye), A.astype(np.float64))
    assert np.array_equal(oracle.nn_ref(A, eye), A.astype(np.float64))
    perm = np.array([3, 0, 11, 5, 1, 2, 4, 10, 9, 8, 7, 6])
    P = eye[perm]                      # row j of P selects column perm[j]
    assert np.array_equal(oracle.nt_ref(A, P), A[:, perm].astype(np.float64))
    # NN with P: C[:, j] = sum_l A[:, l] P[l, j] -> column j takes A[:, l] where perm[l] == j
    inv = np.argsort(perm)
    assert np.array_equal(oracle.nn_ref(A, P), A[:, inv].astype(np.float64))


def test_rank_one_closed_form():
    u = np.array([1.5, -2.0, 0.25], np.float32)
    v = np.array([4.0, -0.5], np.float32)
    k = 50
    A = np.repeat(u[:, None], k, axis=1)
    B = np.repeat(v[:, None], k, axis=1)
    assert np.array_equal(oracle.nt_ref(A, B), k * np.outer(u, v).astype(np.float64))


def test_against_library_matmul_and_bound():
    A, B = I.nt_operands(50, 60, 333, 8, dist="normal")
    C, S = oracle.nt_ref(A, B, with_bound=True)
    lib = A.astype(np.float64) @ B.astype(np.float64).T
    assert np.max(np.abs(C - lib) / S) < 1e-14
    libS = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64).T
    assert np.max(np.abs(S - libS) / S) < 1e-14
    assert np.all(S >= np.abs(C))
    Bt = np.ascontiguousarray(B.T)
    assert np.max(np.abs(oracle.nn_ref(A, Bt) - lib) / S) < 1e-14


def test_linearity_in_b():
    A = I.uniform_pm1(9, 0, 11, 40)
    B1 = I.small_integers(9, 1, 13, 40)
    B2 = I.small_integers(9, 2, 13, 40)
    lhs = oracle.nt_ref(A, (B1 + B2).astype(np.float32))     # integer sums are exact in fp32
    rhs = oracle.nt_ref(A, B1) + oracle.nt_ref(A, B2)
    assert np.max(np.abs(lhs - rhs)) < 1e-12


def test_leading_dimensions_and_nan_padding_are_ignored():
    A, B = I.nt_operands(9, 6, 14, 10)
    Ap = I.with_leading_dim(A, 17)[:, :14]
    Bp = I.with_leading_dim(B, 20)[:, :14]
    assert np.array_equal(oracle.nt_ref(Ap, Bp), oracle.nt_ref(A, B))
    Bt = I.with_leading_dim(np.ascontiguousarray(B.T), 11)[:, :6]
    assert np.array_equal(oracle.nn_ref(Ap, Bt), oracle.nt_ref(A, B))


def test_row_subset():
    A, B = I.nt_operands(30, 8, 21, 12)
    full = oracle.nt_ref(A, B)
    rows = [29, 0, 7, 7]
    assert np.array_equal(oracle.nt_ref(A, B, rows=rows), full[rows])
    assert np.array_equal(oracle.nn_ref(A, np.ascontiguousarray(B.T), rows=rows), full[rows])


def test_degenerate_sizes():
    A = np.zeros((3, 0), np.float32)
    B = np.zeros((4, 0), np.float32)
    assert np.array_equal(oracle.nt_ref(A, B), np.zeros((3, 4)))          # empty sum
    assert oracle.nt_ref(np.zeros((0, 5), np.float32), np.zeros((4, 5), np.float32)).shape == (0, 4)
    assert oracle.nt_ref(np.zeros((2, 5), np.float32), np.zeros((0, 5), np.float32)).shape == (2, 0)


# ---- transpose

def test_transpose_by_index_formula_small():
    X = np.arange(35, dtype=np.float32).reshape(5, 7)
    T = oracle.transpose_ref(X)
    assert T.shape == (7, 5)
    for r in range(5):
        for c in range(7):
            assert T[c, r] == X[r, c]


def test_transpose_index_coded_and_involution_bit_exact():
    X = I.index_coded(67, 130)
    T = oracle.transpose_ref(X)
    r = np.arange(67, dtype=np.float32).reshape(1, -1)
    c = np.arange(130, dtype=np.float32).reshape(-1, 1)
    assert np.array_equal(T, r * 4096 + c)
    back = oracle.transpose_ref(np.ascontiguousarray(T))
    assert back.tobytes() == X.tobytes()


def test_transpose_keeps_bit_patterns():
    bits = np.array([[0x7FC00001, 0x80000000, 0xFF800000], [0x00000001, 0x7F800000, 0xFFC12345]], np.uint32)
    X = bits.view(np.float32)
    T = np.ascontiguousarray(oracle.transpose_ref(X))
    assert np.array_equal(T.view(np.uint32), bits.T)


def test_transpose_vectors_and_padding():
    row = np.arange(9, dtype=np.float32).reshape(1, 9)
    assert np.array_equal(oracle.transpose_ref(row), row.reshape(9, 1))
    col = row.reshape(9, 1)
    assert np.array_equal(oracle.transpose_ref(col), row)
    X = I.with_leading_dim(I.uniform_pm1(3, 0, 4, 6), 9)[:, :6]      # NaN-padded input
    T = oracle.transpose_ref(X, ldout=7, fill=np.float32(-7.0))
    assert np.array_equal(T, X.T) and not np.isnan(T).any()
    base = T.base if T.base is not None else T
    assert np.all(np.asarray(base)[:, 4:] == -7.0)                      # output padding untouched
    assert oracle.transpose_ref(np.zeros((0, 3), np.float32)).shape == (3, 0)


def test_float64_products_against_hand_expansion_and_an_independent_routine():
    """The double-operand products the training-step oracle uses (Eq. 2 forward, Eq. 1 backward, and
    Eq. 1 on a transposed left operand): a hand-expanded 2 x 3 x 2 case each, exact integer inputs,
    and numpy's matmul as an independent routine within fp64 rounding."""
    A = np.array([[1.0, 2.0], [3.0, 4.0]])                      # 2 x 2
    B = np.array([[5.0, 6.0], [7.0, 8.0], [9.0, 10.0]])         # 3 x 2
    assert oracle.nt_f64(A, B).tolist() == [[1 * 5 + 2 * 6, 1 * 7 + 2 * 8, 1 * 9 + 2 * 10],
                                            [3 * 5 + 4 * 6, 3 * 7 + 4 * 8, 3 * 9 + 4 * 10]]
    Bn = np.array([[5.0, 6.0, 7.0], [8.0, 9.0, 10.0]])          # 2 x 3
    assert oracle.nn_f64(A, Bn).tolist() == [[1 * 5 + 2 * 8, 1 * 6 + 2 * 9, 1 * 7 + 2 * 10],
                                             [3 * 5 + 4 * 8, 3 * 6 + 4 * 9, 3 * 7 + 4 * 10]]
    # tn: A is k x m = 2 x 2 (rows are the summed index), B is k x n = 2 x 3: C[i][j] = sum_r A[r][i] B[r][j]
    assert oracle.tn_f64(A, Bn).tolist() == [[1 * 5 + 3 * 8, 1 * 6 + 3 * 9, 1 * 7 + 3 * 10],
                                             [2 * 5 + 4 * 8, 2 * 6 + 4 * 9, 2 * 7 + 4 * 10]]
    rng = np.random.RandomState(5)
    Ai = rng.randint(-9, 10, size=(17, 23)).astype(np.float64)
    Bi = rng.randint(-9, 10, size=(11, 23)).astype(np.float64)
    assert np.array_equal(oracle.nt_f64(Ai, Bi), (Ai.astype(np.int64) @ Bi.astype(np.int64).T).astype(np.float64))
    assert np.array_equal(oracle.nn_f64(Ai, Bi.T), oracle.nt_f64(Ai, Bi))          # same terms, same order
    assert np.array_equal(oracle.tn_f64(Ai.T, Bi.T), oracle.nt_f64(Ai, Bi))
    Ar, Br = rng.normal(size=(33, 70)), rng.normal(size=(45, 70))
    bound = 70 * 2.0 ** -52 * (np.abs(Ar) @ np.abs(Br).T)
    assert (np.abs(oracle.nt_f64(Ar, Br) - Ar @ Br.T) <= bound).all()
    assert (np.abs(oracle.nn_f64(Ar, Br.T) - Ar @ Br.T) <= bound).all()
    assert (np.abs(oracle.tn_f64(Ar.T, Br.T) - Ar @ Br.T) <= bound).all()
    # the float32-operand routines are the same sums: widening the operands first changes nothing
    A32, B32 = Ar.astype(np.float32), Br.astype(np.float32)
    assert np.array_equal(oracle.nt_f64(A32, B32), oracle.nt_ref(A32, B32))
    assert oracle.nt_f64(np.zeros((0, 4)), np.zeros((3, 4))).shape == (0, 3)
