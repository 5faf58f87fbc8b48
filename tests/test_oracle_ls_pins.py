"""Pins for the oracle's stacked least-squares solve (paper Eq. 4) against things other than itself: a system
solved by hand, the closed form for orthonormal columns, the vanishing normal-equation residual, the explicit
inverse of the normal matrix on a small case, and the property the paper builds the join on: the replicas of an
exactly low-rank tensor carry U_p A, from which the solve returns A."""
import numpy as np

import oracle


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_by_hand():
    # one unknown, two equations: x = 1, 2x = 3  ->  x = (1*1 + 2*3) / (1 + 4)
    Us = np.array([[[1.0]], [[2.0]]])  # P=2, L=1, I=1
    X = oracle.stacked_ls(Us, np.array([[1.0], [3.0]]))
    assert X.shape == (1, 1) and abs(X[0, 0] - 1.4) < 1e-15
    # two unknowns, three equations with a known residual: columns e1, e2 padded by a zero row
    Us = np.array([[[1.0, 0.0]], [[0.0, 2.0]], [[0.0, 0.0]]])
    X = oracle.stacked_ls(Us, np.array([[3.0, -1.0], [4.0, 6.0], [7.0, 7.0]]))
    assert np.allclose(X, [[3.0, -1.0], [2.0, 3.0]], rtol=0, atol=1e-15)


def test_orthonormal_columns_closed_form():
    P, L, I, R = 4, 6, 9, 3
    Q = np.linalg.qr(_rand(0, P * L, I))[0]  # orthonormal columns: the minimiser is Q^T A
    A = _rand(1, P * L, R)
    X = oracle.stacked_ls(Q.reshape(P, L, I), A)
    assert np.abs(X - Q.T @ A).max() < 1e-13


def test_normal_equations_and_explicit_inverse():
    P, L, I, R = 5, 4, 7, 3
    Us = _rand(2, P, L, I)
    A = _rand(3, P * L, R)
    X = oracle.stacked_ls(Us, A)
    U = np.concatenate([Us[p] for p in range(P)], axis=0)  # replica p occupies rows p*L .. p*L+L-1
    assert np.abs(U.T @ (U @ X - A)).max() < 1e-12
    assert np.abs(X - np.linalg.inv(U.T @ U) @ (U.T @ A)).max() < 1e-11
    # a transposed or mis-stacked operand fails: swapping two replicas' rows of A changes the answer
    A2 = A.copy()
    A2[:L], A2[L:2 * L] = A[L:2 * L], A[:L]
    assert np.abs(oracle.stacked_ls(Us, A2) - X).max() > 1e-3


def test_replicas_of_a_low_rank_tensor_return_its_factor():
    # X = a o b o c (rank 1).  Its replica Y_p = X x1 U_p x2 V_p x3 W_p is (U_p a) o (V_p b) o (W_p c)
    # (the Kronecker property the decomposition stage rests on), so the first mode-1 fibre of Y_p divided
    # by (V_p b)[0] (W_p c)[0] is U_p a, and the stacked solve returns a.
    I, J, K, L, M, N, P = 10, 9, 8, 4, 3, 3, 3  # P*L = 12 >= I
    a, b, c = _rand(4, I), _rand(5, J), _rand(6, K)
    X = np.einsum("i,j,k->ijk", a, b, c).astype(np.float32)
    Us, Vs, Ws = (_rand(7, P, L, I).astype(np.float32), _rand(8, P, M, J).astype(np.float32),
                  _rand(9, P, N, K).astype(np.float32))
    Y = oracle.comp_multi(X, Us.reshape(P * L, I), Vs.reshape(P * M, J), Ws.reshape(P * N, K), P)
    rows = []  # Y is (L, M, N, P)
    for p in range(P):
        scale = (Vs[p].astype(np.float64) @ b)[0] * (Ws[p].astype(np.float64) @ c)[0]
        rows.append(Y[:, 0, 0, p] / scale)
    got = oracle.stacked_ls(Us, np.concatenate(rows)[:, None])[:, 0]
    assert np.abs(got - a).max() <= 2e-5 * np.abs(a).max()  # X and Y are rounded to fp32 on the way
