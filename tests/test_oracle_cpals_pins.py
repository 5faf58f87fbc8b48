"""Pins for the oracle's CP-ALS (paper Alg. 1) against things other than itself: the matricisations and the
Khatri-Rao product against their index definitions, every update against numpy's least-squares routine on the
explicit Khatri-Rao system and against the vanishing gradient of the fit, monotone decrease of the residual,
and recovery of an exactly low-rank tensor."""
import numpy as np

import oracle


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_unfold_and_khatri_rao_index_definitions():
    L, M, N, R = 3, 4, 5, 2
    Y = _rand(0, L, M, N)
    B, C = _rand(1, M, R), _rand(2, N, R)
    Y1, Y2, Y3 = oracle.unfold(Y, 0), oracle.unfold(Y, 1), oracle.unfold(Y, 2)
    K = oracle.khatri_rao(C, B)
    assert Y1.shape == (L, M * N) and Y2.shape == (M, L * N) and Y3.shape == (N, L * M) and K.shape == (M * N, R)
    for l in range(L):
        for m in range(M):
            for n in range(N):
                assert Y1[l, m + M * n] == Y[l, m, n] and Y2[m, l + L * n] == Y[l, m, n] and Y3[n, l + L * m] == Y[l, m, n]
    for m in range(M):
        for n in range(N):
            assert np.array_equal(K[m + M * n], C[n] * B[m])
    # the CP model in matricised form (Eq. 2): X_(1) = A (C kr B)^T
    A = _rand(3, L, R)
    assert np.allclose(oracle.unfold(oracle.cp_reconstruct(A, B, C), 0), A @ K.T, rtol=0, atol=1e-13)


def test_one_sweep_against_lstsq_and_gradient():
    L, M, N, R = 6, 5, 7, 3
    Y = _rand(10, L, M, N)
    A0, B0, C0 = _rand(11, L, R), _rand(12, M, R), _rand(13, N, R)
    A, B, C = oracle.cp_als(Y, A0, B0, C0, 1)
    # each update is the least-squares solution of the explicit Khatri-Rao system (library routine)
    A_ref = np.linalg.lstsq(oracle.khatri_rao(C0, B0), oracle.unfold(Y, 0).T, rcond=None)[0].T
    B_ref = np.linalg.lstsq(oracle.khatri_rao(C0, A_ref), oracle.unfold(Y, 1).T, rcond=None)[0].T
    C_ref = np.linalg.lstsq(oracle.khatri_rao(B_ref, A_ref), oracle.unfold(Y, 2).T, rcond=None)[0].T
    for got, ref in ((A, A_ref), (B, B_ref), (C, C_ref)):
        assert np.abs(got - ref).max() <= 1e-10 * np.abs(ref).max()
    # after the C update the gradient of ||Y - [[A,B,C]]||^2 with respect to C vanishes
    res = oracle.unfold(Y - oracle.cp_reconstruct(A, B, C), 2)
    grad = res @ oracle.khatri_rao(B, A)
    assert np.abs(grad).max() <= 1e-10 * np.abs(oracle.unfold(Y, 2)).max()


def test_residual_never_increases_and_low_rank_is_recovered():
    L, M, N, R = 8, 7, 9, 3
    At, Bt, Ct = _rand(20, L, R), _rand(21, M, R), _rand(22, N, R)
    Y = oracle.cp_reconstruct(At, Bt, Ct)
    A0, B0, C0 = _rand(23, L, R), _rand(24, M, R), _rand(25, N, R)
    prev = np.inf
    for sweeps in (1, 2, 4, 8, 16):
        A, B, C = oracle.cp_als(Y, A0, B0, C0, sweeps)
        err = np.linalg.norm(Y - oracle.cp_reconstruct(A, B, C)) / np.linalg.norm(Y)
        assert err <= prev * (1 + 1e-12)
        prev = err
    A, B, C = oracle.cp_als(Y, A0, B0, C0, 200)
    assert np.linalg.norm(Y - oracle.cp_reconstruct(A, B, C)) / np.linalg.norm(Y) <= 1e-6
    # sweeps compose: 3 sweeps = 1 sweep started from the result of 2
    A2, B2, C2 = oracle.cp_als(Y, A0, B0, C0, 2)
    A3, B3, C3 = oracle.cp_als(Y, A0, B0, C0, 3)
    A3b, B3b, C3b = oracle.cp_als(Y, A2, B2, C2, 1)
    assert np.allclose(A3, A3b) and np.allclose(B3, B3b) and np.allclose(C3, C3b)
