"""Pins for the CPU oracle's Comp (paper Sec. 3, Eq. 3) against things other than itself:
the literal six-loop definition, the Kronecker vec identity built with a library routine,
numpy's einsum, the closed form for exactly low-rank input, mode-order invariance, block
additivity, linearity and textbook special cases.  Shapes are non-cubic with all six
extents distinct so that a transposed operand or swapped index cannot pass."""
import itertools

import numpy as np
import pytest

import oracle
import workloads as wl


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def _tiny(seed=0, I=7, J=5, K=6, L=3, M=4, N=2):
    X = np.asfortranarray(_rand(seed, I, J, K))
    return X, _rand(seed + 1, L, I), _rand(seed + 2, M, J), _rand(seed + 3, N, K)


def test_mode_by_mode_equals_six_loop_definition():
    X, U, V, W = _tiny()
    Yb = oracle.comp_brute(X, U, V, W)
    Y = oracle.comp(X, U, V, W)
    assert Y.shape == (3, 4, 2)
    assert np.abs(Y - Yb).max() <= 1e-13 * np.abs(Yb).max()


def test_brute_against_hand_computed_case():
    # 2x2x2 tensor, 1x2 matrices: Y = sum_ijk u_i v_j w_k X_ijk, worked by hand.
    X = np.zeros((2, 2, 2), dtype=np.float32, order="F")
    X[0, 0, 0], X[1, 0, 0], X[0, 1, 0], X[1, 1, 0] = 1, 2, 3, 4
    X[0, 0, 1], X[1, 0, 1], X[0, 1, 1], X[1, 1, 1] = 5, 6, 7, 8
    U = np.array([[1, 10]], dtype=np.float32)
    V = np.array([[1, 100]], dtype=np.float32)
    W = np.array([[1, 1000]], dtype=np.float32)
    # = 1 + 20 + 300 + 4000 + 5000 + 60000 + 700000 + 8000000
    expect = 8769321.0
    assert oracle.comp_brute(X, U, V, W)[0, 0, 0] == expect
    assert oracle.comp(X, U, V, W)[0, 0, 0] == expect


def test_kronecker_vec_identity():
    # column-major vec: vec(X x1 U x2 V x3 W) = (W kron V kron U) vec(X)
    X, U, V, W = _tiny(seed=10, I=4, J=3, K=5, L=2, M=3, N=2)
    big = np.kron(W.astype(np.float64), np.kron(V.astype(np.float64), U.astype(np.float64)))
    y = big @ X.astype(np.float64).reshape(-1, order="F")
    Y = oracle.comp(X, U, V, W)
    assert np.abs(Y.reshape(-1, order="F") - y).max() <= 1e-12 * np.abs(y).max()


def test_against_einsum_library_routine():
    X, U, V, W = _tiny(seed=20, I=33, J=17, K=29, L=6, M=5, N=7)
    Ye = np.einsum("li,mj,nk,ijk->lmn", U.astype(np.float64), V.astype(np.float64), W.astype(np.float64),
                   X.astype(np.float64), optimize=True)
    Y = oracle.comp(X, U, V, W)
    assert np.abs(Y - Ye).max() <= 1e-12 * np.abs(Ye).max()


def test_all_six_mode_orders_agree():
    X, U, V, W = _tiny(seed=30, I=9, J=8, K=7, L=4, M=3, N=5)
    Y0 = oracle.comp(X, U, V, W)
    for order in itertools.permutations((0, 1, 2)):
        Y = oracle.comp(X, U, V, W, order=order)
        assert np.abs(Y - Y0).max() <= 1e-12 * np.abs(Y0).max(), order


def test_closed_form_exact_on_integer_low_rank_input():
    # integer factors => X = [[A,B,C]] is exactly representable in fp32, so Comp(X) must equal
    # sum_r (U a_r) o (V b_r) o (W c_r) up to fp64 rounding only
    rng = np.random.default_rng(40)
    I, J, K, R, L, M, N = 12, 10, 11, 3, 4, 5, 3
    A = rng.integers(-3, 4, (I, R)).astype(np.float32)
    B = rng.integers(-3, 4, (J, R)).astype(np.float32)
    C = rng.integers(-3, 4, (K, R)).astype(np.float32)
    X = oracle.gen_box(A, B, C, seed=1, sigma=0.0)
    Xe = np.einsum("ir,jr,kr->ijk", A.astype(np.float64), B.astype(np.float64), C.astype(np.float64))
    assert np.array_equal(X.astype(np.float64), Xe)
    U, V, W = _rand(41, L, I), _rand(42, M, J), _rand(43, N, K)
    Yc = oracle.closed_form(A, B, C, U, V, W)
    Y = oracle.comp(X, U, V, W)
    assert np.abs(Y - Yc).max() <= 1e-12 * np.abs(Yc).max()
    # and the closed form itself against its definition via library matmuls
    UA, VB, WC = U.astype(np.float64) @ A, V.astype(np.float64) @ B, W.astype(np.float64) @ C
    Yd = np.einsum("lr,mr,nr->lmn", UA, VB, WC)
    assert np.abs(Yc - Yd).max() <= 1e-12 * np.abs(Yd).max()


def test_closed_form_gaussian_factors_within_fp32_input_rounding():
    cfg = wl.small(sigma=0.0)
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, 0.0)
    Y = oracle.comp_multi(X, U, V, W, cfg.P)
    Yc = oracle.closed_form_multi(A, B, C, U, V, W, cfg.P)
    assert Y.shape == (cfg.L, cfg.M, cfg.N, cfg.P)
    assert oracle.rel_fro(Y, Yc) <= 5e-7   # X is rounded to fp32 once: ~2^-24 per element


def test_block_additivity():
    # Sec. 4.3 / Fig. 2(a): blocks are compressed with the matching column slices and merged by summation
    cfg = wl.small()
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    Y = oracle.comp_multi(X, U, V, W, cfg.P)
    acc = np.zeros_like(Y)
    for i0 in range(0, cfg.I, cfg.dI):
        for j0 in range(0, cfg.J, cfg.dJ):
            for k0 in range(0, cfg.K, cfg.dK):
                box = (i0, i0 + cfg.dI, j0, j0 + cfg.dJ, k0, k0 + cfg.dK)
                Xb = np.asfortranarray(X[box[0]:box[1], box[2]:box[3], box[4]:box[5]])
                acc += oracle.comp_box(Xb, U, V, W, cfg.P, box)
    assert oracle.rel_fro(acc, Y) <= 1e-12


def test_stacked_layout_is_replica_outermost():
    cfg = wl.small()
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    Y = oracle.comp_multi(X, U, V, W, cfg.P)
    flat = Y.reshape(-1, order="F")
    p, l, m, n = 2, 1, 3, 4
    Yp = oracle.comp_brute(X, U[p * cfg.L:(p + 1) * cfg.L], V[p * cfg.M:(p + 1) * cfg.M], W[p * cfg.N:(p + 1) * cfg.N])
    assert abs(flat[l + cfg.L * (m + cfg.M * (n + cfg.N * p))] - Yp[l, m, n]) <= 1e-12 * abs(Yp).max()
    sub = oracle.comp_multi(X, U, V, W, cfg.P, replicas=[2, 0])
    assert np.array_equal(sub[..., 0], Y[..., 2]) and np.array_equal(sub[..., 1], Y[..., 0])


def test_linearity_in_x():
    X1, U, V, W = _tiny(seed=50)
    X2 = np.asfortranarray(_rand(51, *X1.shape))
    Xs = np.asfortranarray((2.0 * X1 + X2).astype(np.float32))
    # use exactly representable combination: recompute from the rounded sum
    Y = oracle.comp(Xs, U, V, W)
    Yl = oracle.comp_brute(Xs, U, V, W)
    assert np.abs(Y - Yl).max() <= 1e-13 * np.abs(Yl).max()
    X1i = np.asfortranarray(np.round(X1 * 8).astype(np.float32))
    X2i = np.asfortranarray(np.round(X2 * 8).astype(np.float32))
    Ysum = oracle.comp(np.asfortranarray(2 * X1i + X2i), U, V, W)
    assert np.abs(Ysum - (2 * oracle.comp(X1i, U, V, W) + oracle.comp(X2i, U, V, W))).max() <= 1e-11 * np.abs(Ysum).max()


def test_identity_matrices_return_x():
    X = np.asfortranarray(_rand(60, 5, 4, 6))
    Y = oracle.comp(X, np.eye(5, dtype=np.float32), np.eye(4, dtype=np.float32), np.eye(6, dtype=np.float32))
    assert np.array_equal(Y, X.astype(np.float64))


def test_row_selectors_return_subtensor_and_ones_return_mode_sums():
    X = np.asfortranarray(_rand(61, 6, 5, 7))
    U = np.zeros((2, 6), np.float32); U[0, 4] = 1; U[1, 1] = 1
    V = np.zeros((3, 5), np.float32); V[0, 0] = 1; V[1, 3] = 1; V[2, 2] = 1
    W = np.zeros((1, 7), np.float32); W[0, 6] = 1
    Y = oracle.comp(X, U, V, W)
    assert np.array_equal(Y, X[[4, 1]][:, [0, 3, 2]][:, :, [6]].astype(np.float64))
    ones = oracle.comp(X, np.ones((1, 6), np.float32), np.eye(5, dtype=np.float32), np.eye(7, dtype=np.float32))
    assert np.abs(ones[0] - X.astype(np.float64).sum(axis=0)).max() <= 1e-13
    ones3 = oracle.comp(X, np.eye(6, dtype=np.float32), np.eye(5, dtype=np.float32), np.ones((1, 7), np.float32))
    assert np.abs(ones3[:, :, 0] - X.astype(np.float64).sum(axis=2)).max() <= 1e-13


def test_rank_one_input_gives_outer_product_of_matvecs():
    rng = np.random.default_rng(62)
    a = rng.integers(-4, 5, 6).astype(np.float32); b = rng.integers(-4, 5, 7).astype(np.float32)
    c = rng.integers(-4, 5, 5).astype(np.float32)
    X = np.asfortranarray(np.einsum("i,j,k->ijk", a, b, c).astype(np.float32))
    U, V, W = _rand(63, 3, 6), _rand(64, 2, 7), _rand(65, 4, 5)
    Y = oracle.comp(X, U, V, W)
    Ye = np.einsum("l,m,n->lmn", U.astype(np.float64) @ a, V.astype(np.float64) @ b, W.astype(np.float64) @ c)
    assert np.abs(Y - Ye).max() <= 1e-12 * np.abs(Ye).max()


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_single_mode_product_matches_matricised_matmul(mode):
    # X x_n M  <=>  M @ X_(n) with the column-major unfolding (Sec. 4.1)
    X = np.asfortranarray(_rand(70 + mode, 5, 6, 4))
    eyes = [np.eye(5, dtype=np.float32), np.eye(6, dtype=np.float32), np.eye(4, dtype=np.float32)]
    Mat = _rand(80 + mode, 3, X.shape[mode])
    mats = list(eyes); mats[mode] = Mat
    Y = oracle.comp(X, *mats)
    Xn = np.moveaxis(X.astype(np.float64), mode, 0).reshape(X.shape[mode], -1, order="F")
    Yn = Mat.astype(np.float64) @ Xn
    shape = [Mat.shape[0]] + [s for a, s in enumerate(X.shape) if a != mode]
    Ye = np.moveaxis(Yn.reshape(shape, order="F"), 0, mode)
    assert np.abs(Y - Ye).max() <= 1e-13 * np.abs(Ye).max()
