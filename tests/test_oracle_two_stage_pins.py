"""Pins for the oracle of the two-stage compression (paper Sec. 4.4: U_p = U'_p U with sparse U, V, W)
against things other than itself: scipy's sparse routines, a scatter-form loop over the non-zeros,
selection matrices (sub-sampling), the closed form for a rank-1 tensor, the Kronecker vec identity and
the dense C oracle applied to the first stage's output.  Extents are all distinct, so a transposed
operand or swapped mode cannot pass.  Also checks the seeded sparse input generator."""
import numpy as np
import scipy.sparse as sp

import oracle
import workloads as wl


def _ts(I=23, J=17, K=29, L=3, M=4, N=2, P=3, alpha=2, beta=3, gamma=2, s=3, index=200):
    base = wl.small(index=index, I=I, J=J, K=K, L=L, M=M, N=N, P=P, dI=I, dJ=J, dK=K)
    return wl.TwoStage(base, alpha, beta, gamma, s)


def _x(seed, I, J, K):
    return np.asfortranarray(np.random.default_rng(seed).standard_normal((I, J, K)).astype(np.float32))


def _scipy(csr, cols):
    rowptr, colidx, val = csr
    return sp.csr_matrix((val.astype(np.float64), colidx, rowptr), shape=(len(rowptr) - 1, cols))


def test_sparse_generator_structure():
    ts = _ts()
    b = ts.base
    for csr, rows, cols in zip(wl.first_stage_matrices(ts), (ts.A1, ts.B1, ts.C1), (b.I, b.J, b.K)):
        rowptr, colidx, val = csr
        assert rowptr.dtype == np.int64 and colidx.dtype == np.int32 and val.dtype == np.float32
        assert rowptr[0] == 0 and rowptr[-1] == len(colidx) == len(val) == ts.nnz_per_col * cols
        D = _scipy(csr, cols).toarray()
        assert D.shape == (rows, cols)
        assert ((D != 0).sum(axis=0) == ts.nnz_per_col).all()           # s distinct rows in every column
        assert np.allclose(np.abs(D[D != 0]), ts.nnz_per_col ** -0.5)
        assert np.allclose((D ** 2).sum(axis=0), 1.0)                    # unit-norm columns
        for r in range(rows):
            c = colidx[rowptr[r]:rowptr[r + 1]]
            assert (np.diff(c) > 0).all()
    again = wl.first_stage_matrices(ts)[0]
    assert all((x == y).all() for x, y in zip(again, wl.first_stage_matrices(ts)[0]))
    signs = np.concatenate([c[2] for c in wl.first_stage_matrices(_ts(I=400, J=300, K=200))])
    assert abs((signs > 0).mean() - 0.5) < 0.03


def test_csr_dense_against_scipy():
    ts = _ts()
    U, V, W = wl.first_stage_matrices(ts)
    for csr, cols in ((U, ts.base.I), (V, ts.base.J), (W, ts.base.K)):
        assert np.array_equal(oracle.csr_dense(csr, cols), _scipy(csr, cols).toarray())
    # duplicates add, an empty row stays zero
    csr = (np.array([0, 2, 2, 3]), np.array([1, 1, 0], dtype=np.int32), np.array([0.5, 0.25, -2.0], dtype=np.float32))
    assert np.array_equal(oracle.csr_dense(csr, 3), [[0, 0.75, 0], [0, 0, 0], [-2, 0, 0]])


def test_first_stage_against_scatter_over_nonzeros():
    # Scatter form: every X element is sent to the (a,b,c) cells its column entries name.
    ts = _ts(I=9, J=7, K=8, L=2, M=3, N=2, alpha=2, beta=1, gamma=2, s=2)
    b = ts.base
    X = _x(1, b.I, b.J, b.K)
    U, V, W = wl.first_stage_matrices(ts)
    cols = []
    for csr, n in ((U, b.I), (V, b.J), (W, b.K)):
        rowptr, colidx, val = csr
        lst = [[] for _ in range(n)]
        for r in range(len(rowptr) - 1):
            for e in range(rowptr[r], rowptr[r + 1]):
                lst[colidx[e]].append((r, float(val[e])))
        cols.append(lst)
    ref = np.zeros((ts.A1, ts.B1, ts.C1))
    for i in range(b.I):
        for j in range(b.J):
            for k in range(b.K):
                for a, u in cols[0][i]:
                    for bb, v in cols[1][j]:
                        for c, w in cols[2][k]:
                            ref[a, bb, c] += u * v * w * float(X[i, j, k])
    got = oracle.first_stage(X, U, V, W)
    assert got.shape == (ts.A1, ts.B1, ts.C1)
    assert np.abs(got - ref).max() <= 1e-13 * np.abs(ref).max()


def test_first_stage_with_selection_matrices_subsamples():
    X = _x(2, 11, 9, 13)
    pick = ([7, 0, 3], [8, 8, 1, 2], [12, 5])

    def sel(idx):
        return (np.arange(len(idx) + 1, dtype=np.int64), np.array(idx, dtype=np.int32), np.ones(len(idx), dtype=np.float32))
    got = oracle.first_stage(X, sel(pick[0]), sel(pick[1]), sel(pick[2]))
    assert np.array_equal(got, X[np.ix_(*pick)].astype(np.float64))


def test_first_stage_rank_one_closed_form():
    ts = _ts(index=201)
    b = ts.base
    rng = np.random.default_rng(3)
    a, bb, c = (rng.standard_normal(n) for n in (b.I, b.J, b.K))
    X = np.asfortranarray(np.einsum("i,j,k->ijk", a, bb, c))
    U, V, W = wl.first_stage_matrices(ts)
    ua, vb, wc = _scipy(U, b.I) @ a, _scipy(V, b.J) @ bb, _scipy(W, b.K) @ c
    ref = np.einsum("a,b,c->abc", ua, vb, wc)
    got = oracle.first_stage(X, U, V, W)
    assert np.abs(got - ref).max() <= 1e-12 * np.abs(ref).max()


def test_ttm_chain_kronecker_identity():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((4, 3, 5))
    U, V, W = rng.standard_normal((2, 4)), rng.standard_normal((3, 3)), rng.standard_normal((2, 5))
    y = np.kron(W, np.kron(V, U)) @ X.reshape(-1, order="F")
    Y = oracle.ttm_chain64(X, U, V, W)
    assert Y.shape == (2, 3, 2)
    assert np.abs(Y.reshape(-1, order="F") - y).max() <= 1e-12 * np.abs(y).max()


def test_two_stage_equals_dense_oracle_on_first_stage_output():
    # Associativity: Comp(X, U'U, V'V, W'W) = Comp(Comp(X, U, V, W), U', V', W'); the right-hand side
    # goes through the C oracle (fp32 inputs, fp64 accumulation), hence the fp32-level tolerance.
    ts = _ts(index=202)
    b = ts.base
    X = _x(5, b.I, b.J, b.K)
    U, V, W = wl.first_stage_matrices(ts)
    U2, V2, W2 = wl.second_stage_matrices(ts)
    assert U2.shape == (b.P * b.L, ts.A1) and V2.shape == (b.P * b.M, ts.B1) and W2.shape == (b.P * b.N, ts.C1)
    Y = oracle.two_stage(X, U, V, W, U2, V2, W2, b.P)
    X1 = np.asfortranarray(oracle.first_stage(X, U, V, W).astype(np.float32))
    Yseq = oracle.comp_multi(X1, U2, V2, W2, b.P)
    assert Y.shape == (b.L, b.M, b.N, b.P)
    assert oracle.rel_fro(Y, Yseq) <= 5e-7
    # and against the literal definition with the composed dense matrices through scipy
    p = 1
    Up = U2[p * b.L:(p + 1) * b.L].astype(np.float64) @ _scipy(U, b.I).toarray()
    Vp = V2[p * b.M:(p + 1) * b.M].astype(np.float64) @ _scipy(V, b.J).toarray()
    Wp = W2[p * b.N:(p + 1) * b.N].astype(np.float64) @ _scipy(W, b.K).toarray()
    ref = np.einsum("li,mj,nk,ijk->lmn", Up, Vp, Wp, X.astype(np.float64), optimize=True)
    assert np.abs(Y[:, :, :, p] - ref).max() <= 1e-12 * np.abs(ref).max()
    sub = oracle.two_stage(X, U, V, W, U2, V2, W2, b.P, replicas=[2, 0])
    assert np.array_equal(sub[:, :, :, 0], Y[:, :, :, 2]) and np.array_equal(sub[:, :, :, 1], Y[:, :, :, 0])
