"""The oracle's three stages chained as in Alg. 2 -- compression of an exactly low-rank tensor into P replicas,
CP-ALS of every replica, alignment by the shared anchor rows, stacked least squares per mode -- return the factor
matrices of the full tensor up to column order and scale.  This pins the pieces against the property the whole
method rests on (Sec. 3: A_p = U_p A Pi_p Sigma_p), which none of them can satisfy alone."""
import numpy as np

import oracle
from pipeline_util import align_replicas, anchored_matrices, column_cosines


def test_chain_recovers_the_factors():
    I, J, K, R, L, M, N, P, S = 20, 18, 16, 2, 6, 6, 6, 8, 3
    rng = np.random.default_rng(42)
    A, B, C = rng.standard_normal((I, R)), rng.standard_normal((J, R)), rng.standard_normal((K, R))
    X = oracle.cp_reconstruct(A, B, C).astype(np.float32)
    Us, Vs, Ws = (anchored_matrices(rng, P, d, n, S) for d, n in ((L, I), (M, J), (N, K)))
    Y = oracle.comp_multi(X, Us.reshape(P * L, I), Vs.reshape(P * M, J), Ws.reshape(P * N, K), P)   # (L, M, N, P)
    As, Bs, Cs = [], [], []
    for p in range(P):
        a, b, c = oracle.cp_als(Y[..., p], rng.standard_normal((L, R)), rng.standard_normal((M, R)),
                                rng.standard_normal((N, R)), 300)
        assert np.linalg.norm(oracle.cp_reconstruct(a, b, c) - Y[..., p]) <= 1e-6 * np.linalg.norm(Y[..., p])
        As.append(a); Bs.append(b); Cs.append(c)
    As, Bs, Cs = align_replicas(As, Bs, Cs, S)
    for Fs, Ustk, true in ((As, Us, A), (Bs, Vs, B), (Cs, Ws, C)):
        got = oracle.stacked_ls(Ustk, np.concatenate(Fs, axis=0))
        assert np.all(column_cosines(got, true) >= 1 - 1e-8)
