"""Host-side pieces of the decomposition stage that sit between the library's entry points in the tests of the
whole chain (Alg. 2): synthetic inputs with shared anchor rows, and the alignment of the replicas' columns
(normalisation by the anchor rows, Hungarian matching against replica 0).  Test code only: numpy and scipy."""
import numpy as np
from scipy.optimize import linear_sum_assignment


def anchored_matrices(rng, P, L, I, S):
    """(P, L, I) Gaussian compression matrices N(0, 1/L) whose first S rows are the same in every replica."""
    U = rng.standard_normal((P, L, I)) / np.sqrt(L)
    U[:, :S, :] = U[0, :S, :]
    return U.astype(np.float32)


def normalise_by_anchor(F, S):
    """Divides each column of F (rows x R) by its entry of largest magnitude among the first S rows (with its sign),
    which removes the replica's own column scaling."""
    idx = np.abs(F[:S]).argmax(axis=0)
    return F / F[idx, np.arange(F.shape[1])]


def align_replicas(As, Bs, Cs, S):
    """As, Bs, Cs: lists over replicas of (L x R), (M x R), (N x R) factor matrices.  Returns them with every replica's
    columns scaled by the anchor rows and permuted to the order of replica 0 (one permutation for all three modes)."""
    As, Bs, Cs = ([normalise_by_anchor(np.asarray(F, dtype=np.float64), S) for F in Fs] for Fs in (As, Bs, Cs))
    out = ([As[0]], [Bs[0]], [Cs[0]])
    for p in range(1, len(As)):
        # after the normalisation matching columns have the same anchor rows: maximise the summed correlations
        score = sum(F0[:S].T @ Fp[:S] for F0, Fp in ((As[0], As[p]), (Bs[0], Bs[p]), (Cs[0], Cs[p])))
        _, perm = linear_sum_assignment(-score)
        for lst, F in zip(out, (As[p], Bs[p], Cs[p])):
            lst.append(F[:, perm])
    return out


def column_cosines(F, Ftrue):
    """Best one-to-one match of the columns of F to those of Ftrue; returns the absolute cosines, one per column."""
    Fn, Tn = F / np.linalg.norm(F, axis=0), Ftrue / np.linalg.norm(Ftrue, axis=0)
    c = np.abs(Tn.T @ Fn)
    r, k = linear_sum_assignment(-c)
    return c[r, k]
