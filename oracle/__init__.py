"""CPU oracle for the multi-replica compression step Y_p = Comp(X, U_p, V_p, W_p).

TEST INFRASTRUCTURE ONLY.  The test-suite, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product (the HIP library and its
Python binding) never does, and this package never imports the product.

Every function is a numpy-facing wrapper over oracle/exat_oracle.c (plain C,
fp64 accumulation), except the two-stage functions (Sec. 4.4), the CP-ALS of the
proxy tensors (Alg. 1) and the stacked least squares (Eq. 4) at the end, which are
plain numpy in fp64.

Conventions (paper Sec. 3, Eq. 3 and Sec. 4.1):
  X   float32 array of shape (I, J, K), Fortran (column-major) order
  U   float32 (L, I), V (M, J), W (N, K), C order (reduction index contiguous)
  Y   float64 (L, M, N), Fortran order
Stacked operands hold replica p in rows p*L .. p*L+L-1.
"""
import ctypes
import os

import numpy as np

from .build import build as _build

_lib = None
_i64 = ctypes.c_int64
_fp = ctypes.POINTER(ctypes.c_float)
_dp = ctypes.POINTER(ctypes.c_double)


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build())
        _lib.orc_noise.restype = ctypes.c_double
        _lib.orc_noise.argtypes = [ctypes.c_uint64, _i64, _i64, _i64]
        _lib.orc_noise_word.restype = ctypes.c_uint32
        _lib.orc_noise_word.argtypes = [ctypes.c_uint64, _i64, _i64, _i64]
        _lib.orc_round_bf16.restype = ctypes.c_float
        _lib.orc_round_bf16.argtypes = [ctypes.c_float]
        _lib.orc_comp.restype = ctypes.c_int
        _lib.orc_closed_form.restype = ctypes.c_int
    return _lib


def num_threads():
    """Threads the oracle's OpenMP loops use."""
    return int(lib().orc_num_threads())


def _f32c(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_fp)


def _x_f(X):
    X = np.asarray(X)
    if X.dtype != np.float32 or X.ndim != 3:
        raise ValueError("X must be a float32 array of shape (I, J, K)")
    return np.asfortranarray(X)


def comp_brute(X, U, V, W):
    """Eq. 3 as six nested loops (tiny sizes only)."""
    X = _x_f(X)
    I, J, K = X.shape
    U, pU = _f32c(U); V, pV = _f32c(V); W, pW = _f32c(W)
    L, M, N = U.shape[0], V.shape[0], W.shape[0]
    assert U.shape[1] == I and V.shape[1] == J and W.shape[1] == K
    Y = np.zeros((L, M, N), dtype=np.float64, order="F")
    lib().orc_comp_brute(X.ctypes.data_as(_fp), _i64(I), _i64(J), _i64(K),
                         pU, _i64(I), _i64(L), pV, _i64(J), _i64(M), pW, _i64(K), _i64(N),
                         Y.ctypes.data_as(_dp))
    return Y


def comp(X, U, V, W, order=(0, 1, 2)):
    """Comp(X,U,V,W) mode by mode (Sec. 4.3), in the given mode order (0-based)."""
    X = _x_f(X)
    I, J, K = X.shape
    U, pU = _f32c(U); V, pV = _f32c(V); W, pW = _f32c(W)
    L, M, N = U.shape[0], V.shape[0], W.shape[0]
    assert U.shape[1] == I and V.shape[1] == J and W.shape[1] == K
    assert sorted(order) == [0, 1, 2]
    Y = np.zeros((L, M, N), dtype=np.float64, order="F")
    o = (ctypes.c_int * 3)(*order)
    rc = lib().orc_comp(X.ctypes.data_as(_fp), _i64(I), _i64(J), _i64(K),
                        pU, _i64(I), _i64(L), pV, _i64(J), _i64(M), pW, _i64(K), _i64(N),
                        o, Y.ctypes.data_as(_dp))
    if rc != 0:
        raise MemoryError("oracle: out of memory")
    return Y


def comp_multi(X, Us, Vs, Ws, P, replicas=None):
    """All (or the listed) replicas, one at a time.  Us is (P*L, I) etc.
    Returns float64 (L, M, N, len(replicas)) in Fortran order: the layout
    Y[l + L*(m + M*(n + N*p))] of the library's output."""
    L, M, N = Us.shape[0] // P, Vs.shape[0] // P, Ws.shape[0] // P
    reps = list(range(P)) if replicas is None else list(replicas)
    Y = np.zeros((L, M, N, len(reps)), dtype=np.float64, order="F")
    for t, p in enumerate(reps):
        Y[:, :, :, t] = comp(X, Us[p * L:(p + 1) * L], Vs[p * M:(p + 1) * M], Ws[p * N:(p + 1) * N])
    return Y


def comp_box(Xbox, Us, Vs, Ws, P, box, replicas=None):
    """Contribution of the sub-box box=(i0,i1,j0,j1,k0,k1) of X (Sec. 4.3: a block is
    compressed with the matching column slices of U, V, W)."""
    i0, i1, j0, j1, k0, k1 = box
    return comp_multi(Xbox, Us[:, i0:i1], Vs[:, j0:j1], Ws[:, k0:k1], P, replicas)


def closed_form(A, B, C, U, V, W):
    """Comp of the exactly rank-R tensor [[A,B,C]]: sum_r (U a_r) o (V b_r) o (W c_r)."""
    A = np.asfortranarray(A, dtype=np.float32); B = np.asfortranarray(B, dtype=np.float32)
    C = np.asfortranarray(C, dtype=np.float32)
    I, R = A.shape; J = B.shape[0]; K = C.shape[0]
    U, pU = _f32c(U); V, pV = _f32c(V); W, pW = _f32c(W)
    L, M, N = U.shape[0], V.shape[0], W.shape[0]
    Y = np.zeros((L, M, N), dtype=np.float64, order="F")
    rc = lib().orc_closed_form(A.ctypes.data_as(_fp), B.ctypes.data_as(_fp), C.ctypes.data_as(_fp),
                               _i64(I), _i64(J), _i64(K), _i64(R),
                               pU, _i64(I), _i64(L), pV, _i64(J), _i64(M), pW, _i64(K), _i64(N),
                               Y.ctypes.data_as(_dp))
    if rc != 0:
        raise MemoryError("oracle: out of memory")
    return Y


def closed_form_multi(A, B, C, Us, Vs, Ws, P, replicas=None):
    L, M, N = Us.shape[0] // P, Vs.shape[0] // P, Ws.shape[0] // P
    reps = list(range(P)) if replicas is None else list(replicas)
    Y = np.zeros((L, M, N, len(reps)), dtype=np.float64, order="F")
    for t, p in enumerate(reps):
        Y[:, :, :, t] = closed_form(A, B, C, Us[p * L:(p + 1) * L], Vs[p * M:(p + 1) * M],
                                    Ws[p * N:(p + 1) * N])
    return Y


def noise(seed, i, j, k):
    """g(seed; i,j,k): one standard-normal draw (see exat_oracle.c for the definition)."""
    return float(lib().orc_noise(ctypes.c_uint64(seed), _i64(i), _i64(j), _i64(k)))


def noise_word(seed, i, j, k):
    return int(lib().orc_noise_word(ctypes.c_uint64(seed), _i64(i), _i64(j), _i64(k)))


def noise_box(seed, box):
    i0, i1, j0, j1, k0, k1 = box
    out = np.zeros((i1 - i0, j1 - j0, k1 - k0), dtype=np.float64, order="F")
    lib().orc_noise_box(ctypes.c_uint64(seed), _i64(i0), _i64(i1), _i64(j0), _i64(j1), _i64(k0), _i64(k1),
                        out.ctypes.data_as(_dp))
    return out


def round_bf16(a):
    """Round-to-nearest-even to bf16, returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty_like(a)
    lib().orc_round_bf16_array(a.ctypes.data_as(_fp), out.ctypes.data_as(_fp), _i64(a.size))
    return out


def gen_box(A, B, C, seed, sigma, box=None, to_bf16=False):
    """X = fl32([[A,B,C]] + sigma*g) on a box (default: everything), float32 Fortran order."""
    A = np.asfortranarray(A, dtype=np.float32); B = np.asfortranarray(B, dtype=np.float32)
    C = np.asfortranarray(C, dtype=np.float32)
    I, R = A.shape; J = B.shape[0]; K = C.shape[0]
    if box is None:
        box = (0, I, 0, J, 0, K)
    i0, i1, j0, j1, k0, k1 = box
    out = np.zeros((i1 - i0, j1 - j0, k1 - k0), dtype=np.float32, order="F")
    lib().orc_gen_box(A.ctypes.data_as(_fp), B.ctypes.data_as(_fp), C.ctypes.data_as(_fp),
                      _i64(I), _i64(J), _i64(K), _i64(R), ctypes.c_uint64(seed), ctypes.c_double(sigma),
                      _i64(i0), _i64(i1), _i64(j0), _i64(j1), _i64(k0), _i64(k1),
                      ctypes.c_int(1 if to_bf16 else 0), out.ctypes.data_as(_fp))
    return out


def rel_fro(Y, Yref):
    """Per-replica relative Frobenius error max_p ||Y_p - Yref_p||_F / ||Yref_p||_F
    for arrays of shape (L, M, N, P)."""
    Y = np.asarray(Y, dtype=np.float64); Yref = np.asarray(Yref, dtype=np.float64)
    num = np.sqrt(((Y - Yref) ** 2).sum(axis=(0, 1, 2)))
    den = np.sqrt((Yref ** 2).sum(axis=(0, 1, 2)))
    return float((num / den).max())


# ---- Two-stage compression (Sec. 4.4): U_p = U'_p U with sparse U, V, W ---------------------------
# Plain numpy in fp64.  The sparse matrices are expanded to dense ones and the definition of the
# mode products is applied with numpy's tensordot; nothing here exploits the sparsity.

def csr_dense(csr, cols):
    """Dense float64 (rows, cols) matrix of a CSR triple (rowptr, colidx, val); duplicates add."""
    rowptr, colidx, val = csr
    rows = len(rowptr) - 1
    D = np.zeros((rows, cols), dtype=np.float64)
    for r in range(rows):
        for e in range(int(rowptr[r]), int(rowptr[r + 1])):
            D[r, int(colidx[e])] += float(val[e])
    return D


def ttm_chain64(X, U, V, W):
    """X x1 U x2 V x3 W (Eq. 3) for float64 matrices U (L,I), V (M,J), W (N,K); returns (L,M,N) float64."""
    Z = np.tensordot(np.asarray(U, dtype=np.float64), np.asarray(X, dtype=np.float64), axes=(1, 0))  # (L,J,K)
    Z = np.tensordot(np.asarray(V, dtype=np.float64), Z, axes=(1, 1))                                # (M,L,K)
    Z = np.tensordot(np.asarray(W, dtype=np.float64), Z, axes=(1, 2))                                # (N,M,L)
    return np.asfortranarray(Z.transpose(2, 1, 0))


def first_stage(X, Ucsr, Vcsr, Wcsr):
    """The implicit first compression of Sec. 4.4: X x1 U x2 V x3 W with the shared sparse matrices."""
    I, J, K = X.shape
    return ttm_chain64(X, csr_dense(Ucsr, I), csr_dense(Vcsr, J), csr_dense(Wcsr, K))


def two_stage(X, Ucsr, Vcsr, Wcsr, U2, V2, W2, P, replicas=None):
    """Y_p = Comp(X, U'_p U, V'_p V, W'_p W) (Sec. 4.4) with the composed matrices formed explicitly.
    U2 is the stacked (P*L, alpha L) matrix etc.  Returns float64 (L, M, N, len(replicas)), Fortran order."""
    I, J, K = X.shape
    Ud, Vd, Wd = csr_dense(Ucsr, I), csr_dense(Vcsr, J), csr_dense(Wcsr, K)
    L, M, N = U2.shape[0] // P, V2.shape[0] // P, W2.shape[0] // P
    reps = list(range(P)) if replicas is None else list(replicas)
    Y = np.zeros((L, M, N, len(reps)), dtype=np.float64, order="F")
    X64 = np.asarray(X, dtype=np.float64)
    for t, p in enumerate(reps):
        Up = U2[p * L:(p + 1) * L].astype(np.float64) @ Ud
        Vp = V2[p * M:(p + 1) * M].astype(np.float64) @ Vd
        Wp = W2[p * N:(p + 1) * N].astype(np.float64) @ Wd
        Y[:, :, :, t] = ttm_chain64(X64, Up, Vp, Wp)
    return Y


# ---- CP-ALS on the proxy tensors (Alg. 1), the consumer of Y ---------------------------------------
# Plain numpy in fp64.  One sweep = the three updates of the algorithm's loop body in its order (A, B, C),
# each the least-squares solution with the two other matrices fixed:
#   A <- Y_(1) (C kr B) [(C^T C) * (B^T B)]^{-1}      (kr = Khatri-Rao product, * = Hadamard product)
# The listing prints the Gram term without the inverse and as C C^T; read as the standard normal equations.

def khatri_rao(C, B):
    """Column-wise Kronecker product: row (m + M*n) of the result is C[n,:] * B[m,:]."""
    N, R = C.shape
    M = B.shape[0]
    return (C[:, None, :] * B[None, :, :]).reshape(N * M, R)


def unfold(Y, mode):
    """Mode-n matricisation of a 3-way array in the column-major convention of Sec. 2:
    Y_(1)[l, m + M*n], Y_(2)[m, l + L*n], Y_(3)[n, l + L*m]."""
    Y = np.asarray(Y, dtype=np.float64)
    L, M, N = Y.shape
    if mode == 0:
        return Y.reshape(L, M * N, order="F")
    if mode == 1:
        return Y.transpose(1, 0, 2).reshape(M, L * N, order="F")
    return Y.transpose(2, 0, 1).reshape(N, L * M, order="F")


def cp_als(Y, A0, B0, C0, sweeps):
    """`sweeps` sweeps of Alg. 1 from the given start; returns float64 (A, B, C)."""
    A, B, C = (np.array(F, dtype=np.float64) for F in (A0, B0, C0))
    Y1, Y2, Y3 = unfold(Y, 0), unfold(Y, 1), unfold(Y, 2)
    for _ in range(sweeps):
        A = np.linalg.solve(((C.T @ C) * (B.T @ B)).T, (Y1 @ khatri_rao(C, B)).T).T
        B = np.linalg.solve(((C.T @ C) * (A.T @ A)).T, (Y2 @ khatri_rao(C, A)).T).T
        C = np.linalg.solve(((B.T @ B) * (A.T @ A)).T, (Y3 @ khatri_rao(B, A)).T).T
    return A, B, C


def cp_reconstruct(A, B, C):
    """sum_r a_r o b_r o c_r (Eq. 1) as a float64 (L, M, N) array."""
    return np.einsum("lr,mr,nr->lmn", np.asarray(A, dtype=np.float64), np.asarray(B, dtype=np.float64),
                     np.asarray(C, dtype=np.float64))


# ---- joining the replicas: the stacked least-squares problem of Eq. 4 ------------------------------
# After the P decompositions (and the alignment of their columns) the factor of the full tensor solves
#   [A_1; ...; A_P] = [U_1; ...; U_P] X        (PL x R) = (PL x I)(I x R),   X = A Pi Sigma,
# in the least-squares sense.  The definition written out: the minimiser of the Frobenius norm of the
# residual, by numpy's SVD-based routine in fp64.

def stacked_ls(Us, Astack):
    """Us: (P, L, I) compression matrices of one mode; Astack: (P*L, R), the replica factors stacked in
    replica order.  Returns the float64 (I, R) minimiser of ||[U_1;...;U_P] X - Astack||_F."""
    Us = np.asarray(Us, dtype=np.float64)
    P, L, I = Us.shape
    Astack = np.asarray(Astack, dtype=np.float64)
    if Astack.shape[0] != P * L:
        raise ValueError("Astack must have P*L rows")
    return np.linalg.lstsq(Us.reshape(P * L, I), Astack, rcond=None)[0]
