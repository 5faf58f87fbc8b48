"""GPU parity of the stacked least-squares solve (paper Eq. 4) against the CPU oracle, through the C ABI.
The GPU runs conjugate gradients on the normal equations in fp32; the oracle is the minimiser itself (fp64).
Tolerance: the attainable accuracy of the fp32 iteration is a small multiple of cond(U) * 2^-24; the stacked
Gaussian matrices used here have P*L >= 2 I, i.e. cond(U) <= (1 + sqrt(1/2)) / (1 - sqrt(1/2)) = 5.8 up to
finite-size effects.  The iteration freezes a column at a relative normal-equation residual of 1e-6 (it is reached
after about 30 of the 80 iterations allowed; in fp32 the iterates drift away again if the iteration runs on), which
leaves a relative error of about 4e-6 (numpy emulation of the same iteration) in X; the tolerance is 1e-5 relative Frobenius error."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_13693_amd import exat

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _problem(seed, P, L, I, R, noise=0.05):
    """Gaussian stacked matrix, replica factors U_p X0 plus estimation noise, in the layout the CP-ALS writes."""
    rng = np.random.default_rng(seed)
    Us = rng.standard_normal((P, L, I)).astype(np.float32)
    X0 = rng.standard_normal((I, R))
    A = Us.reshape(P * L, I).astype(np.float64) @ X0 + noise * np.sqrt(I) * rng.standard_normal((P * L, R))
    A = A.astype(np.float32)
    flat = np.concatenate([A[p * L:(p + 1) * L].reshape(-1, order="F") for p in range(P)])  # A[l + L*(r + R*p)]
    return Us, A, flat


def _rel(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def _solve(Us, flat, P, L, I, R, iters, ld=None, tol=1e-6):
    U2 = torch.from_numpy(Us.reshape(P * L, I))
    if ld is not None:  # a leading dimension larger than I
        buf = torch.full((P * L, ld), float("nan"), dtype=torch.float32)
        buf[:, :I] = U2
        Ud = buf.cuda()[:, :I]
    else:
        Ud = U2.cuda()
    X, relres = exat.ls(Ud, P, L, I, torch.from_numpy(flat).cuda(), R, iters, tol)
    torch.cuda.synchronize()
    return X.cpu().numpy().astype(np.float64).reshape((I, R), order="F"), relres.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("shape", [
    dict(P=3, L=5, I=7, R=3),                 # everything ragged, scalar loads (leading dimension 7)
    dict(P=4, L=16, I=24, R=16, ld=32),       # padded leading dimension, 16-byte loads
    dict(P=5, L=20, I=40, R=40),              # two column tiles
    dict(P=7, L=33, I=100, R=64),             # R at its limit, several row tiles with a ragged tail
    dict(P=24, L=50, I=500, R=32),            # cfg5's L and R at a size where P*L >= 2 I
    dict(P=1, L=64, I=1, R=1),                # one unknown
], ids=lambda s: "P{P}_L{L}_I{I}_R{R}".format(**s))
def test_small_shapes_against_oracle(shape):
    P, L, I, R = shape["P"], shape["L"], shape["I"], shape["R"]
    print("case", shape, flush=True)
    Us, A, flat = _problem(100 + I, P, L, I, R)
    X, relres = _solve(Us, flat, P, L, I, R, 80, ld=shape.get("ld"))
    ref = oracle.stacked_ls(Us, A)
    assert _rel(X, ref) <= TOL
    assert relres.shape == (R,) and np.all(relres < 1e-4)


@pytest.mark.parametrize("cfg", [dict(P=32, L=64, I=1024, R=32), dict(P=32, L=32, I=512, R=16)],
                         ids=["cfg3_shapes", "cfg2_shapes_P_doubled"])
def test_benchmark_shapes_against_oracle(cfg):
    # cfg3: the stacked matrix of the 1024^3 configuration (2048 x 1024).  cfg2's own stacked matrix is square
    # (16 * 32 = 512 = I), which fp32 cannot solve accurately; twice the replicas give the 2:1 system.
    P, L, I, R = cfg["P"], cfg["L"], cfg["I"], cfg["R"]
    print("case", cfg, flush=True)
    Us, A, flat = _problem(7, P, L, I, R)
    X, relres = _solve(Us, flat, P, L, I, R, 80)
    assert _rel(X, oracle.stacked_ls(Us, A)) <= TOL


def test_exact_system_returns_the_factor():
    # noise-free replica factors U_p X0: the solve returns X0 (the Kronecker property the join rests on)
    P, L, I, R = 6, 32, 96, 8
    rng = np.random.default_rng(5)
    Us = rng.standard_normal((P, L, I)).astype(np.float32)
    X0 = rng.standard_normal((I, R))
    A = (Us.reshape(P * L, I).astype(np.float64) @ X0).astype(np.float32)
    flat = np.concatenate([A[p * L:(p + 1) * L].reshape(-1, order="F") for p in range(P)])
    X, _ = _solve(Us, flat, P, L, I, R, 80)
    assert _rel(X, X0) <= TOL


def test_reported_residual_and_zero_iterations():
    P, L, I, R = 8, 16, 48, 5
    Us, A, flat = _problem(9, P, L, I, R)
    U = Us.reshape(P * L, I).astype(np.float64)
    X, relres = _solve(Us, flat, P, L, I, R, 0)
    assert np.all(X == 0.0) and np.allclose(relres, 1.0)
    # after a few iterations the reported figure is the normal-equation residual of the returned X
    X, relres = _solve(Us, flat, P, L, I, R, 3)
    want = np.linalg.norm(U.T @ (A - U @ X), axis=0) / np.linalg.norm(U.T @ A, axis=0)
    assert np.all(relres > 1e-4) and np.allclose(relres, want, rtol=1e-3)
    # and the iterates approach the minimiser monotonically in the residual norm
    ref = oracle.stacked_ls(Us, A)
    errs = [np.linalg.norm(U @ _solve(Us, flat, P, L, I, R, k)[0] - A) for k in (1, 2, 4, 8, 16)]
    assert all(b <= a * (1 + 1e-6) for a, b in zip(errs, errs[1:]))
    assert errs[-1] <= np.linalg.norm(U @ ref - A) * (1 + 1e-5)


def test_zero_right_hand_side_column():
    # a column of zeros must give zeros (no division by a vanishing norm)
    P, L, I, R = 4, 16, 20, 4
    Us, A, _ = _problem(11, P, L, I, R)
    A[:, 2] = 0.0
    flat = np.concatenate([A[p * L:(p + 1) * L].reshape(-1, order="F") for p in range(P)])
    X, relres = _solve(Us, flat, P, L, I, R, 40)
    assert np.all(np.isfinite(X)) and np.all(X[:, 2] == 0.0) and relres[2] == 0.0
    assert _rel(X, oracle.stacked_ls(Us, A)) <= TOL


def test_unaligned_matrix_pointer():
    # a stacked matrix that starts 4 bytes into an allocation: the 16-byte loads are off, every row tile and
    # k step goes through the scalar path, at a size that spans several tiles
    P, L, I, R = 4, 40, 72, 8
    Us, A, flat = _problem(21, P, L, I, R)
    ld = I + 3
    buf = torch.full((P * L * ld + 1,), float("nan"), dtype=torch.float32).cuda()
    view = buf[1:].view(P * L, ld)[:, :I]
    view.copy_(torch.from_numpy(Us.reshape(P * L, I)))
    assert view.data_ptr() % 16 != 0
    X, relres = exat.ls(view, P, L, I, torch.from_numpy(flat).cuda(), R, 80)
    torch.cuda.synchronize()
    got = X.cpu().numpy().astype(np.float64).reshape((I, R), order="F")
    assert _rel(got, oracle.stacked_ls(Us, A)) <= TOL
