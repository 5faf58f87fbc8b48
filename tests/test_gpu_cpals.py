"""GPU parity of the batched CP-ALS (paper Alg. 1) against the CPU oracle, through the C ABI: the factor matrices
after a fixed number of sweeps from the same start values.  fp32 on the GPU against fp64 in the oracle; a sweep
solves well-conditioned normal equations on these inputs, so the factors agree to ~1e-5 and the tolerance is 1e-4
(relative Frobenius error per factor matrix and replica)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_13693_amd import exat

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _problem(seed, L, M, N, R, P, noise=0.05):
    """P tensors 'rank R + noise' and start values; numpy, float32 data."""
    rng = np.random.default_rng(seed)
    Ys, starts = [], []
    for _ in range(P):
        A, B, C = (rng.standard_normal((d, R)) for d in (L, M, N))
        Y = oracle.cp_reconstruct(A, B, C) + noise * np.sqrt(R) * rng.standard_normal((L, M, N))
        Ys.append(Y.astype(np.float32))
        starts.append(tuple(rng.standard_normal((d, R)).astype(np.float32) for d in (L, M, N)))
    return Ys, starts


def _dev_tensor(Ys):
    """replicas outermost, each column-major: the layout of the compression's output"""
    return torch.from_numpy(np.concatenate([Y.reshape(-1, order="F") for Y in Ys])).cuda()


def _dev_factors(starts, which):
    return torch.from_numpy(np.concatenate([s[which].reshape(-1, order="F") for s in starts])).cuda()


def _rel(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def _run_and_compare(L, M, N, R, P, sweeps, seed):
    Ys, starts = _problem(seed, L, M, N, R, P)
    Yd = _dev_tensor(Ys)
    A, B, C = (_dev_factors(starts, i) for i in range(3))
    exat.cpals(Yd, L, M, N, P, R, sweeps, A, B, C)
    torch.cuda.synchronize()
    worst = 0.0
    for p in range(P):
        ref = oracle.cp_als(Ys[p], *starts[p], sweeps)
        for F, D, r in ((A, L, ref[0]), (B, M, ref[1]), (C, N, ref[2])):
            got = F[p * D * R:(p + 1) * D * R].cpu().numpy().astype(np.float64).reshape((D, R), order="F")
            worst = max(worst, _rel(got, r))
        got_rec = oracle.cp_reconstruct(*(F[p * D * R:(p + 1) * D * R].cpu().numpy().reshape((D, R), order="F")
                                          for F, D in ((A, L), (B, M), (C, N))))
        assert _rel(got_rec, oracle.cp_reconstruct(*ref)) <= TOL
    return worst


@pytest.mark.parametrize("shape", [
    dict(L=12, M=10, N=8, R=3, P=3, sweeps=1),
    dict(L=12, M=10, N=8, R=3, P=3, sweeps=5),
    dict(L=32, M=32, N=32, R=16, P=16, sweeps=3),     # the proxy tensors of cfg2
    dict(L=50, M=50, N=50, R=32, P=4, sweeps=2),      # cfg5's shape: extents that are no multiple of 4
    dict(L=64, M=64, N=64, R=64, P=2, sweeps=1),      # the largest supported
    dict(L=7, M=64, N=3, R=17, P=2, sweeps=2),        # lopsided, R just above a wave-quarter boundary
    dict(L=1, M=1, N=1, R=1, P=1, sweeps=2),
])
def test_factors_match_oracle(shape):
    print("case", shape, flush=True)
    worst = _run_and_compare(seed=40, **shape)
    print("  worst factor rel_fro=%.3e" % worst, flush=True)
    assert worst <= TOL


def test_zero_sweeps_leaves_start_values_and_input_untouched():
    L, M, N, R, P = 9, 8, 7, 4, 2
    Ys, starts = _problem(41, L, M, N, R, P)
    Yd = _dev_tensor(Ys)
    Y0 = Yd.clone()
    A, B, C = (_dev_factors(starts, i) for i in range(3))
    A0, B0, C0 = A.clone(), B.clone(), C.clone()
    exat.cpals(Yd, L, M, N, P, R, 0, A, B, C)
    torch.cuda.synchronize()
    assert torch.equal(A, A0) and torch.equal(B, B0) and torch.equal(C, C0) and torch.equal(Yd, Y0)
    # and a run is reproducible bit for bit
    exat.cpals(Yd, L, M, N, P, R, 3, A, B, C)
    exat.cpals(Yd, L, M, N, P, R, 3, A0, B0, C0)
    torch.cuda.synchronize()
    assert torch.equal(A, A0) and torch.equal(B, B0) and torch.equal(C, C0) and torch.equal(Yd, Y0)


def test_exact_low_rank_tensor_is_recovered():
    """Alg. 1 on an exactly rank-R tensor drives the residual to fp32 rounding level."""
    L, M, N, R, P = 16, 14, 12, 3, 2
    Ys, starts = _problem(42, L, M, N, R, P, noise=0.0)
    Yd = _dev_tensor(Ys)
    A, B, C = (_dev_factors(starts, i) for i in range(3))
    exat.cpals(Yd, L, M, N, P, R, 100, A, B, C)
    torch.cuda.synchronize()
    for p in range(P):
        rec = oracle.cp_reconstruct(*(F[p * D * R:(p + 1) * D * R].cpu().numpy().reshape((D, R), order="F")
                                      for F, D in ((A, L), (B, M), (C, N))))
        assert _rel(rec, Ys[p].astype(np.float64)) <= 1e-4


def test_checked_variant_reports_replicas_whose_normal_matrix_is_not_positive_definite():
    """Alg. 1 applies a pseudo-inverse; the Cholesky solve cannot.  A replica whose start factor B has a zero column gives
    the first update a normal matrix (C^T C) * (B^T B) with a zero row and column: exat_cpals_checked must count it for
    that replica, leave the healthy replicas' status at zero, and compute them exactly as exat_cpals does."""
    L, M, N, R, P, sweeps = 12, 10, 8, 4, 3, 2
    Ys, starts = _problem(43, L, M, N, R, P)
    starts = [tuple(f.copy() for f in s) for s in starts]
    starts[1][1][:, 2] = 0.0                      # replica 1: column 2 of the start value of B
    Yd = _dev_tensor(Ys)
    A, B, C = (_dev_factors(starts, i) for i in range(3))
    A0, B0, C0 = A.clone(), B.clone(), C.clone()
    exat.cpals(Yd, L, M, N, P, R, sweeps, A0, B0, C0)
    _, _, _, status = exat.cpals_checked(Yd, L, M, N, P, R, sweeps, A, B, C)
    torch.cuda.synchronize()
    st = status.cpu().numpy()
    print("  status", st, flush=True)
    assert st[0] == 0 and st[2] == 0 and st[1] >= 1
    for F, F0, D in ((A, A0, L), (B, B0, M), (C, C0, N)):
        for p in (0, 2):
            assert torch.equal(F[p * D * R:(p + 1) * D * R], F0[p * D * R:(p + 1) * D * R])
            assert torch.isfinite(F[p * D * R:(p + 1) * D * R]).all()
    # a second call on healthy input clears the counters
    Ys2, starts2 = _problem(44, L, M, N, R, P)
    A, B, C = (_dev_factors(starts2, i) for i in range(3))
    exat.cpals_checked(_dev_tensor(Ys2), L, M, N, P, R, sweeps, A, B, C, status=status)
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
