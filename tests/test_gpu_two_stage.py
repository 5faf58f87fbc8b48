"""GPU parity of the two-stage compression (paper Sec. 4.4) against the CPU oracle, through the C ABI:
the sparse first stage on its own (element by element) and the whole chain first stage -> dense
multi-replica compression.  Tolerance: relative Frobenius error <= 1e-5 (fp32 arithmetic)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2311_13693_amd import exat
import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _ts(I, J, K, L, M, N, P=3, alpha=2, beta=2, gamma=2, s=4, index=300):
    base = wl.small(index=index, I=I, J=J, K=K, L=L, M=M, N=N, P=P, dI=I, dJ=J, dK=K)
    return wl.TwoStage(base, alpha, beta, gamma, s)


def _x(seed, I, J, K):
    return np.asfortranarray(np.random.default_rng(seed).standard_normal((I, J, K)).astype(np.float32))


def _rel(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def _first_stage_gpu(ts, X, mats):
    b = ts.base
    st = exat.Stage1(b.I, b.J, b.K, *mats)
    assert st.dims == (ts.A1, ts.B1, ts.C1)
    X1 = st.apply(gu.to_dev_x(X))
    torch.cuda.synchronize()
    out = X1.cpu().numpy().astype(np.float64).reshape(st.dims, order="F")
    st.close()
    return out


# several tiles in i (128) and j (64) with ragged tails, both row-count instantiations of a and b
@pytest.mark.parametrize("shape", [
    dict(I=300, J=150, K=9, L=8, M=5, N=3),                              # A1=16, B1=10: small row counts
    dict(I=129, J=65, K=5, L=32, M=32, N=4),                             # A1=B1=64: exactly one lane tile
    dict(I=257, J=200, K=7, L=50, M=20, N=6),                            # A1=100 (two lane tiles), B1=40
    dict(I=140, J=70, K=6, L=11, M=45, N=9, beta=2),                     # A1=22, B1=90
    dict(I=384, J=130, K=4, L=64, M=64, N=2),                            # A1=B1=128: the largest supported
    dict(I=5, J=3, K=2, L=1, M=1, N=1, alpha=1, beta=1, gamma=1, s=1),   # everything smaller than a tile
    # the matrix-core form (I a multiple of 4, values +-1/2): three row tiles of a (result blocks of a wave in different
    # row tiles), three 256-column tiles with a ragged last one, a ragged last step of 32 rows
    dict(I=268, J=600, K=5, L=48, M=24, N=3),                            # A1=96, B1=48
    dict(I=512, J=512, K=3, L=16, M=64, N=2),                            # A1=32, B1=128: one row tile, four result blocks
    dict(I=96, J=40, K=4, L=32, M=32, N=2, s=3),                         # values 3**-0.5 are no bf16 numbers: the sparse form
])
def test_first_stage_matches_oracle(shape):
    ts = _ts(**shape)
    b = ts.base
    print("case", shape, flush=True)
    X = _x(11, b.I, b.J, b.K)
    mats = wl.first_stage_matrices(ts)
    ref = oracle.first_stage(X, *mats)
    got = _first_stage_gpu(ts, X, mats)
    err = _rel(got, ref)
    print("  rel_fro=%.3e" % err, flush=True)
    assert err <= TOL
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()


def test_first_stage_matrix_core_form_agrees_with_sparse_form(monkeypatch):
    """Both forms compute the same sums from the same operands; the matrix-core form splits X exactly, so they differ
    by the order of fp32 additions only."""
    ts = _ts(I=320, J=300, K=6, L=32, M=32, N=4, index=303)
    b = ts.base
    X = _x(17, b.I, b.J, b.K)
    mats = wl.first_stage_matrices(ts)
    got = _first_stage_gpu(ts, X, mats)
    monkeypatch.setenv("EXAT_STAGE1_MFMA", "0")
    sparse = _first_stage_gpu(ts, X, mats)
    err = _rel(got, sparse)
    print("  matrix-core form against sparse form: rel_fro=%.3e" % err, flush=True)
    assert err <= 1e-6 and err > 0.0   # > 0: the two runs did take different kernels


def test_first_stage_general_csr_and_run_to_run():
    # a general CSR matrix: unsorted columns, repeated entries, empty rows, arbitrary values
    rng = np.random.default_rng(5)
    I, J, K = 200, 90, 12

    def rand_csr(rows, cols, density):
        rowptr, ci, v = [0], [], []
        for r in range(rows):
            n = 0 if r % 5 == 3 else int(rng.integers(1, max(2, int(cols * density))))
            c = rng.integers(0, cols, n)
            ci.extend(c.tolist()); v.extend(rng.standard_normal(n).tolist())
            rowptr.append(len(ci))
        return np.array(rowptr, dtype=np.int64), np.array(ci, dtype=np.int32), np.array(v, dtype=np.float32)
    mats = (rand_csr(37, I, 0.2), rand_csr(70, J, 0.3), rand_csr(9, K, 0.9))
    X = _x(6, I, J, K)
    ref = oracle.first_stage(X, *mats)
    st = exat.Stage1(I, J, K, *mats)
    Xd = gu.to_dev_x(X)
    a = st.apply(Xd).clone()
    b = st.apply(Xd)
    torch.cuda.synchronize()
    assert torch.equal(a, b)                                     # fixed summation order
    got = a.cpu().numpy().astype(np.float64).reshape(st.dims, order="F")
    assert _rel(got, ref) <= TOL
    assert (got[3] == 0).all() and (got[:, 3] == 0).all()        # empty rows give exact zeros
    st.close()


def test_two_stage_chain_matches_oracle():
    ts = _ts(I=200, J=136, K=90, L=12, M=10, N=8, P=3, alpha=2, beta=3, gamma=2, s=4, index=301)
    b = ts.base
    X = _x(7, b.I, b.J, b.K)
    mats = wl.first_stage_matrices(ts)
    U2, V2, W2 = wl.second_stage_matrices(ts)
    ref = oracle.two_stage(X, *mats, U2, V2, W2, b.P)
    st = exat.Stage1(b.I, b.J, b.K, *mats)
    plan = gu.plan_with_factors(ts.second, U2, V2, W2)
    Y = plan.compress(st.apply(gu.to_dev_x(X)))
    torch.cuda.synchronize()
    err = oracle.rel_fro(gu.y_to_numpy(Y, b), ref)
    print("two-stage chain rel_fro=%.3e" % err, flush=True)
    assert err <= TOL
    plan.close(); st.close()


@pytest.mark.parametrize("name,reps", [("cfg2", [0, 7, 15]), ("cfg3", [31])])
def test_two_stage_at_benchmark_sizes(name, reps):
    """The launch configuration `bench.py --two-stage` times: first stage compared element by element with
    the oracle, the chain on sampled replicas."""
    cfg = wl.CONFIGS[name]
    ts = wl.TwoStage(cfg)
    print("case", name, flush=True)
    A, B, C = wl.cp_factors(cfg)
    gen = gu.gen_of(cfg, A, B, C)
    whole = exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.I, cfg.J, cfg.K, exat.EXAT_F32)
    Xd = torch.empty(cfg.elements, dtype=torch.float32, device="cuda")
    exat.gen_block(whole, gen, 0, 0, 0, Xd)
    mats = wl.first_stage_matrices(ts)
    U2, V2, W2 = wl.second_stage_matrices(ts)
    st = exat.Stage1(cfg.I, cfg.J, cfg.K, *mats)
    plan = gu.plan_with_factors(ts.second, U2, V2, W2)
    X1 = st.apply(Xd)
    Y = plan.compress(X1)
    torch.cuda.synchronize()
    X = Xd.cpu().numpy().reshape((cfg.I, cfg.J, cfg.K), order="F")
    ref1 = oracle.first_stage(X, *mats)
    e1 = _rel(X1.cpu().numpy().astype(np.float64).reshape(st.dims, order="F"), ref1)
    ref = oracle.two_stage(X, *mats, U2, V2, W2, cfg.P, replicas=reps)
    e2 = oracle.rel_fro(gu.y_to_numpy(Y, cfg)[..., reps], ref)
    print("  first stage rel_fro=%.3e, chain rel_fro=%.3e" % (e1, e2), flush=True)
    assert e1 <= TOL and e2 <= TOL
    plan.close(); st.close()


def test_first_stage_degenerate_shapes():
    """Single fibre / slice / row, an all-zero matrix, and a dense (every entry present) matrix whose per-wave
    chunk streams are longer than anything the sparse ensemble produces."""
    rng = np.random.default_rng(9)

    def dense_csr(D):
        rows, cols = D.shape
        return (np.arange(rows + 1, dtype=np.int64) * cols, np.tile(np.arange(cols, dtype=np.int32), rows),
                D.reshape(-1).astype(np.float32))

    def zero_csr(rows):
        return np.zeros(rows + 1, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32)
    cases = [
        (1, 1, 1, dense_csr(np.array([[2.0]])), dense_csr(np.array([[3.0]])), dense_csr(np.array([[5.0]]))),
        (130, 1, 1, dense_csr(rng.standard_normal((3, 130))), dense_csr(np.array([[1.0], [2.0]])), dense_csr(np.array([[1.0]]))),
        (40, 70, 3, zero_csr(4), dense_csr(rng.standard_normal((5, 70))), dense_csr(rng.standard_normal((2, 3)))),
        (300, 90, 5, dense_csr(rng.standard_normal((128, 300))), dense_csr(rng.standard_normal((128, 90))),
         dense_csr(rng.standard_normal((7, 5)))),
        # bf16-valued U and V with I a multiple of 4: the matrix-core form, on one short step of one ragged tile, with an
        # all-zero U, and with dense sign matrices over three column tiles
        (4, 1, 1, dense_csr(np.array([[1.0, -2.0, 0.5, 4.0]])), dense_csr(np.array([[3.0]])), dense_csr(np.array([[5.0]]))),
        (8, 3, 2, zero_csr(4), dense_csr(np.sign(rng.standard_normal((5, 3)))), dense_csr(rng.standard_normal((2, 2)))),
        (64, 520, 3, dense_csr(0.5 * np.sign(rng.standard_normal((128, 64)))), dense_csr(np.sign(rng.standard_normal((128, 520)))),
         dense_csr(rng.standard_normal((7, 3)))),
    ]
    for I, J, K, U, V, W in cases:
        print("case", I, J, K, len(U[0]) - 1, len(V[0]) - 1, len(W[0]) - 1, flush=True)
        X = _x(12, I, J, K)
        ref = oracle.first_stage(X, U, V, W)
        st = exat.Stage1(I, J, K, U, V, W)
        got = st.apply(gu.to_dev_x(X))
        torch.cuda.synchronize()
        got = got.cpu().numpy().astype(np.float64).reshape(st.dims, order="F")
        st.close()
        if np.abs(ref).max() == 0:
            assert (got == 0).all()
        else:
            assert _rel(got, ref) <= TOL


def test_first_stage_from_host_memory(monkeypatch):
    """exat_stage1_apply_host: slabs of slices copied from host memory ahead of the kernels; bit-identical to the
    device-resident call.  The slab size is forced down so that the 23 slices take 8 slabs (ring of 3 reused)."""
    ts = _ts(I=150, J=100, K=23, L=10, M=9, N=5, index=302)
    b = ts.base
    monkeypatch.setenv("EXAT_STAGE1_SLAB_BYTES", str(3 * b.I * b.J * 4))
    X = _x(13, b.I, b.J, b.K)
    mats = wl.first_stage_matrices(ts)
    st = exat.Stage1(b.I, b.J, b.K, *mats)
    Xflat = torch.from_numpy(np.ascontiguousarray(X.reshape(-1, order="F")))
    ref = st.apply(Xflat.cuda()).clone()
    a = st.apply_host(Xflat.pin_memory()).clone()
    c = st.apply_host(Xflat.clone()).clone()      # pageable, second pass over the ring
    torch.cuda.synchronize()
    assert torch.equal(a, ref) and torch.equal(c, ref)
    got = a.cpu().numpy().astype(np.float64).reshape(st.dims, order="F")
    assert _rel(got, oracle.first_stage(X, *mats)) <= TOL
    st.close()
