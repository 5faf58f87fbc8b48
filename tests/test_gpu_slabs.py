"""GPU parity of exat_compress_blocks: slabs of resident blocks (whole block columns along i) compressed in one
launch through a table of block pointers, against the CPU oracle and against the other entry points."""
import ctypes
import os
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2311_13693_amd import exat
import workloads as wl

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import gpu_util as gu  # noqa: E402

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True)
def _announce(request):
    _say("[case] " + request.node.nodeid)
    for v in ("EXAT_RT", "EXAT_SLAB"):
        os.environ.pop(v, None)
    yield
    for v in ("EXAT_RT", "EXAT_SLAB"):
        os.environ.pop(v, None)
    torch.cuda.synchronize()


def _inputs(cfg):
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    return A, B, C, U, V, W


def _nb(n, d):
    return (n + d - 1) // d


def _block(X, cfg, bi, bj, bk):
    return gu.to_dev_x(np.asfortranarray(X[bi * cfg.dI:(bi + 1) * cfg.dI, bj * cfg.dJ:(bj + 1) * cfg.dJ, bk * cfg.dK:(bk + 1) * cfg.dK]),
                       bf16=cfg.dtype == "bf16")


def _slab(X, cfg, bj0, bj1, bk0, bk1):
    return [_block(X, cfg, bi, bj, bk) for bk in range(bk0, bk1) for bj in range(bj0, bj1) for bi in range(_nb(cfg.I, cfg.dI))]


# shapes the one-launch kernels take (dI a multiple of the stage, 16 fp32 / 32 bf16 values, that divides I; dJ % 128 == 0);
# ragged last blocks along j and k; mode 2 from the accumulators (L % 32 == 0) and through LDS; fp32 and bf16 plans
CASES = {
    "two_by_two_by_two": dict(I=64, J=256, K=6, R=4, P=3, L=32, M=8, N=5, dI=32, dJ=128, dK=3),
    "ragged_j_and_k": dict(I=96, J=300, K=7, R=3, P=2, L=32, M=33, N=4, dI=32, dJ=128, dK=3),
    "two_row_groups_l64": dict(I=48, J=128, K=5, R=5, P=10, L=64, M=20, N=3, dI=16, dJ=128, dK=2),
    "l50_mode2_through_lds": dict(I=64, J=200, K=5, R=4, P=7, L=50, M=50, N=6, dI=16, dJ=128, dK=3),
    "forty_eight_blocks": dict(I=64, J=384, K=4, R=3, P=2, L=32, M=6, N=4, dI=16, dJ=128, dK=1),   # two launches fill the pointer table
    "split_fp16": dict(I=128, J=300, K=5, R=4, P=9, L=32, M=20, N=6, dI=32, dJ=128, dK=2, dtype="f32s"),   # 288 rows: a remainder launch too
    "bf16": dict(I=128, J=300, K=5, R=4, P=7, L=50, M=50, N=6, dI=64, dJ=128, dK=2, dtype="bf16"),
}


@pytest.mark.parametrize("rt", ["default", "4"])
@pytest.mark.parametrize("name", list(CASES))
def test_slabs_match_oracle_one_shot_and_any_order(name, rt):
    if rt != "default":
        os.environ["EXAT_RT"] = rt
    cfg = wl.small(name=name, index=700 + list(CASES).index(name), **CASES[name])
    A, B, C, U, V, W = _inputs(cfg)
    bf = cfg.dtype == "bf16"
    # bf16 plans: a tensor that is exactly representable in bf16, against the oracle on bf16-rounded matrices (what
    # isolates the kernel from the quantisation of its inputs)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, to_bf16=bf)
    rb = oracle.round_bf16 if bf else (lambda a: a)
    Yo = oracle.comp_multi(X, rb(U), rb(V), rb(W), cfg.P)
    plan = gu.plan_with_factors(cfg, U, V, W)
    nbj, nbk = _nb(cfg.J, cfg.dJ), _nb(cfg.K, cfg.dK)
    # one slab that holds every block: the same launches as the one-shot call, so the same bits
    y_one = plan.compress(gu.to_dev_x(X, bf16=bf)).clone()
    plan.compress_blocks(_slab(X, cfg, 0, nbj, 0, nbk), 0, nbj, 0, nbk)
    y_all = plan.finalize().clone()
    assert torch.equal(y_one, y_all)
    # one slab per block column, in two orders: same bits; against the oracle within the fp32 tolerance
    cols = [(bj, bk) for bk in range(nbk) for bj in range(nbj)]

    def run(order):
        for bj, bk in order:
            plan.compress_blocks(_slab(X, cfg, bj, bj + 1, bk, bk + 1), bj, bj + 1, bk, bk + 1)
        return plan.finalize().clone()

    y1, y2 = run(cols), run(cols[::-1])
    assert torch.equal(y1, y2)
    e_all, e_cols = oracle.rel_fro(gu.y_to_numpy(y_all, cfg), Yo), oracle.rel_fro(gu.y_to_numpy(y1, cfg), Yo)
    _say("  %s: one slab %.3e, one slab per column %.3e" % (name, e_all, e_cols))
    assert max(e_all, e_cols) <= TOL_F32
    plan.close()


def test_slabs_and_single_blocks_in_one_pass():
    cfg = wl.small(name="slab_mix", index=710, **CASES["two_by_two_by_two"])
    A, B, C, U, V, W = _inputs(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    plan = gu.plan_with_factors(cfg, U, V, W)
    plan.compress_blocks(_slab(X, cfg, 0, 2, 0, 1), 0, 2, 0, 1)        # layer bk = 0 as a slab
    for bj in range(2):
        for bi in range(2):
            plan.compress_block(_block(X, cfg, bi, bj, 1), bi, bj, 1)    # layer bk = 1 block by block
    err = oracle.rel_fro(gu.y_to_numpy(plan.finalize(), cfg), Yo)
    _say("  slab + single blocks rel_fro=%.3e" % err)
    assert err <= TOL_F32
    plan.close()


@pytest.mark.parametrize("why", ["l_not_multiple_of_32", "switched_off"])
def test_slab_that_does_not_qualify_runs_block_by_block(why):
    """Bit-identical to the same exat_compress_block sequence, and within tolerance of the oracle."""
    if why == "switched_off":
        os.environ["EXAT_SLAB"] = "0"
        cfg = wl.small(name="slab_off", index=721, **CASES["two_by_two_by_two"])
    else:
        cfg = wl.small(name="slab_fb", index=720, I=48, J=40, K=12, R=4, P=5, L=6, M=7, N=4, dI=16, dJ=20, dK=4)
    A, B, C, U, V, W = _inputs(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    plan = gu.plan_with_factors(cfg, U, V, W)
    nbi, nbj, nbk = _nb(cfg.I, cfg.dI), _nb(cfg.J, cfg.dJ), _nb(cfg.K, cfg.dK)
    plan.compress_blocks(_slab(X, cfg, 0, nbj, 0, nbk), 0, nbj, 0, nbk)
    y_slab = plan.finalize().clone()
    for bk in range(nbk):
        for bj in range(nbj):
            for bi in range(nbi):
                plan.compress_block(_block(X, cfg, bi, bj, bk), bi, bj, bk)
    y_blk = plan.finalize().clone()
    assert torch.equal(y_slab, y_blk)
    assert oracle.rel_fro(gu.y_to_numpy(y_slab, cfg), Yo) <= TOL_F32
    plan.close()


def test_slab_errors():
    cfg = wl.small(name="slab_err", index=730, **CASES["two_by_two_by_two"])
    A, B, C, U, V, W = _inputs(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    plan = gu.plan_with_factors(cfg, U, V, W)
    col = _slab(X, cfg, 0, 1, 0, 1)
    for rng in ((0, 0, 0, 1), (0, 3, 0, 1), (-1, 1, 0, 1), (0, 1, 1, 1), (0, 1, 0, 3)):
        with pytest.raises(exat.ExatError) as e:
            plan.compress_blocks(col * 4, *rng)
        assert e.value.status == exat.ERR_SHAPE
    plan.compress_blocks(col, 0, 1, 0, 1)
    with pytest.raises(exat.ExatError) as e:
        plan.compress_blocks(col, 0, 1, 0, 1)          # the same column twice
    assert e.value.status == exat.ERR_STATE
    with pytest.raises(exat.ExatError) as e:
        plan.compress_block(col[0], 0, 0, 0)           # one of its blocks again
    assert e.value.status == exat.ERR_STATE
    L = exat.lib()
    arr = (ctypes.c_void_p * 2)(col[0].data_ptr(), None)
    assert L.exat_compress_blocks(plan._h, arr, 1, 2, 0, 1, None) == exat.ERR_NULL
    assert L.exat_compress_blocks(plan._h, None, 1, 2, 0, 1, None) == exat.ERR_NULL
    plan.finalize()
    plan.close()
