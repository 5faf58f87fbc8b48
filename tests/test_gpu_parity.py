"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element / per
replica on the same seeded inputs.  Tolerances (relative Frobenius error per replica, the
benchmark contract): 1e-5 on fp32 paths, 2e-2 on bf16-input/fp32-accumulate paths."""
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
TOL_BF16 = 2e-2


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True)
def _announce(request):
    _say("[case] " + request.node.nodeid)
    os.environ.pop("EXAT_RT", None)
    yield
    torch.cuda.synchronize()


SMALL = {
    "tiny": dict(I=24, J=20, K=28, R=3, P=3, L=5, M=4, N=6, dI=12, dJ=10, dK=7),
    "odd_scalar_path": dict(I=37, J=29, K=11, R=4, P=21, L=7, M=33, N=5, dI=37, dJ=29, dK=11),
    "two_row_groups": dict(I=64, J=140, K=9, R=5, P=9, L=32, M=16, N=3, dI=32, dJ=70, dK=3),
    "l_below_tile": dict(I=40, J=36, K=10, R=2, P=40, L=4, M=3, N=2, dI=20, dJ=12, dK=5),
    "ragged_j_chunks": dict(I=100, J=300, K=6, R=6, P=2, L=50, M=50, N=50, dI=50, dJ=150, dK=3),
}


def _inputs(cfg):
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    return A, B, C, U, V, W


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("rt", [0, 1, 4])
def test_compress_materialised_fp32_small(name, rt):
    cfg = wl.small(name=name, index=200 + list(SMALL).index(name), **SMALL[name])
    if rt:
        os.environ["EXAT_RT"] = str(rt)
    A, B, C, U, V, W = _inputs(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    plan = gu.plan_with_factors(cfg, U, V, W)
    Y = gu.y_to_numpy(plan.compress(gu.to_dev_x(X)), cfg)
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    err = oracle.rel_fro(Y, Yo)
    _say("  rel_fro=%.3e" % err)
    assert err <= TOL_F32
    plan.close()


def test_compress_is_bit_identical_run_to_run():
    cfg = wl.small(name="det", index=210, **SMALL["two_row_groups"])
    A, B, C, U, V, W = _inputs(cfg)
    X = gu.to_dev_x(oracle.gen_box(A, B, C, cfg.seed, cfg.sigma))
    plan = gu.plan_with_factors(cfg, U, V, W)
    y1 = plan.compress(X).clone()
    y2 = plan.compress(X).clone()
    assert torch.equal(y1, y2)
    plan.close()


def _worst_element(Y, Yo):
    """Largest element error of any replica, in units of the root mean square of that replica's exact entries."""
    d = np.abs(Y - Yo).reshape(-1, Y.shape[-1]).max(axis=0)
    rms = np.sqrt((Yo.reshape(-1, Yo.shape[-1]) ** 2).mean(axis=0))
    return float((d / rms).max())


def test_cfg1_full_parity():
    cfg = wl.CONFIGS["cfg1"]
    A, B, C, U, V, W = _inputs(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    plan = gu.plan_with_factors(cfg, U, V, W)
    Y = gu.y_to_numpy(plan.compress(gu.to_dev_x(X)), cfg)
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    err = oracle.rel_fro(Y, Yo)
    _say("  cfg1 rel_fro=%.3e" % err)
    assert err <= TOL_F32
    # the same tensor produced on the GPU by the block generator, then compressed
    Xg = torch.empty(cfg.elements, dtype=torch.float32, device="cuda")
    exat.gen_block(gu.desc_of(cfg), gu.gen_of(cfg, A, B, C), 0, 0, 0, Xg)
    Y2 = gu.y_to_numpy(plan.compress(Xg), cfg)
    err2 = oracle.rel_fro(Y2, Yo)
    _say("  cfg1 (GPU-generated X) rel_fro=%.3e" % err2)
    assert err2 <= TOL_F32
    # and never materialised
    Y3 = gu.y_to_numpy(plan.compress_gen(gu.gen_of(cfg, A, B, C)), cfg)
    err3 = oracle.rel_fro(Y3, Yo)
    _say("  cfg1 (generated in kernel) rel_fro=%.3e" % err3)
    assert err3 <= TOL_F32
    # element by element: no entry of any replica is off by more than the tolerance times the replica's rms entry (the
    # Frobenius figure is an average; an error of fp32 rounding size with Gaussian tails stays below 5 times its rms)
    worst = max(_worst_element(Y, Yo), _worst_element(Y2, Yo), _worst_element(Y3, Yo))
    _say("  cfg1 worst element error / rms entry: %.3e" % worst)
    assert worst <= TOL_F32
    plan.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gen_block_matches_oracle_elementwise(dtype):
    cfg = wl.small(name="gen", index=220, I=52, J=18, K=10, R=7, dI=26, dJ=9, dK=5, dtype=dtype)
    A, B, C = wl.cp_factors(cfg)
    desc = gu.desc_of(cfg)
    gen = gu.gen_of(cfg, A, B, C)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    for (bi, bj, bk) in [(0, 0, 0), (1, 1, 1), (1, 0, 1)]:
        out = torch.empty(cfg.dI * cfg.dJ * cfg.dK, dtype=tdt, device="cuda")
        exat.gen_block(desc, gen, bi, bj, bk, out)
        got = out.float().cpu().numpy().reshape((cfg.dI, cfg.dJ, cfg.dK), order="F")
        box = (bi * cfg.dI, (bi + 1) * cfg.dI, bj * cfg.dJ, (bj + 1) * cfg.dJ, bk * cfg.dK, (bk + 1) * cfg.dK)
        want = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, box, to_bf16=(dtype == "bf16"))
        diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
        scale = 1.0 + np.abs(want).max()
        if dtype == "f32":
            _say("  block %s max|diff|=%.3e (scale %.1f)" % ((bi, bj, bk), diff.max(), scale))
            assert diff.max() <= 2e-6 * scale        # fp32 evaluation of an R-term sum vs fp64-then-round
        else:
            flips = (diff > 0).mean()
            _say("  block %s bf16 flips=%.2e max|diff|=%.3e" % ((bi, bj, bk), flips, diff.max()))
            assert flips <= 5e-3 and np.all(diff <= np.abs(want) * 2.0 ** -7 + 1e-30)


def test_noise_alone_matches_oracle():
    # zero factors: the block is sigma * g exactly
    cfg = wl.small(name="noise", index=221, I=64, J=33, K=9, R=1, dI=64, dJ=33, dK=9, sigma=1.0)
    Z = np.zeros((cfg.I, 1), np.float32, order="F")
    gen = exat.make_gen(gu.to_dev_factor(Z), gu.to_dev_factor(np.zeros((cfg.J, 1), np.float32)),
                        gu.to_dev_factor(np.zeros((cfg.K, 1), np.float32)), cfg.seed, 1.0)
    out = torch.empty(cfg.elements, dtype=torch.float32, device="cuda")
    exat.gen_block(gu.desc_of(cfg), gen, 0, 0, 0, out)
    got = out.cpu().numpy().astype(np.float64).reshape((cfg.I, cfg.J, cfg.K), order="F")
    want = oracle.noise_box(cfg.seed, (0, cfg.I, 0, cfg.J, 0, cfg.K))
    d = np.abs(got - want).max()
    _say("  max|g_gpu - g_oracle| = %.3e" % d)
    assert d <= 5e-6   # hardware log2/sqrt/sin/cos in fp32 against libm in fp64, |g| < 4.9


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_gen_small_and_subboxes(dtype):
    cfg = wl.small(name="cgen", index=230, I=100, J=60, K=12, R=5, P=6, L=10, M=9, N=8, dI=50, dJ=30, dK=4, dtype=dtype)
    A, B, C, U, V, W = _inputs(cfg)
    plan = gu.plan_with_factors(cfg, U, V, W)
    gen = gu.gen_of(cfg, A, B, C)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    Y = gu.y_to_numpy(plan.compress_gen(gen), cfg)
    err = oracle.rel_fro(Y, Yo)
    _say("  full: rel_fro=%.3e" % err)
    assert err <= (TOL_BF16 if dtype == "bf16" else TOL_F32)
    if dtype == "bf16":
        # against the oracle on bf16-rounded inputs: isolates kernel errors from quantisation
        rb = oracle.round_bf16
        Yr = oracle.comp_multi(np.asfortranarray(rb(X.reshape(-1, order="F")).reshape(X.shape, order="F")),
                               rb(U), rb(V), rb(W), cfg.P)
        err_r = oracle.rel_fro(Y, Yr)
        _say("  full vs oracle on bf16-rounded inputs: rel_fro=%.3e" % err_r)
        assert err_r <= 5e-4
    # sub-boxes, including ones that are not aligned to anything
    acc = np.zeros_like(Yo)
    boxes = [(0, 50, 0, 30, 0, 4), (50, 100, 30, 60, 8, 12), (13, 71, 7, 41, 3, 10)]
    for box in boxes:
        Yb = gu.y_to_numpy(plan.compress_gen(gen, box), cfg)
        i0, i1, j0, j1, k0, k1 = box
        Xb = np.asfortranarray(X[i0:i1, j0:j1, k0:k1])
        Yob = oracle.comp_box(Xb, U, V, W, cfg.P, box)
        e = oracle.rel_fro(Yb, Yob)
        _say("  box %s rel_fro=%.3e" % (box, e))
        assert e <= (TOL_BF16 if dtype == "bf16" else TOL_F32)
    plan.close()


def test_block_streamed_equals_one_shot_and_is_order_independent():
    cfg = wl.small(name="blk", index=240, I=48, J=40, K=12, R=4, P=5, L=6, M=7, N=4, dI=16, dJ=20, dK=4)
    A, B, C, U, V, W = _inputs(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    plan = gu.plan_with_factors(cfg, U, V, W)
    blocks = [(bi, bj, bk) for bi in range(3) for bj in range(2) for bk in range(3)]

    def run(order):
        for (bi, bj, bk) in order:
            Xb = np.asfortranarray(X[bi * 16:(bi + 1) * 16, bj * 20:(bj + 1) * 20, bk * 4:(bk + 1) * 4])
            plan.compress_block(gu.to_dev_x(Xb), bi, bj, bk)
        return plan.finalize().clone()

    y1 = run(blocks)
    y2 = run(list(reversed(blocks)))
    assert torch.equal(y1, y2)
    err = oracle.rel_fro(gu.y_to_numpy(y1, cfg), Yo)
    _say("  block-streamed rel_fro=%.3e" % err)
    assert err <= TOL_F32
    # state errors: finalize with nothing, a block twice, an index out of range
    with pytest.raises(exat.ExatError) as e:
        plan.finalize()
    assert e.value.status == exat.ERR_STATE
    Xb = gu.to_dev_x(np.asfortranarray(X[:16, :20, :4]))
    plan.compress_block(Xb, 0, 0, 0)
    with pytest.raises(exat.ExatError) as e:
        plan.compress_block(Xb, 0, 0, 0)
    assert e.value.status == exat.ERR_STATE
    with pytest.raises(exat.ExatError) as e:
        plan.compress_block(Xb, 3, 0, 0)
    assert e.value.status == exat.ERR_SHAPE
    plan.finalize()
    plan.close()


def test_compress_before_set_factors_is_a_state_error():
    cfg = wl.small()
    plan = exat.Plan(gu.desc_of(cfg))
    X = torch.zeros(cfg.elements, dtype=torch.float32, device="cuda")
    with pytest.raises(exat.ExatError) as e:
        plan.compress(X)
    assert e.value.status == exat.ERR_STATE
    plan.close()


def test_compress_materialised_bf16_small():
    cfg = wl.small(name="bf16mat", index=250, I=96, J=72, K=10, R=4, P=7, L=50, M=50, N=50, dI=48, dJ=36, dK=5, dtype="bf16")
    A, B, C, U, V, W = _inputs(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, to_bf16=True)      # exactly representable in bf16
    plan = gu.plan_with_factors(cfg, U, V, W)
    Y = gu.y_to_numpy(plan.compress(gu.to_dev_x(X, bf16=True)), cfg)
    rb = oracle.round_bf16
    Yr = oracle.comp_multi(X, rb(U), rb(V), rb(W), cfg.P)
    err_r = oracle.rel_fro(Y, Yr)
    Yo = oracle.comp_multi(oracle.gen_box(A, B, C, cfg.seed, cfg.sigma), U, V, W, cfg.P)
    err = oracle.rel_fro(Y, Yo)
    _say("  bf16 materialised: vs rounded-input oracle %.3e, vs fp32-input oracle %.3e" % (err_r, err))
    assert err_r <= 1e-5
    assert err <= TOL_BF16
    plan.close()


# Every instantiation of the pipelined kernel at sizes the oracle finishes in seconds: 4- and 8-wave
# workgroups (P*L above / below 256 stacked rows), both generator depths (R <= 32, R <= 64), sub-range
# boxes, several row groups, ragged last column chunk.
PIPELINED = {
    "f32_8w_r32": dict(dtype="f32", I=96, J=150, K=5, R=20, P=9, L=40, M=33, N=7, dI=48, dJ=75, dK=5),
    "f32_8w_r64": dict(dtype="f32", I=64, J=130, K=4, R=50, P=20, L=32, M=20, N=9, dI=32, dJ=65, dK=2),
    "f32_4w_r64": dict(dtype="f32", I=80, J=40, K=6, R=40, P=4, L=50, M=50, N=50, dI=40, dJ=20, dK=3),
    "bf16_4w_r32": dict(dtype="bf16", I=96, J=140, K=5, R=32, P=5, L=50, M=50, N=50, dI=48, dJ=70, dK=5),
    "bf16_4w_r64": dict(dtype="bf16", I=64, J=40, K=6, R=64, P=3, L=64, M=64, N=64, dI=32, dJ=20, dK=3),
}


@pytest.mark.parametrize("name", list(PIPELINED))
def test_pipelined_generator_variants(name):
    kw = dict(PIPELINED[name])
    cfg = wl.small(name=name, index=300 + list(PIPELINED).index(name), **kw)
    A, B, C, U, V, W = _inputs(cfg)
    plan = gu.plan_with_factors(cfg, U, V, W)
    gen = gu.gen_of(cfg, A, B, C)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    tol = TOL_BF16 if cfg.dtype == "bf16" else TOL_F32
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    e = oracle.rel_fro(gu.y_to_numpy(plan.compress_gen(gen), cfg), Yo)
    _say("  %s full: rel_fro=%.3e" % (name, e))
    assert e <= tol
    box = (cfg.dI // 2, cfg.I - 3, 5, cfg.J - 1, 1, cfg.K)          # proper sub-range in every mode
    Xb = np.asfortranarray(X[box[0]:box[1], box[2]:box[3], box[4]:box[5]])
    eb = oracle.rel_fro(gu.y_to_numpy(plan.compress_gen(gen, box), cfg), oracle.comp_box(Xb, U, V, W, cfg.P, box))
    _say("  %s box %s: rel_fro=%.3e" % (name, box, eb))
    assert eb <= tol
    plan.close()


@pytest.mark.parametrize("dtype,P,L", [("f32", 20, 32), ("f32", 3, 50), ("bf16", 11, 50), ("bf16", 4, 40)])
def test_pipelined_materialised_variants(dtype, P, L):
    cfg = wl.small(name="pipe_mat", index=320 + P, dtype=dtype, I=96, J=200, K=4, R=6, P=P, L=L, M=L, N=9, dI=32, dJ=100, dK=2)
    A, B, C, U, V, W = _inputs(cfg)
    bf = dtype == "bf16"
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, to_bf16=bf)
    plan = gu.plan_with_factors(cfg, U, V, W)
    rb = oracle.round_bf16 if bf else (lambda a: a)
    Yo = oracle.comp_multi(X, rb(U), rb(V), rb(W), cfg.P)
    Xd = gu.to_dev_x(X, bf16=bf)
    e = oracle.rel_fro(gu.y_to_numpy(plan.compress(Xd), cfg), Yo)
    # the same through the block-streamed entry point (blocks are whole 64-byte stages of i)
    Xv = Xd.view(cfg.K, cfg.J, cfg.I)
    for bk in range(cfg.K // cfg.dK):
        for bj in range(cfg.J // cfg.dJ):
            for bi in range(cfg.I // cfg.dI):
                blk = Xv[bk * cfg.dK:(bk + 1) * cfg.dK, bj * cfg.dJ:(bj + 1) * cfg.dJ, bi * cfg.dI:(bi + 1) * cfg.dI].contiguous()
                plan.compress_block(blk, bi, bj, bk)
    eb = oracle.rel_fro(gu.y_to_numpy(plan.finalize(), cfg), Yo)
    _say("  %s P=%d L=%d: one shot %.3e, block-streamed %.3e" % (dtype, P, L, e, eb))
    assert max(e, eb) <= 1e-5
    plan.close()


# The stage loop of the fragment-ordered kernel is unrolled by the number of register sets (2 for fp32, 6 for
# bf16 materialised tiles) and finishes with a guarded remainder: every stage count from 1 up to past two
# unrolled bodies, for the 4- and the 8-wave tile, materialised and generated.
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("P", [2, 6])
def test_stage_count_sweep(dtype, P):
    ei = 32 if dtype == "bf16" else 16
    worst_m, worst_g = 0.0, 0.0
    for nstage in (1, 2, 3, 5, 6, 7, 13):
        cfg = wl.small(name="stages", index=400 + nstage, dtype=dtype, I=ei * nstage, J=140, K=3, R=5, P=P, L=50, M=34, N=5,
                       dI=ei * nstage, dJ=70, dK=3)
        A, B, C, U, V, W = _inputs(cfg)
        plan = gu.plan_with_factors(cfg, U, V, W)
        bf = dtype == "bf16"
        X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, to_bf16=bf)
        rb = oracle.round_bf16 if bf else (lambda a: a)
        Yr = oracle.comp_multi(X, rb(U), rb(V), rb(W), cfg.P)
        em = oracle.rel_fro(gu.y_to_numpy(plan.compress(gu.to_dev_x(X, bf16=bf)), cfg), Yr)
        Yo = oracle.comp_multi(oracle.gen_box(A, B, C, cfg.seed, cfg.sigma), U, V, W, cfg.P)
        eg = oracle.rel_fro(gu.y_to_numpy(plan.compress_gen(gu.gen_of(cfg, A, B, C)), cfg), Yo)
        _say("  %s P=%d stages=%d: materialised %.3e, generated %.3e" % (dtype, P, nstage, em, eg))
        worst_m, worst_g = max(worst_m, em), max(worst_g, eg)
        plan.close()
    assert worst_m <= 1e-5
    assert worst_g <= (TOL_BF16 if dtype == "bf16" else TOL_F32)


# bf16 generator: 384-row groups plus a remainder launch with a 128- or 256-row tile (P*L = 450, 600),
# and the case where the remainder is a group of its own (P*L = 700 = 384 + 316).
@pytest.mark.parametrize("P", [9, 12, 14])
def test_bf16_generator_remainder_rows(P):
    cfg = wl.small(name="remainder", index=420 + P, dtype="bf16", I=96, J=140, K=4, R=20, P=P, L=50, M=50, N=6, dI=48, dJ=70, dK=2)
    A, B, C, U, V, W = _inputs(cfg)
    plan = gu.plan_with_factors(cfg, U, V, W)
    gen = gu.gen_of(cfg, A, B, C)
    Yo = oracle.comp_multi(oracle.gen_box(A, B, C, cfg.seed, cfg.sigma), U, V, W, cfg.P)
    e = oracle.rel_fro(gu.y_to_numpy(plan.compress_gen(gen), cfg), Yo)
    box = (48, 96, 0, 70, 1, 3)
    Yb = oracle.comp_box(oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, box), U, V, W, cfg.P, box)
    eb = oracle.rel_fro(gu.y_to_numpy(plan.compress_gen(gen, box), cfg), Yb)
    _say("  P*L=%d: full %.3e, box %.3e" % (P * 50, e, eb))
    assert max(e, eb) <= TOL_BF16
    plan.close()


# fp32 data on the fp16 matrix cores (two-piece operands, Eq. 5's residual split): same tolerance as the fp32 path.
# Stage counts around the unrolled loop, row counts that take the 1-, 2- and 3-tile variants and a remainder
# launch, M above and below 32, a ragged last column chunk, block streaming, and a box the split kernel does not
# cover (falls back to the fp32 kernels).
@pytest.mark.parametrize("P", [2, 5, 9, 14])
def test_split_fp16_matches_oracle(P):
    worst = 0.0
    for nstage, M in ((1, 34), (2, 20), (3, 50), (5, 34), (8, 64)):
        cfg = wl.small(name="split", index=440 + nstage, dtype="f32s", I=32 * nstage, J=140, K=3, R=5, P=P, L=50, M=M, N=5,
                       dI=32 * nstage, dJ=70, dK=3)
        A, B, C, U, V, W = _inputs(cfg)
        plan = gu.plan_with_factors(cfg, U, V, W)
        X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
        Yo = oracle.comp_multi(X, U, V, W, cfg.P)
        e = oracle.rel_fro(gu.y_to_numpy(plan.compress(gu.to_dev_x(X)), cfg), Yo)
        _say("  P*L=%d stages=%d M=%d: %.3e" % (P * 50, nstage, M, e))
        worst = max(worst, e)
        plan.close()
    assert worst <= TOL_F32


def test_split_fp16_block_streamed_and_fallbacks():
    cfg = wl.small(name="splitblk", index=450, dtype="f32s", I=96, J=60, K=8, R=6, P=7, L=40, M=33, N=9, dI=32, dJ=30, dK=4)
    A, B, C, U, V, W = _inputs(cfg)
    plan = gu.plan_with_factors(cfg, U, V, W)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    for bk in range(2):
        for bj in range(2):
            for bi in range(3):
                Xb = np.asfortranarray(X[bi * 32:(bi + 1) * 32, bj * 30:(bj + 1) * 30, bk * 4:(bk + 1) * 4])
                plan.compress_block(gu.to_dev_x(Xb), bi, bj, bk)
    e_blk = oracle.rel_fro(gu.y_to_numpy(plan.finalize(), cfg), Yo)
    e_gen = oracle.rel_fro(gu.y_to_numpy(plan.compress_gen(gu.gen_of(cfg, A, B, C)), cfg), Yo)   # fp32 generator kernels
    plan.close()
    # extent 37 is not a multiple of the stage: fp32 kernels
    cfg2 = wl.small(name="splitodd", index=451, dtype="f32s", I=37, J=29, K=5, R=4, P=3, L=7, M=5, N=4, dI=37, dJ=29, dK=5)
    A, B, C, U, V, W = _inputs(cfg2)
    plan = gu.plan_with_factors(cfg2, U, V, W)
    X = oracle.gen_box(A, B, C, cfg2.seed, cfg2.sigma)
    e_odd = oracle.rel_fro(gu.y_to_numpy(plan.compress(gu.to_dev_x(X)), cfg2), oracle.comp_multi(X, U, V, W, cfg2.P))
    plan.close()
    _say("  block-streamed %.3e, generated %.3e, odd extents %.3e" % (e_blk, e_gen, e_odd))
    assert max(e_blk, e_gen, e_odd) <= TOL_F32


@pytest.mark.parametrize("case", ["small_noncubic", "cfg1", "bf16_small"])
def test_host_streamed_matches_block_sequence_and_oracle(case):
    """exat_compress_host: blocks copied from (pinned or pageable) host memory on the plan's copy stream while the
    previous ones are compressed.  Bit-identical to the same exat_compress_block sequence; two passes in a row
    exercise the reuse of the ring buffers."""
    if case == "cfg1":
        cfg = wl.CONFIGS["cfg1"]
        cfg = type(cfg)(**{**cfg.__dict__, "dI": 64, "dJ": 32, "dK": 64})      # 2 x 4 x 2 = 16 non-cubic blocks
    elif case == "bf16_small":
        cfg = wl.small(I=48, J=40, K=28, dI=16, dJ=8, dK=7, dtype="bf16", P=3, L=6, M=5, N=4)
    else:
        cfg = wl.small()                                                        # 24x20x28 in 12x10x7 blocks
    print("case", case, flush=True)
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma)
    bf = cfg.dtype == "bf16"
    Xflat = torch.from_numpy(np.ascontiguousarray(X.reshape(-1, order="F")))
    if bf:
        Xflat = Xflat.to(torch.bfloat16)
    plan = gu.plan_with_factors(cfg, U, V, W)
    # reference: the same blocks through exat_compress_block, same order
    Xd = Xflat.cuda().view(cfg.K, cfg.J, cfg.I)
    for bk in range(cfg.K // cfg.dK):
        for bj in range(cfg.J // cfg.dJ):
            for bi in range(cfg.I // cfg.dI):
                blk = Xd[bk * cfg.dK:(bk + 1) * cfg.dK, bj * cfg.dJ:(bj + 1) * cfg.dJ, bi * cfg.dI:(bi + 1) * cfg.dI].contiguous()
                plan.compress_block(blk, bi, bj, bk)
    Yref = plan.finalize().clone()
    Y1 = plan.compress_host(Xflat.pin_memory()).clone()
    Y2 = plan.compress_host(Xflat.clone()).clone()              # pageable memory, second pass over the ring
    torch.cuda.synchronize()
    assert torch.equal(Y1, Yref) and torch.equal(Y2, Yref)
    Xo = Xflat.float().numpy().reshape((cfg.I, cfg.J, cfg.K), order="F") if bf else X
    err = oracle.rel_fro(gu.y_to_numpy(Y1, cfg), oracle.comp_multi(np.asfortranarray(Xo), U, V, W, cfg.P))
    print("  rel_fro=%.3e" % err, flush=True)
    assert err <= (2e-2 if bf else 1e-5)      # bf16: U, V, W are rounded inside the plan as well
    plan.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_blocks(dtype):
    """Block edges that do not divide the extents: the last block of an axis is shorter.  Blocks through
    exat_gen_block / exat_compress_block, the same tensor through exat_compress_host and in one shot."""
    cfg = wl.small(I=24, J=20, K=28, dI=10, dJ=8, dK=9, dtype=dtype)     # blocks 10,10,4 x 8,8,4 x 9,9,9,1
    print("case ragged", dtype, flush=True)
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    bf = dtype == "bf16"
    tdt = torch.bfloat16 if bf else torch.float32
    plan = gu.plan_with_factors(cfg, U, V, W)
    desc, gen = gu.desc_of(cfg), gu.gen_of(cfg, A, B, C)
    cuts = lambda n, d: [(o, min(n, o + d)) for o in range(0, n, d)]
    for bk, (k0, k1) in enumerate(cuts(cfg.K, cfg.dK)):
        for bj, (j0, j1) in enumerate(cuts(cfg.J, cfg.dJ)):
            for bi, (i0, i1) in enumerate(cuts(cfg.I, cfg.dI)):
                blk = torch.empty((i1 - i0) * (j1 - j0) * (k1 - k0), dtype=tdt, device="cuda")
                exat.gen_block(desc, gen, bi, bj, bk, blk)
                ref = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, (i0, i1, j0, j1, k0, k1), to_bf16=bf)
                got = blk.float().cpu().numpy().reshape(ref.shape, order="F")
                assert np.abs(got - ref).max() <= (0.05 if bf else 2e-6 * (1 + np.abs(ref).max()))
                plan.compress_block(blk, bi, bj, bk)
    Yb = plan.finalize().clone()
    X = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, to_bf16=bf)
    Xflat = torch.from_numpy(np.ascontiguousarray(X.reshape(-1, order="F"))).to(tdt)
    Yh = plan.compress_host(Xflat.pin_memory()).clone()
    Y1 = plan.compress(Xflat.cuda()).clone()
    torch.cuda.synchronize()
    Yo = oracle.comp_multi(X, U, V, W, cfg.P)
    tol = 2e-2 if bf else 1e-5
    for name, Y in (("blocks", Yb), ("host", Yh), ("one shot", Y1)):
        err = oracle.rel_fro(gu.y_to_numpy(Y, cfg), Yo)
        print("  %s rel_fro=%.3e" % (name, err), flush=True)
        assert err <= tol
    L = exat.lib()
    assert L.exat_compress_block(plan._h, ctypes.c_void_p(Xflat.cuda().data_ptr()), 3, 0, 0, None) == exat.ERR_SHAPE   # 3 blocks along i
    plan.close()
