"""The launch-bound entry points (many short kernels per call: the CGLS iterations of exat_ls, the sweeps of
exat_cpals) and exat_compress only enqueue kernels on the caller's stream -- no allocation, no memset, no
synchronisation -- so a caller may record them into a HIP graph and replay it.  Each test captures one call,
replays the graph several times with eager work and synchronisations of its own in between, and compares every
replay bit for bit with the eager result."""
import numpy as np
import pytest
import torch

from paper_2311_13693_amd import exat

pytestmark = pytest.mark.gpu


def _capture(fn):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()                      # warm-up outside the capture, as torch asks
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    torch.cuda.synchronize()
    return g


def _replays_match(g, outputs, eager):
    junk = torch.randn(1 << 16, device="cuda")
    for rep in range(3):
        for o in outputs:
            o.fill_(float("nan"))
        (junk * 2).sum().item()   # the program's own eager work and a synchronisation between replays
        g.replay()
        torch.cuda.synchronize()
        for o, e in zip(outputs, eager):
            assert torch.equal(o, e), "replay %d differs from the eager result" % rep


def test_ls_in_a_graph():
    P, L, I, R = 6, 16, 40, 5
    gen = torch.Generator(device="cpu").manual_seed(1)
    U = (torch.randn(P * L, I, generator=gen) / 4).cuda()
    A = torch.randn(P * L * R, generator=gen).cuda()
    X, rel = torch.empty(I * R, device="cuda"), torch.empty(R, device="cuda")
    work = torch.empty(exat.lib().exat_ls_workspace_floats(P, L, I, R), device="cuda")
    run = lambda: exat.ls(U, P, L, I, A, R, 25, 1e-6, X, rel, work)
    run()
    torch.cuda.synchronize()
    eager = [X.clone(), rel.clone()]
    _replays_match(_capture(run), [X, rel], eager)


def test_cpals_in_a_graph():
    L, M, N, P, R = 10, 9, 8, 3, 3
    gen = torch.Generator(device="cpu").manual_seed(2)
    Y = torch.randn(P * L * M * N, generator=gen).cuda()
    S = [torch.randn(P * d * R, generator=gen).cuda() for d in (L, M, N)]
    F = [s.clone() for s in S]
    work = torch.empty(exat.lib().exat_cpals_workspace_floats(L, M, N, P), device="cuda")

    def run():
        for f, s in zip(F, S):
            f.copy_(s)            # start values restored inside the graph: the call works in place
        exat.cpals(Y, L, M, N, P, R, 4, F[0], F[1], F[2], work)
    run()
    torch.cuda.synchronize()
    eager = [f.clone() for f in F]
    _replays_match(_capture(run), F, eager)


def test_compress_in_a_graph():
    I, J, K, L, M, N, P = 64, 48, 40, 8, 8, 8, 4
    gen = torch.Generator(device="cpu").manual_seed(3)
    plan = exat.Plan(exat.make_desc(I, J, K, L, M, N, P, I, J, K, exat.EXAT_F32))
    plan.set_factors(*(torch.randn(P * d, n, generator=gen).cuda() for d, n in ((L, I), (M, J), (N, K))))
    X = torch.randn(I * J * K, generator=gen).cuda()
    Y = plan.new_y()
    run = lambda: plan.compress(X, Y)
    run()
    torch.cuda.synchronize()
    eager = [Y.clone()]
    _replays_match(_capture(run), [Y], eager)
    plan.close()


def test_block_streamed_pass_in_a_graph():
    """A whole block-streamed pass -- a slab through exat_compress_blocks (its table entries travel in the arguments of
    a small launch, nothing is copied from the host), single blocks through exat_compress_block, the merge of
    exat_finalize -- recorded once the first eager pass has made the plan's allocations."""
    I, J, K, L, M, N, P, dI, dJ, dK = 64, 256, 4, 32, 8, 6, 3, 32, 128, 2
    gen = torch.Generator(device="cpu").manual_seed(4)
    plan = exat.Plan(exat.make_desc(I, J, K, L, M, N, P, dI, dJ, dK, exat.EXAT_F32))
    plan.set_factors(*(torch.randn(P * d, n, generator=gen).cuda() for d, n in ((L, I), (M, J), (N, K))))
    blocks = {(bi, bj, bk): torch.randn(dI * dJ * dK, generator=gen).cuda() for bk in range(2) for bj in range(2) for bi in range(2)}
    Y = plan.new_y()

    def run():
        plan.compress_blocks([blocks[(bi, bj, 0)] for bj in range(2) for bi in range(2)], 0, 2, 0, 1)   # layer 0 as a slab
        for bj in range(2):
            for bi in range(2):
                plan.compress_block(blocks[(bi, bj, 1)], bi, bj, 1)                                      # layer 1 block by block
        plan.finalize(Y)
    run()                         # the allocating pass
    torch.cuda.synchronize()
    eager = [Y.clone()]
    _replays_match(_capture(run), [Y], eager)
    plan.close()
