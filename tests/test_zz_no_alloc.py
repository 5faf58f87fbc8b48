"""The allocation-free variant of the batched CP-ALS entry point (exat_cpals_noalloc: workspace in a static device
array) against exat_cpals with a caller-owned workspace, through the C ABI: same kernels, same order, so the factor
matrices must agree bit for bit.  Two calls in a row, the second on a smaller problem (the static array keeps the first
call's contents), then a problem that exceeds the static workspace, which must be refused."""
import numpy as np
import pytest
import torch

from paper_2311_13693_amd import exat

pytestmark = pytest.mark.gpu


def _inputs(seed, L, M, N, R, P):
    rng = np.random.default_rng(seed)
    Y = torch.from_numpy(rng.standard_normal(P * L * M * N).astype(np.float32)).cuda()
    start = [torch.from_numpy(rng.standard_normal(P * d * R).astype(np.float32)).cuda() for d in (L, M, N)]
    return Y, start


def _both(seed, L, M, N, R, P, sweeps):
    Y, start = _inputs(seed, L, M, N, R, P)
    ref = [s.clone() for s in start]
    exat.cpals(Y, L, M, N, P, R, sweeps, *ref)
    got = [s.clone() for s in start]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    exat.cpals_noalloc(Y, L, M, N, P, R, sweeps, *got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for g, r in zip(got, ref):
        assert torch.isfinite(r).all()
        assert torch.equal(g, r)


def test_noalloc_cpals_matches_workspace_variant_twice_second_smaller():
    print("[case] exat_cpals_noalloc 16 x 32^3 rank 16, 3 sweeps", flush=True)
    _both(11, 32, 32, 32, 16, 16, 3)       # cfg2's proxy tensors: 8 MiB of the 16 MiB array
    print("[case] exat_cpals_noalloc 4 x 16x12x9 rank 8, 2 sweeps (smaller, after the larger call)", flush=True)
    _both(12, 16, 12, 9, 8, 4, 2)


def test_noalloc_cpals_refuses_what_does_not_fit():
    L = M = N = 64
    P, R = 32, 32                          # cfg3's proxy tensors need 67 MB of workspace
    assert exat.lib().exat_cpals_workspace_floats(L, M, N, P) > (4 << 20)
    Y, start = _inputs(13, 8, 8, 8, 4, 1)  # contents are never touched: the call must fail before any launch
    rc = exat.lib().exat_cpals_noalloc(Y.data_ptr(), L, M, N, P, R, 1, start[0].data_ptr(), start[1].data_ptr(),
                                       start[2].data_ptr(), None)
    assert rc == exat.ERR_SHAPE
