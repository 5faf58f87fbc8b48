"""The measurement aid of the plan: HIP events around the two kernels of every compress call, kept for the last
128 calls, so that a benchmark can enqueue its passes back to back and read the kernel times afterwards."""
import pytest
import torch

from paper_2311_13693_amd import exat

pytestmark = pytest.mark.gpu


def test_timing_ring():
    I, J, K, L, M, N, P = 64, 48, 40, 8, 8, 8, 4
    gen = torch.Generator(device="cpu").manual_seed(3)
    plan = exat.Plan(exat.make_desc(I, J, K, L, M, N, P, I, J, K, exat.EXAT_F32))
    plan.set_factors(*(torch.randn(P * d, n, generator=gen).cuda() for d, n in ((L, I), (M, J), (N, K))))
    X = torch.randn(I * J * K, generator=gen).cuda()
    Y = plan.new_y()
    with pytest.raises(exat.ExatError):      # timing is off
        plan.last_timing()
    plan.set_timing(True)
    with pytest.raises(exat.ExatError):      # no call yet
        plan.last_timing()
    for _ in range(3):
        plan.compress(X, Y)
    for age in range(3):
        a, b = plan.timing_of(age)
        assert 0.0 < a < 50.0 and 0.0 < b < 50.0
    assert plan.last_timing() == plan.timing_of(0)
    with pytest.raises(exat.ExatError):      # only three calls so far
        plan.timing_of(3)
    for _ in range(200):                     # the ring wraps
        plan.compress(X, Y)
    torch.cuda.synchronize()
    assert all(0.0 < plan.timing_of(age)[0] < 50.0 for age in (0, 64, 127))
    with pytest.raises(exat.ExatError):
        plan.timing_of(128)
    plan.set_timing(False)
    plan.compress(X, Y)
    with pytest.raises(exat.ExatError):
        plan.last_timing()
    plan.close()


def test_mfma_probe_reports_a_rate_below_the_published_peak():
    """exat_probe_mfma (measurement aid): a short launch of each kind gives a positive rate that does not exceed the
    published MFMA peak, and a plausible core clock; bad arguments are refused."""
    import ctypes
    for kind, peak in ((0, 2500.0), (1, 157.3)):
        for rnd in (False, True):
            tf, ghz = exat.probe_mfma(kind, rnd, 2000, 256)
            print("  kind %d random %d: %.1f TFLOP/s at %.2f GHz" % (kind, rnd, tf, ghz), flush=True)
            assert 0.05 * peak < tf <= 1.02 * peak
            assert 0.5 < ghz < 3.0
    L = exat.lib()
    tf, ghz = ctypes.c_double(), ctypes.c_double()
    assert L.exat_probe_mfma(2, 0, 10, 256, ctypes.byref(tf), ctypes.byref(ghz)) == exat.ERR_SHAPE
    assert L.exat_probe_mfma(0, 0, 0, 256, ctypes.byref(tf), ctypes.byref(ghz)) == exat.ERR_SHAPE
    assert L.exat_probe_mfma(0, 0, 10, 256, None, ctypes.byref(ghz)) == exat.ERR_NULL
