"""The entry point that allocates nothing, hdc_vsum_static (vertical summation, Sec. IV-B2, with
its kernels' scratch in a static device array): called through the C ABI, compared element by
element with hdc_vsum (and the CPU oracle) on calls in a row that share the array, a smaller one
after a larger one; sizes beyond its limit are refused.  Collected last on purpose."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload  # noqa: E402


def _rows(n, D, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    W = (D + 31) // 32
    hv = torch.randint(-2 ** 31, 2 ** 31 - 1, (n, W), dtype=torch.int32, device="cuda", generator=g)
    if D % 32:
        hv[:, -1] &= (1 << (D % 32)) - 1
    return hv


def _static(lib, D, hv, out):
    rc = lib.hdc_vsum_static(ctypes.c_int32(D), ctypes.c_void_p(hv.data_ptr() if hv.numel() else 0),
                             ctypes.c_int64(hv.shape[0]), ctypes.c_void_p(out.data_ptr()),
                             ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


@pytest.mark.parametrize("D", [10000, 1000, 16384, 33])
def test_vsum_static_matches_vsum_on_calls_in_a_row(D):
    from paper_2206_04746_amd import binding
    wl = make_workload(1, D=D, F=8, L=4)
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    big = _rows(300000 if D <= 10000 else 270000, D, 1)      # more than one round of 262144 rows, ragged
    small = _rows(4099, D, 2)
    for hv in (big, small, big[:70001], small[:1]):          # the second call smaller than the first, and so on
        want = torch.full((D,), -7, dtype=torch.int32, device="cuda")
        got = torch.full((D,), -9, dtype=torch.int32, device="cuda")
        ctx.hdc_vsum(hv, want)
        assert _static(binding.lib, D, hv, got) == binding.HDC_OK
        torch.cuda.synchronize()
        assert torch.equal(got, want)
    # against the oracle on a size it finishes quickly
    got = torch.empty(D, dtype=torch.int32, device="cuda")
    assert _static(binding.lib, D, small, got) == binding.HDC_OK
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.vsum(small.cpu().numpy().view(np.uint32), D))
    # no rows: zeros
    assert _static(binding.lib, D, small[:0], got) == binding.HDC_OK
    torch.cuda.synchronize()
    assert int(got.abs().sum()) == 0
    ctx.close()


def test_vsum_static_refuses_what_is_beyond_its_limits():
    from paper_2206_04746_amd import binding
    hv = _rows(4, 16416, 3)
    out = torch.zeros(16416, dtype=torch.int32, device="cuda")
    assert _static(binding.lib, 16416, hv, out) == binding.HDC_ELIMIT
    assert _static(binding.lib, 0, hv, out) == binding.HDC_EINVAL
    assert binding.lib.hdc_vsum_static(ctypes.c_int32(64), None, ctypes.c_int64(4), ctypes.c_void_p(out.data_ptr()),
                                       None) == binding.HDC_EINVAL
    torch.cuda.synchronize()
    assert int(out.abs().sum()) == 0
