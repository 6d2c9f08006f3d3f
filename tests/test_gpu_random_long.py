"""GPU parity on randomly drawn LONG calls: the kernels that only long streams take (the
contraction encoder for jobs of 128 samples, the accumulating pass that orders a block's rows
by label itself, the long-stream search kernels) against the CPU oracle for seeded (D, F, L, C, N)
draws: sampled rows of the encoding (first, last and random ones), the whole class sums and
class vectors, and distances and predictions of sampled rows."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload  # noqa: E402


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("seed", range(10))
def test_random_long_calls_match_oracle(seed):
    from paper_2206_04746_amd import binding
    rng = np.random.default_rng(5000 + seed)
    D = int(rng.choice([96, 1000, 4097, 8192, 10000, 10016]))
    F = int(rng.choice([4, 15, 33, 100, 342, 617]))
    L = int(rng.choice([2, 16, 64, 100, 256]))
    C = int(rng.choice([1, 2, 3, 4, 5, 12]))
    N = int(rng.choice([32768, 33001, 40000, 70001, 131072 + 5]))
    what = f"D={D} F={F} L={L} C={C} N={N}"
    wl = make_workload(2, seed=seed, D=D, F=F, L=L, C=C, n_train=4096)
    x0, _ = wl.train(4096)
    x = np.ascontiguousarray(np.tile(x0, ((N + 4095) // 4096, 1))[:N])
    x[rng.integers(0, N, 50), rng.integers(0, F, 50)] = np.nan     # NaN and out-of-range values: the end bins
    x[rng.integers(0, N, 50), rng.integers(0, F, 50)] = 1e30
    y = rng.integers(0, C, N).astype(np.int32)
    if C > 1:
        y[rng.random(N) < 0.9] = 0                                   # an uneven split: class 0 takes most rows
    y[rng.integers(0, N, 200)] = C + 1                               # labels outside [0, C) are skipped
    y[rng.integers(0, N, 200)] = -3
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    hv = torch.full((N, ctx.W), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_encode(xd, hv)
    got = _u32(hv)
    rows = np.unique(np.concatenate([np.arange(0, 200), np.arange(N - 200, N), rng.integers(0, N, 800)]))
    want_rows = oracle.encode(x[rows], wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)
    assert np.array_equal(got[rows], want_rows), what

    # training and inference on the GPU's own rows (checked above on a sample): everything exact
    acc = torch.zeros((C, D), dtype=torch.int32, device="cuda")
    cn = torch.zeros(C, dtype=torch.int64, device="cuda")
    cls = torch.empty((C, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_train_classical(hv, yd, acc, cn)
    ctx.hdc_binarize_classical(acc, cn, cls)
    o_acc, o_cn = oracle.train_classical(got, y, D, C)
    o_cls = oracle.binarize_classical(o_acc, o_cn, wl.tie)
    assert np.array_equal(acc.cpu().numpy(), o_acc), what
    assert np.array_equal(cn.cpu().numpy(), o_cn), what
    assert np.array_equal(_u32(cls), o_cls), what
    vs = torch.empty(D, dtype=torch.int32, device="cuda")
    hs = torch.empty(N, dtype=torch.int32, device="cuda")
    ctx.hdc_vsum(hv, vs)
    ctx.hdc_hsum(hv, hs)
    assert np.array_equal(vs.cpu().numpy(), oracle.vsum(got, D)), what
    assert np.array_equal(hs.cpu().numpy(), oracle.hsum(got, D)), what

    dist = torch.empty((N, C), dtype=torch.int32, device="cuda")
    pred = torch.empty(N, dtype=torch.int32, device="cuda")
    pred2 = torch.empty(N, dtype=torch.int32, device="cuda")
    ctx.hdc_search(hv, cls, pred, dist)
    ctx.hdc_search(hv, cls, pred2, None)
    o_d, o_p = oracle.search(got[rows], o_cls, D)
    assert np.array_equal(_u32(dist)[rows], o_d), what
    assert np.array_equal(pred.cpu().numpy()[rows], o_p), what
    assert torch.equal(pred, pred2), what
    ctx.close()
