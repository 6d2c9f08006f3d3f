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


# The search alone over a wider range of class counts and dimensions than the workloads have: one
# pass or several over the class slots of the matrix-core kernel, several launches, rows of one
# tile per job, and the vector kernels around it.  Sampled rows against the oracle, both outputs;
# the predictions of every row against the distances the GPU wrote (lowest class of the minimum).
@pytest.mark.parametrize("seed", range(12))
def test_random_search_draws_match_oracle(seed):
    from paper_2206_04746_amd import binding
    rng = np.random.default_rng(7000 + seed)
    D = int(rng.choice([130, 1000, 4097, 10000, 10240, 10241, 13000, 16384, 20001, 27000, 32768, 33000]))
    C = int(rng.choice([8, 9, 13, 26, 31, 32, 45, 62, 63, 100, 124, 125, 200, 260]))
    N = int(rng.choice([8192, 9001, 20480, 32768 + 7, 50000]))
    if D * C * N > 3e10:
        N = 8192 + seed
    what = f"D={D} C={C} N={N}"
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    W = (D + 31) // 32
    tail = np.uint32((1 << (D - 32 * (W - 1))) - 1) if D % 32 else np.uint32(0xffffffff)
    cls = rng.integers(0, 2 ** 32, size=(C, W), dtype=np.uint64).astype(np.uint32)
    cls[:, -1] &= tail
    cls[C // 2] = cls[1]                                             # a duplicate: the lower class wins
    q = rng.integers(0, 2 ** 32, size=(N, W), dtype=np.uint64).astype(np.uint32)
    near = np.arange(0, N, 2)                                        # every other query: near some class
    q[near] = cls[rng.integers(0, C, near.size)]
    q[near, rng.integers(0, W, near.size)] ^= np.uint32(0x0ff00ff0)
    q[:, -1] &= tail
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    qd = torch.from_numpy(q.view(np.int32)).cuda()
    cd = torch.from_numpy(cls.view(np.int32)).cuda()
    dist = torch.full((N, C), -1, dtype=torch.int32, device="cuda")
    pred = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    pred2 = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    ctx.hdc_search(qd, cd, pred, dist)
    ctx.hdc_search(qd, cd, pred2, None)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, 100), np.arange(N - 100, N), rng.integers(0, N, 600)]))
    o_d, o_p = oracle.search(q[rows], cls, D)
    assert np.array_equal(_u32(dist)[rows], o_d), what
    assert np.array_equal(pred.cpu().numpy()[rows], o_p), what
    assert torch.equal(pred, pred2), what
    first_min = (dist == dist.min(dim=1, keepdim=True).values).int().argmax(dim=1)
    assert torch.equal(pred.long(), first_min), what
    ctx.close()


# Very long hypervectors (D above 32768, where the rows no longer fit a wave's registers and the
# wide-row forms of every kernel run) on calls long enough for the streaming kernels: encoding,
# classical training, the sums and the search against the oracle, everything compared in full.
@pytest.mark.parametrize("seed", range(8))
def test_random_very_wide_rows_match_oracle(seed):
    from paper_2206_04746_amd import binding
    rng = np.random.default_rng(8000 + seed)
    D = int(rng.choice([32800, 40000, 50001, 65536, 65600, 100000, 131072 + 5, 200000]))
    F = int(rng.choice([4, 9, 20, 33]))
    L = int(rng.choice([2, 8, 64]))
    C = int(rng.choice([1, 2, 3, 5, 12, 26]))
    N = int(rng.choice([300, 5000, 8193, 9000, 20000]))
    while D * F * N > 1.2e10:
        N = N * 2 // 3
    what = f"D={D} F={F} L={L} C={C} N={N}"
    wl = make_workload(2, seed=seed, D=D, F=F, L=L, C=C, n_train=min(N, 4096))
    x0, _ = wl.train(min(N, 4096))
    x = np.ascontiguousarray(np.tile(x0, ((N + x0.shape[0] - 1) // x0.shape[0], 1))[:N])
    y = rng.integers(0, C, N).astype(np.int32)
    y[rng.integers(0, N, 20)] = C + 2
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    hv = torch.full((N, ctx.W), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_encode(xd, hv)
    got = _u32(hv)
    assert np.array_equal(got, oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)), what
    hv_s = torch.full_like(hv, -1)
    ctx.hdc_encode_sparse(xd, hv_s)
    assert torch.equal(hv_s, hv), what
    n_bits = min(N, 257)                                             # the byte form of a few hundred rows
    bits = torch.empty((n_bits, D), dtype=torch.uint8, device="cuda")
    back = torch.full((n_bits, ctx.W), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_unpack(hv[:n_bits], bits)
    ctx.hdc_pack(bits, back)
    assert np.array_equal(bits.cpu().numpy(), oracle.unpack(got[:n_bits], D)), what
    assert torch.equal(back, hv[:n_bits]), what
    del bits, back, hv_s
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
    ctx.hdc_search(hv, cls, pred, dist)
    o_d, o_p = oracle.search(got, o_cls, D)
    assert np.array_equal(_u32(dist), o_d), what
    assert np.array_equal(pred.cpu().numpy(), o_p), what
    ctx.close()
