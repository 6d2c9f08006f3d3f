"""GPU parity along the paper's second evaluation axis (Sec. VI-D1: hypervector dimension from
1024 to 32768) and at the small-feature end of Table II (PAMAP shape: 31 features, 5 classes,
about 80k samples).  Every stage bit-exact against the oracle fed with the oracle's own stage
before; at the PAMAP shape's full size the oracle checks sampled rows."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload  # noqa: E402

from test_gpu_parity import dev_u32, gpu_classical, gpu_encode, host_u32, make_ctx, orc_encode  # noqa: E402


def classical_pipeline(wl, ntr, nte):
    xt, yt = wl.train(ntr)
    xs, ys = wl.test(nte)
    ctx = make_ctx(wl)
    ht, hs = gpu_encode(ctx, xt), gpu_encode(ctx, xs)
    o_ht, o_hs = orc_encode(wl, xt), orc_encode(wl, xs)
    assert np.array_equal(host_u32(ht), o_ht) and np.array_equal(host_u32(hs), o_hs)
    acc, cn = gpu_classical(ctx, ht, yt)
    o_acc, o_cn = oracle.train_classical(o_ht, yt, wl.D, wl.C)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(cn.cpu().numpy(), o_cn)
    m = torch.empty((wl.C, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_binarize_classical(acc, cn, m)
    torch.cuda.synchronize()
    o_m = oracle.binarize_classical(o_acc, o_cn, wl.tie)
    assert np.array_equal(host_u32(m), o_m)
    dist = torch.empty((nte, wl.C), dtype=torch.int32, device="cuda")
    pred = torch.empty(nte, dtype=torch.int32, device="cuda")
    ctx.hdc_search(hs, m, pred, dist)
    torch.cuda.synchronize()
    o_dist, o_pred = oracle.search(o_hs, o_m, wl.D)
    assert np.array_equal(host_u32(dist), o_dist) and np.array_equal(pred.cpu().numpy(), o_pred)
    ctx.close()
    return float((o_pred == ys).mean())


@pytest.mark.parametrize("D", [1024, 2048, 4096, 8192, 16384, 32768])
def test_dimension_sweep_isolet_shape(D):
    wl = make_workload(2, D=D)
    ntr = int(np.clip(600 * 10000 // D, 250, 1500))
    assert classical_pipeline(wl, ntr, ntr // 3) > 0.5


@pytest.mark.parametrize("D", [1024, 10000, 32768])
def test_dimension_sweep_online(D):
    wl = make_workload(4, D=D)
    n = int(np.clip(300 * 10000 // D, 100, 600))
    xt, yt = wl.train(n)
    ctx = make_ctx(wl)
    ht = gpu_encode(ctx, xt)
    o_ht = orc_encode(wl, xt)
    assert np.array_equal(host_u32(ht), o_ht)
    yd = torch.from_numpy(yt).cuda()
    for batch in (None, 32):
        acc = torch.zeros((wl.C, wl.D), dtype=torch.float32, device="cuda")
        if batch is None:
            ctx.hdc_train_online(ht, yd, acc, epochs=2, lr=wl.lr)
            want = oracle.train_online(o_ht, yt, wl.D, wl.C, epochs=2, lr=wl.lr)
        else:
            ctx.hdc_train_online_batched(ht, yd, acc, batch, epochs=2, lr=wl.lr)
            want = oracle.train_online_batched(o_ht, yt, wl.D, wl.C, batch, epochs=2, lr=wl.lr)
        torch.cuda.synchronize()
        got = acc.cpu().numpy()
        scale = np.maximum(np.abs(want), 1e-3 * np.abs(want).max())
        assert float(np.max(np.abs(got - want) / scale)) < 1e-4
    ctx.close()


def test_pamap_shape_pipeline():
    wl = make_workload(6)
    assert (wl.F, wl.C) == (31, 5)
    assert classical_pipeline(wl, 12000, 4000) > 0.5


def test_pamap_shape_full_size_sampled():
    """All 64000 + 16000 samples through encode, training and search; the oracle encodes a
    prefix and a random scatter of rows and trains on the prefix."""
    wl = make_workload(6)
    xt, yt = wl.train()
    xs, _ = wl.test()
    ctx = make_ctx(wl)
    ht, hs = gpu_encode(ctx, xt), gpu_encode(ctx, xs)
    rng = np.random.default_rng(6)
    for x, h in ((xt, ht), (xs, hs)):
        rows = np.unique(np.concatenate([np.arange(2000), rng.choice(x.shape[0], 2000)]))
        assert np.array_equal(host_u32(h[torch.from_numpy(rows).cuda()]), orc_encode(wl, x[rows]))
    acc, cn = gpu_classical(ctx, ht, yt)
    assert np.array_equal(cn.cpu().numpy(), np.bincount(yt, minlength=wl.C))
    # two halves accumulate to the same integers as one call
    half = wl.n_train // 2
    acc2, cn2 = gpu_classical(ctx, ht[:half].contiguous(), yt[:half])
    acc2, cn2 = gpu_classical(ctx, ht[half:].contiguous(), yt[half:], acc2, cn2)
    assert torch.equal(acc2, acc) and torch.equal(cn2, cn)
    # prefix model from the oracle; search of every test row against it, sampled rows checked
    nsub = 4000
    o_ht = orc_encode(wl, xt[:nsub])
    o_acc, o_cn = oracle.train_classical(o_ht, yt[:nsub], wl.D, wl.C)
    a_s, n_s = gpu_classical(ctx, ht[:nsub].contiguous(), yt[:nsub])
    assert np.array_equal(a_s.cpu().numpy(), o_acc) and np.array_equal(n_s.cpu().numpy(), o_cn)
    o_m = oracle.binarize_classical(o_acc, o_cn, wl.tie)
    dist = torch.empty((wl.n_test, wl.C), dtype=torch.int32, device="cuda")
    pred = torch.empty(wl.n_test, dtype=torch.int32, device="cuda")
    ctx.hdc_search(hs, dev_u32(o_m), pred, dist)
    torch.cuda.synchronize()
    rows = np.unique(rng.choice(wl.n_test, 3000))
    o_d, o_p = oracle.search(orc_encode(wl, xs[rows]), o_m, wl.D)
    idx = torch.from_numpy(rows).cuda()
    assert np.array_equal(host_u32(dist[idx]), o_d) and np.array_equal(pred[idx].cpu().numpy(), o_p)
    ctx.close()
