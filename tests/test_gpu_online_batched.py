"""GPU parity of hdc_train_online_batched (Sec. VI-D2) against the CPU oracle, through the C ABI.
fp32 accumulators within 1e-5 relative (fp64 sums on both sides, different summation order);
class vectors and predictions derived from them bit-exact wherever the accumulators are not
within rounding of zero."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload, pack_bits_lsb  # noqa: E402

from test_gpu_parity import dev_u32, gpu_encode, host_u32, make_ctx, orc_encode, rel_err  # noqa: E402

TOL = 1e-5


def clustered(rng, N, D, C, flip=0.35):
    protos = rng.integers(0, 2, size=(C, D), dtype=np.uint8)
    y = rng.integers(0, C, N).astype(np.int32)
    bits = protos[y] ^ (rng.random((N, D)) < flip).astype(np.uint8)
    return pack_bits_lsb(bits), y


# batch sizes: inside one forward tile, several tiles, ragged last batch, >= N, 1, and (9000) more
# than one forward sub-batch; C = 300 takes two class windows in the backward step; D = 40000 is
# beyond what the sequential trainer accepts
@pytest.mark.parametrize("D,C,N,epochs,lr,batch", [
    (1024, 5, 600, 2, 1.0, 32), (10000, 6, 1500, 3, 1.0, 256), (10000, 26, 300, 1, 0.5, 300),
    (10000, 26, 300, 1, 0.5, 100000), (33, 1, 20, 2, 1.0, 3), (2049, 3, 100, 1, 0.0, 7),
    (32768, 2, 40, 1, 1.0, 16), (1024, 4, 100, 1, 1.0, 1), (1000, 3, 9000, 1, 1.0, 9000),
    (4096, 300, 700, 1, 1.0, 128), (40000, 2, 30, 1, 1.0, 8),
    # from 1024 samples per piece on the backward step goes by class lists
    (10000, 26, 3000, 2, 1.0, 1024), (10000, 26, 2100, 1, 0.5, 4096), (2049, 17, 1500, 3, 1.0, 1500),
    (100, 1, 1100, 2, 1.0, 1100), (4097, 40, 9000, 1, 1.0, 5000), (10000, 6, 20000, 1, 1.0, 20000)])
def test_batched_online_training_matches_oracle(D, C, N, epochs, lr, batch):
    rng = np.random.default_rng(D + C + N + batch)
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    hv, y = clustered(rng, N, D, C)
    y[N // 2] = C                                            # one out-of-range label: skipped
    ctx = make_ctx(wl)
    acc = torch.zeros((C, D), dtype=torch.float32, device="cuda")
    hvd, yd = dev_u32(hv), torch.from_numpy(y).cuda()
    ctx.hdc_train_online_batched(hvd, yd, acc, batch, epochs=epochs, lr=lr)
    torch.cuda.synchronize()
    want = oracle.train_online_batched(hv, y, D, C, batch, epochs=epochs, lr=lr)
    assert rel_err(acc.cpu().numpy(), want) < TOL
    if epochs == 1:     # continuing from a non-zero model: a second call equals one more epoch
        ctx.hdc_train_online_batched(hvd, yd, acc, batch, epochs=1, lr=lr)
        torch.cuda.synchronize()
        want2 = oracle.train_online_batched(hv, y, D, C, batch, epochs=2, lr=lr)
        assert rel_err(acc.cpu().numpy(), want2) < TOL
    ctx.close()


def test_batched_whole_set_from_zero_model_is_exact():
    # one batch from a zero model: all cosines 0, all weights 1 (lr for the subtraction from class
    # 0): small integers and halves, so the result is exact whatever the summation order
    rng = np.random.default_rng(5)
    D, C, N = 10000, 6, 3000
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    hv, y = clustered(rng, N, D, C)
    ctx = make_ctx(wl)
    acc = torch.zeros((C, D), dtype=torch.float32, device="cuda")
    ctx.hdc_train_online_batched(dev_u32(hv), torch.from_numpy(y).cuda(), acc, N, epochs=1, lr=0.5)
    torch.cuda.synchronize()
    want = oracle.train_online_batched(hv, y, D, C, N, epochs=1, lr=0.5)
    assert np.array_equal(acc.cpu().numpy(), want)
    ctx.close()


def test_batched_argument_errors():
    from paper_2206_04746_amd import binding as b
    wl = make_workload(1, D=64, F=4, L=4, C=2)
    ctx = make_ctx(wl)
    hv = torch.zeros((4, ctx.W), dtype=torch.int32, device="cuda")
    acc = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
    f = b.lib.hdc_train_online_batched
    assert f(ctx._h, hv.data_ptr(), hv.data_ptr(), 4, 1, 1.0, 0, acc.data_ptr(), None) == b.HDC_EINVAL
    assert f(ctx._h, hv.data_ptr(), hv.data_ptr(), 4, -1, 1.0, 2, acc.data_ptr(), None) == b.HDC_EINVAL
    assert f(ctx._h, None, hv.data_ptr(), 4, 1, 1.0, 2, acc.data_ptr(), None) == b.HDC_EINVAL
    assert f(ctx._h, None, None, 0, 1, 1.0, 2, None, None) == b.HDC_OK          # N == 0 is a no-op
    ctx.close()


@pytest.mark.parametrize("batch", [64, 8192])
def test_config4_full_size_batched_online_pipeline(batch):
    # UCIHAR-shaped configuration at full size: encode -> batched online training (3 epochs) ->
    # class vectors -> search, every stage against the oracle fed with the oracle's own stage before
    wl = make_workload(4)
    xt, yt = wl.train(wl.n_train)
    xs, ys = wl.test(wl.n_test)
    ctx = make_ctx(wl)
    ht, hs = gpu_encode(ctx, xt), gpu_encode(ctx, xs)
    o_ht, o_hs = orc_encode(wl, xt), orc_encode(wl, xs)
    assert np.array_equal(host_u32(ht), o_ht) and np.array_equal(host_u32(hs), o_hs)
    acc = torch.zeros((wl.C, wl.D), dtype=torch.float32, device="cuda")
    ctx.hdc_train_online_batched(ht, torch.from_numpy(yt).cuda(), acc, batch, epochs=wl.epochs, lr=wl.lr)
    m = torch.empty((wl.C, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_binarize_online(acc, m)
    torch.cuda.synchronize()
    o_acc = oracle.train_online_batched(o_ht, yt, wl.D, wl.C, batch, epochs=wl.epochs, lr=wl.lr)
    got = acc.cpu().numpy()
    assert rel_err(got, o_acc) < TOL
    o_m = oracle.binarize_online(o_acc, wl.tie)
    # class bits can only differ where the accumulator is within rounding of zero
    diff = np.unpackbits((host_u32(m) ^ o_m).view(np.uint8), bitorder="little").reshape(wl.C, -1)[:, :wl.D]
    assert np.all(np.abs(o_acc[diff == 1]) < TOL * np.abs(o_acc).max())
    # inference from the oracle's class vectors: bit-exact
    md = dev_u32(o_m)
    pred = torch.empty(wl.n_test, dtype=torch.int32, device="cuda")
    ctx.hdc_search(hs, md, pred, None)
    torch.cuda.synchronize()
    o_pred = oracle.search(o_hs, o_m, wl.D)[1]
    assert np.array_equal(pred.cpu().numpy(), o_pred)
    assert (o_pred == ys).mean() > 0.5
    ctx.close()
