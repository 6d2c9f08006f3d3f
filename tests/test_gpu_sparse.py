"""GPU parity of hdc_encode_sparse (Sec. III Eq. 1, bundled as a constant plus corrections for
the features that leave bin 0): bit-exact against the CPU oracle's encode on inputs from
all-background to fully dense, through compact and full tables, fp32 and u8 features."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload, pack_bits_lsb  # noqa: E402


def _ctx(wl):
    from paper_2206_04746_amd import binding
    return binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)


def _sparse(ctx, x):
    xd = torch.from_numpy(x).cuda()
    hv = torch.full((x.shape[0], ctx.W), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_encode_sparse(xd, hv)
    torch.cuda.synchronize()
    return hv.cpu().numpy().view(np.uint32)


def _oracle(wl, x):
    return oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)


# config 3 is the digit-image shape (u8, L = 256, about 80 % background, compact tables);
# 14001 samples give every wave several samples and a ragged last round
@pytest.mark.parametrize("n", [1, 700, 14001])
def test_sparse_encode_image_shape_bit_exact(n):
    wl = make_workload(3)
    x, _ = wl.train(n)
    ctx = _ctx(wl)
    assert ctx.hdc_encoded_words() < ctx.W          # the compact tables are in use
    assert np.array_equal(_sparse(ctx, x), _oracle(wl, x))
    ctx.close()


def _thin_out(rng, x, keep, background):
    """Sends all but a `keep` fraction of the entries of x to the background value."""
    x = x.copy()
    x[rng.random(x.shape) >= keep] = background
    return x


# fp32 features, lo = -1: the value -1 lies in bin 0.  From every feature listed to none.
@pytest.mark.parametrize("keep", [1.0, 0.6, 0.2, 0.03, 0.0])
def test_sparse_encode_fp32_all_densities(keep):
    wl = make_workload(2, n_train=300)
    x, _ = wl.train(300)
    x = _thin_out(np.random.default_rng(int(keep * 100)), x, keep, -1.0)
    x[7] = -1.0                       # one sample with nothing listed at all
    x[8, 5] = np.nan                  # NaN goes to bin 0 as well
    ctx = _ctx(wl)
    assert np.array_equal(_sparse(ctx, x), _oracle(wl, x))
    ctx.close()


@pytest.mark.parametrize("D,F,L,N", [
    (1, 1, 1, 3), (31, 2, 2, 5), (33, 31, 16, 17), (64, 32, 16, 15), (1000, 33, 7, 63),
    (2048, 64, 256, 65), (4097, 63, 3, 33), (10000, 128, 100, 21), (12345, 1000, 5, 9), (10000, 2100, 9, 6),
])
def test_sparse_encode_ragged_shapes(D, F, L, N):
    wl = make_workload(2, seed=D + F, D=D, F=F, L=L, n_train=N)
    x, _ = wl.train(N)
    x = _thin_out(np.random.default_rng(D), x, 0.3, -1.0)
    ctx = _ctx(wl)
    got = _sparse(ctx, x)
    assert np.array_equal(got, _oracle(wl, x))
    last_bits = D - 32 * (ctx.W - 1)
    if last_bits < 32:
        assert np.all(got[:, -1] >> last_bits == 0)
    ctx.close()


def test_sparse_encode_unrelated_level_vectors_full_tables():
    # random level vectors: every dimension varies, so the full (not the compact) tables are
    # the ones the corrections are derived from
    rng = np.random.default_rng(11)
    for L in (256, 100, 2):
        wl = make_workload(3, F=36, L=L, D=777, n_train=80)
        wl.level = pack_bits_lsb(rng.integers(0, 2, size=(L, wl.D), dtype=np.uint8))
        x = rng.integers(0, 256, size=(80, wl.F), dtype=np.uint8)
        x[rng.random(x.shape) < 0.7] = 0
        ctx = _ctx(wl)
        if L > 2:    # (two random vectors agree in half of the dimensions: compact tables again)
            assert ctx.hdc_encoded_words() == ctx.W
        assert np.array_equal(_sparse(ctx, x), _oracle(wl, x))
        ctx.close()


def test_sparse_encode_equal_level_vectors():
    # all level vectors equal: nothing varies, every sample encodes to the same constant
    wl = make_workload(3, F=25, L=8, D=500, n_train=10)
    wl.level = np.repeat(wl.level[:1], 8, axis=0)
    x, _ = wl.train(10)
    ctx = _ctx(wl)
    assert np.array_equal(_sparse(ctx, x), _oracle(wl, x))
    ctx.close()


def test_sparse_encode_chunked_stream_and_agreement_with_dense():
    # more samples than one quantiser chunk (65536): sampled rows against the oracle, every row
    # against hdc_encode, and a second call on the same context (tables already derived)
    wl = make_workload(3, n_train=70000)
    x, _ = wl.train(70000)
    ctx = _ctx(wl)
    got = _sparse(ctx, x)
    rows = np.concatenate([np.arange(0, 70000, 997), [65535, 65536, 69999]])
    assert np.array_equal(got[rows], _oracle(wl, x[rows]))
    xd = torch.from_numpy(x).cuda()
    dense = torch.empty((70000, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_encode(xd, dense)
    torch.cuda.synchronize()
    assert np.array_equal(got, dense.cpu().numpy().view(np.uint32))
    assert np.array_equal(_sparse(ctx, x[:100]), got[:100])
    ctx.close()


def test_sparse_encode_argument_errors():
    from paper_2206_04746_amd import binding
    wl = make_workload(1, n_train=8)
    ctx = _ctx(wl)
    x = torch.zeros((0, wl.F), dtype=torch.float32, device="cuda")
    hv = torch.empty((0, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_encode_sparse(x, hv)                                  # N = 0: a no-op
    hv4 = torch.empty((4, ctx.W), dtype=torch.int32, device="cuda")
    assert binding.lib.hdc_encode_sparse(None, None, 4, None, None) == binding.HDC_EINVAL
    assert binding.lib.hdc_encode_sparse(ctx._h, None, 4, hv4.data_ptr(), None) == binding.HDC_EINVAL
    assert binding.lib.hdc_encode_sparse(ctx._h, None, -1, None, None) == binding.HDC_EINVAL
    ctx.close()
