"""GPU parity of hdc_encode where it runs as a contraction over the features on the matrix cores
(Sec. III Eq. 1; level tables whose dimensions flip at most once along the levels, L <= 256,
F <= 896, 1024 samples or more, 256 for large models): bit-exact against the CPU oracle, over feature counts on both
sides of a multiple of 64, even and odd (the tie vote), u8 and fp32 features, sample counts that
leave a ragged last block (and few enough that the words of a row are split over blocks), and
rows whose last word is partial; and the tables that are not of
that shape, which must take the other kernel and give the same bits."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload  # noqa: E402


def _ctx(wl):
    from paper_2206_04746_amd import binding
    return binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)


def _encode(ctx, x):
    xd = torch.from_numpy(x).cuda()
    hv = torch.full((x.shape[0], ctx.W), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_encode(xd, hv)
    torch.cuda.synchronize()
    return hv.cpu().numpy().view(np.uint32)


def _oracle(wl, x):
    return oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)


@pytest.mark.parametrize("cfg,D,F,L,N", [
    (2, 10000, 617, 64, 2049), (2, 10000, 617, 64, 6238), (2, 1000, 64, 16, 2080), (2, 4099, 640, 64, 2048),
    (2, 777, 33, 7, 2500), (2, 5000, 200, 32, 2111), (2, 10000, 342, 64, 4097), (2, 2048, 65, 2, 2050),
    (2, 16384, 128, 64, 2048), (2, 96, 10, 3, 3000), (2, 10000, 31, 64, 2300),
    (4, 10000, 561, 100, 2200), (2, 8000, 300, 256, 2100), (2, 6000, 90, 65, 2049), (2, 3000, 50, 129, 2048),
    (3, 2048, 400, 32, 2100), (3, 10000, 625, 64, 2065), (3, 3000, 36, 5, 2048), (2, 10000, 617, 64, 1024), (2, 1024, 100, 16, 1055),
    # few samples: a row's words are split over two or four blocks per 32 samples
    (2, 10000, 617, 64, 1559), (2, 10000, 617, 64, 4000), (2, 200, 50, 8, 1100), (2, 128, 20, 4, 1030), (3, 10000, 625, 64, 3333),
    (2, 10000, 617, 64, 4096), (2, 9999, 100, 200, 1500),
    # large models take the contraction from 256 samples on
    (2, 10000, 617, 64, 256), (2, 10000, 617, 64, 300), (4, 10000, 561, 100, 700), (3, 10000, 625, 64, 513),
    # rows of more than 512 words are always split (a thread per word of a range)
    (2, 32768, 617, 64, 2100), (2, 20000, 200, 32, 5000), (2, 65536, 64, 16, 1100), (2, 40001, 100, 64, 9000),
    # 641 to 896 features: 12 or 14 MFMA steps, the bit planes shared through LDS
    (3, 10000, 784, 256, 2100), (3, 10000, 784, 256, 9000), (2, 10000, 700, 64, 2222), (2, 5000, 896, 64, 1300),
    (2, 10000, 769, 100, 600), (3, 3000, 841, 32, 4100), (2, 20000, 650, 16, 2050),
])
def test_encode_contraction_bit_exact(cfg, D, F, L, N):
    wl = make_workload(cfg, seed=D + F + L, D=D, F=F, L=L, n_train=N)
    x, _ = wl.train(N)
    if wl.dtype == "f32":
        x[5, :] = np.nan                       # NaN and values outside the range go to the end bins
        x[6, ::2] = -1e30
        x[7, 1::2] = 1e30
    ctx = _ctx(wl)
    got = _encode(ctx, x)
    want = _oracle(wl, x)
    assert np.array_equal(got, want)
    last_bits = D - 32 * (ctx.W - 1)
    if last_bits < 32:
        assert np.all(got[:, -1] >> last_bits == 0)
    t, n = ctx.hdc_profile_read("encode_contract")
    ctx.hdc_profile_enable(True)
    _encode(ctx, x[:2048] if N >= 1024 else x)
    t, n = ctx.hdc_profile_read("encode_contract")
    assert n == 1, "the call was expected to take the contraction kernel"
    ctx.close()


def test_encode_tables_that_flip_twice_take_the_other_kernel():
    wl = make_workload(2, D=2000, F=100, L=16, n_train=2100)
    lv = wl.level.copy()
    # dimension 3 differs from level 0 at level 5 only: it flips and flips back
    lv[:, 0] &= ~np.uint32(8)
    lv[:, 0] |= lv[0, 0] & np.uint32(8)
    lv[5, 0] ^= np.uint32(8)
    wl.level = lv
    x, _ = wl.train(2100)
    ctx = _ctx(wl)
    ctx.hdc_profile_enable(True)
    got = _encode(ctx, x)
    _, n = ctx.hdc_profile_read("encode_contract")
    assert n == 0
    assert np.array_equal(got, _oracle(wl, x))
    ctx.close()


def test_encode_tables_whose_every_dimension_flips_once_take_the_contraction():
    """Level vectors that run from a vector to its complement (the other usual construction of
    Sec. III): no dimension is level-invariant, every one flips exactly once."""
    wl = make_workload(2, D=2048, F=100, L=17, n_train=3000)
    rng = np.random.default_rng(5)
    order = rng.permutation(2048)
    bits = np.zeros((17, 2048), dtype=np.uint8)
    bits[0] = rng.integers(0, 2, 2048)
    for l in range(1, 17):
        bits[l] = bits[l - 1]
        bits[l, order[(l - 1) * 128:l * 128]] ^= 1
    assert np.array_equal(bits[16], 1 - bits[0])
    wl.level = np.packbits(bits, axis=1, bitorder="little").view(np.uint32).reshape(17, 64).copy()
    x, _ = wl.train(3000)
    ctx = _ctx(wl)
    ctx.hdc_profile_enable(True)
    got = _encode(ctx, x)
    assert ctx.hdc_profile_read("encode_contract")[1] == 1
    assert np.array_equal(got, _oracle(wl, x))
    ctx.close()


def test_encode_contraction_many_samples_and_agreement_with_small_calls():
    # more samples than blocks in flight (several jobs per block); the same rows encoded in calls too
    # small for the contraction must give the same bits
    wl = make_workload(2, n_train=40000)
    x, _ = wl.train(40000)
    ctx = _ctx(wl)
    got = _encode(ctx, x)
    rows = np.concatenate([np.arange(0, 40000, 613), [31, 32, 39967, 39968, 39999]])
    assert np.array_equal(got[rows], _oracle(wl, x[rows]))
    ctx.hdc_profile_enable(True)
    small = _encode(ctx, x[:200])
    assert ctx.hdc_profile_read("encode_contract")[1] == 0, "200 samples were expected to take the vector kernel"
    assert np.array_equal(small, got[:200])
    ctx.close()
