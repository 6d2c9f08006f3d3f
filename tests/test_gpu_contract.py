"""GPU parity of hdc_encode where it runs as a contraction over the features on the matrix cores
(Sec. III Eq. 1; level tables whose dimensions flip once along the levels, or up to 8 times where
they share the levels at which they do, L <= 256,
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


def test_encode_tables_that_flip_twice_take_the_contraction_and_match():
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
    assert n == 1, "a dimension that flips twice enters two tiles with opposite signs"
    assert np.array_equal(got, _oracle(wl, x))
    ctx.close()


def _levels_from_flips(rng, D, L, flips_at):
    """Packed level table [L][W]: level 0 random, dimension d changes at the levels flips_at[d]."""
    bits = np.zeros((L, D), dtype=np.uint8)
    bits[0] = rng.integers(0, 2, D)
    change = np.zeros((L, D), dtype=np.uint8)
    for d, at in enumerate(flips_at):
        change[list(at), d] = 1
    bits = (bits[0][None, :] ^ (np.cumsum(change, axis=0) & 1)).astype(np.uint8)
    W = (D + 31) // 32
    padded = np.zeros((L, W * 32), dtype=np.uint8)
    padded[:, :D] = bits
    return np.packbits(padded.reshape(L, W, 32), axis=2, bitorder="little").view(np.uint32).reshape(L, W)


@pytest.mark.parametrize("D,F,L,N,kind,frac,most,nsets", [
    # level vectors on a circle (level l and level l + L/2 are complements in the dimensions that
    # vary, the last level is one step from the first): what flips at level l flips back at l + L/2
    (10000, 617, 64, 2100, "circle", 0, 0, 0), (10000, 342, 64, 5000, "circle", 0, 0, 0), (2049, 400, 16, 1559, "circle", 0, 0, 0),
    (10000, 617, 64, 300, "circle", 0, 0, 0), (4000, 256, 8, 1100, "circle", 0, 0, 0), (10000, 640, 128, 2048, "circle", 0, 0, 0),
    # a share `frac` of the dimensions in `nsets` sets that flip at the same 2 to `most` levels, single flips elsewhere
    (10000, 617, 64, 2111, "sets", 0.2, 8, 12), (3000, 100, 8, 4097, "sets", 0.2, 3, 3), (5000, 400, 100, 1500, "sets", 0.2, 4, 4),
    (1000, 342, 9, 2048, "sets", 0.2, 4, 2), (10000, 617, 64, 1559, "sets", 0.1, 8, 6), (2048, 896, 16, 1024, "sets", 0.3, 4, 3),
])
def test_encode_dimensions_that_flip_several_times_take_the_contraction_and_match(D, F, L, N, kind, frac, most, nsets):
    """Sec. III Eq. 1 on level tables whose dimensions change more than once along the levels:
    the sums of the single-flip form, one per level at which the dimension changes, with
    alternating sign.  Same bits as the oracle; u8 and fp32 features."""
    rng = np.random.default_rng(D + F + L)
    wl = make_workload(2, D=D, F=F, L=L, n_train=N)
    if kind == "circle":
        half = L // 2
        step = rng.integers(1, half + 1, D)                    # the level at which a dimension first flips
        vary = rng.random(D) < 0.5
        flips_at = [((int(s), int(s) + half) if v and s + half < L else ((int(s),) if v else ())) for s, v in zip(step, vary)]
    else:
        sets = [tuple(sorted(rng.choice(np.arange(1, L), size=int(rng.integers(2, min(most, L - 1) + 1)), replace=False).tolist()))
                for _ in range(nsets)]
        flips_at = []
        for d in range(D):
            r = rng.random()
            flips_at.append(sets[int(rng.integers(0, nsets))] if r < frac else ((int(rng.integers(1, L)),) if r < 0.6 else ()))
    wl.level = _levels_from_flips(rng, D, L, flips_at)
    x, _ = wl.train(N)
    x[rng.integers(0, N, 20), rng.integers(0, F, 20)] = np.nan
    ctx = _ctx(wl)
    ctx.hdc_profile_enable(True)
    got = _encode(ctx, x)
    _, n = ctx.hdc_profile_read("encode_contract")
    assert n == 1, "the call was expected to take the contraction kernel"
    assert np.array_equal(got, _oracle(wl, x))
    ctx.close()
    if int(np.sqrt(F)) ** 2 == F:                              # the same table with byte features (a square grid of them)
        wl8 = make_workload(3, D=D, F=F, L=L, n_train=N)
        wl8.item, wl8.level, wl8.tie = wl.item, wl.level, wl.tie
        x8, _ = wl8.train(N)
        ctx = _ctx(wl8)
        assert np.array_equal(_encode(ctx, x8), _oracle(wl8, x8))
        ctx.close()


def test_encode_tables_with_too_many_or_too_scattered_flips_take_the_other_kernel():
    """A dimension that changes nine times, and a table whose repeated flips share no levels (every
    level vector drawn afresh): not worth or not fit for the contraction; same bits from the vector kernel."""
    rng = np.random.default_rng(77)
    for case in ("nine", "random"):
        wl = make_workload(2, D=2000, F=100, L=16, n_train=2100)
        if case == "nine":
            flips_at = [(int(rng.integers(1, 16)),) if rng.random() < 0.5 else () for _ in range(2000)]
            flips_at[7] = tuple(range(1, 10))
            wl.level = _levels_from_flips(rng, 2000, 16, flips_at)
        else:
            wl.level = rng.integers(0, 2 ** 32, size=wl.level.shape, dtype=np.uint64).astype(np.uint32)
            wl.level[:, -1] &= np.uint32((1 << (2000 - 32 * (wl.level.shape[1] - 1))) - 1)
        x, _ = wl.train(2100)
        ctx = _ctx(wl)
        ctx.hdc_profile_enable(True)
        got = _encode(ctx, x)
        _, n = ctx.hdc_profile_read("encode_contract")
        assert n == 0, case
        assert np.array_equal(got, _oracle(wl, x)), case
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


@pytest.mark.parametrize("seed", range(10))
def test_random_multi_flip_tables_match_oracle(seed):
    """Randomly drawn level tables with dimensions that flip several times, in shared sets of levels
    of random size and number (so that some models take the chained contraction and some the vector
    kernel): the bits are the oracle's either way."""
    rng = np.random.default_rng(9000 + seed)
    D = int(rng.choice([500, 2049, 4096, 10000, 20000]))
    F = int(rng.choice([16, 100, 342, 617, 896]))
    L = int(rng.choice([3, 8, 16, 64, 100, 256]))
    N = int(rng.choice([256, 700, 1024, 1559, 2048, 3001, 4500]))
    while D * F * N > 1.5e10:
        N //= 2
    N = max(N, 256)
    frac = float(rng.choice([0.02, 0.2, 0.5, 1.0]))
    nsets = int(rng.choice([1, 3, 10, 40]))
    most = int(rng.choice([2, 3, 5, 8]))
    sets = [tuple(sorted(rng.choice(np.arange(1, L), size=int(rng.integers(2, max(2, min(most, L - 1)) + 1)), replace=False).tolist()))
            for _ in range(nsets)] if L > 2 else [(1,)]
    flips_at = []
    for d in range(D):
        r = rng.random()
        flips_at.append(sets[int(rng.integers(0, len(sets)))] if r < frac else ((int(rng.integers(1, L)),) if r < 0.7 else ()))
    u8 = int(round(F ** 0.5)) ** 2 == F and bool(rng.integers(0, 2))
    wl = make_workload(3 if u8 else 2, seed=seed, D=D, F=F, L=L, n_train=N)
    wl.level = _levels_from_flips(rng, D, L, flips_at)
    x, _ = wl.train(N)
    what = f"D={D} F={F} L={L} N={N} frac={frac} sets={nsets} most={most} u8={u8}"
    ctx = _ctx(wl)
    got = _encode(ctx, x)
    assert np.array_equal(got, _oracle(wl, x)), what
    ctx.close()
