"""GPU parity: every entry point of libhdc, called through the C ABI binding, against the CPU
oracle on the same seeded inputs.  Bit-exact for encode / classical accumulators / class
vectors / Hamming distances / predictions; 1e-4 relative for the online fp32 accumulators
(fixed sample order).  Sizes span several tiles of every kernel plus ragged tails."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload, pack_bits_lsb  # noqa: E402


def _binding():
    from paper_2206_04746_amd import binding
    return binding


def dev_u32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).cuda()


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)


def make_ctx(wl):
    b = _binding()
    return b.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)


def gpu_encode(ctx, x):
    xd = torch.from_numpy(x).cuda()
    hv = torch.empty((x.shape[0], ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_encode(xd, hv)
    torch.cuda.synchronize()
    return hv


def orc_encode(wl, x):
    return oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)


def rand_hv(rng, N, D):
    return pack_bits_lsb(rng.integers(0, 2, size=(N, D), dtype=np.uint8))


# ------------------------------------------------------------------------------ encode
# small batches take the feature-split launch, the 14000-sample cases the unsplit one
@pytest.mark.parametrize("cfg,n", [(1, 2000), (2, 1500), (3, 1200), (4, 1000), (5, 1100), (5, 14000), (3, 14001)])
def test_encode_configs_bit_exact(cfg, n):
    wl = make_workload(cfg)
    x, _ = wl.train(n)
    ctx = make_ctx(wl)
    got = host_u32(gpu_encode(ctx, x))
    want = orc_encode(wl, x)
    assert np.array_equal(got, want)
    ctx.close()


@pytest.mark.parametrize("D,F,L,N", [
    (1, 1, 1, 1), (31, 2, 2, 5), (32, 3, 2, 16), (33, 31, 16, 17), (64, 32, 16, 15),
    (1000, 33, 7, 63), (2048, 64, 256, 65), (2049, 100, 16, 130), (4097, 63, 3, 33),
    (10000, 127, 64, 19), (10000, 128, 100, 21), (12345, 1000, 5, 9), (10000, 2100, 9, 6),
])
def test_encode_ragged_shapes_bit_exact(D, F, L, N):
    wl = make_workload(2, seed=D + F, D=D, F=F, L=L, n_train=N)
    x, _ = wl.train(N)
    # push some values onto and beyond the range edges, and a NaN
    x = x.copy()
    x.ravel()[::7] = -1.0
    x.ravel()[3::11] = 1.0
    x.ravel()[5::13] = 1.5
    x.ravel()[::97] = np.nan
    ctx = make_ctx(wl)
    got = host_u32(gpu_encode(ctx, x))
    assert np.array_equal(got, orc_encode(wl, x))
    last_bits = D - 32 * (ctx.W - 1)
    if last_bits < 32:
        assert np.all(got[:, -1] >> last_bits == 0)        # pad bits are written as zero
    ctx.close()


# few samples: the waves of a block share one sample (16 waves each up to 256 sample-slices, 8 up
# to 2048, one-sample units beyond); feature counts chosen to need 8, 10, 12 and 16 count planes
# and half-block counts that do not divide by the waves
@pytest.mark.parametrize("D,F,L,N", [
    (10000, 617, 64, 1), (10000, 617, 64, 2), (10000, 617, 64, 85), (10000, 617, 64, 86),
    (10000, 617, 64, 682), (10000, 617, 64, 683), (10000, 100, 16, 40), (10000, 1100, 7, 30),
    (2048, 5000, 9, 5), (2048, 5000, 9, 70), (100, 15, 256, 300), (64, 1, 2, 3000), (4100, 784, 256, 25),
])
def test_encode_few_samples_bit_exact(D, F, L, N):
    wl = make_workload(2, seed=D + F + N, D=D, F=F, L=L, n_train=N)
    x, _ = wl.train(N)
    ctx = make_ctx(wl)
    assert np.array_equal(host_u32(gpu_encode(ctx, x)), orc_encode(wl, x))
    ctx.close()


def test_encode_u8_levels_and_random_tables():
    rng = np.random.default_rng(5)
    for L in (256, 100, 2):
        wl = make_workload(3, F=36, L=L, D=777, n_train=50)
        wl.level = rand_hv(rng, L, wl.D)                    # unrelated level vectors, not linear
        x = rng.integers(0, 256, size=(50, wl.F), dtype=np.uint8)
        ctx = make_ctx(wl)
        assert np.array_equal(host_u32(gpu_encode(ctx, x)), orc_encode(wl, x))
        ctx.close()


def test_encode_forced_ties_follow_tie_vector():
    # F = 2 with complementary level choice forces an exact tie in every dimension where the
    # two bound vectors differ.
    wl = make_workload(1, D=300, F=2, L=4, n_train=40)
    x, _ = wl.train(40)
    ctx = make_ctx(wl)
    assert np.array_equal(host_u32(gpu_encode(ctx, x)), orc_encode(wl, x))
    ctx.close()


def test_encode_empty_and_chunk_boundary():
    wl = make_workload(1, D=96, F=5, L=4, n_train=70000)
    ctx = make_ctx(wl)
    hv = torch.empty((0, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_encode(torch.empty((0, wl.F), dtype=torch.float32, device="cuda"), hv)
    x, _ = wl.train(70000)                                   # crosses the 65536-sample chunk
    got = host_u32(gpu_encode(ctx, x))
    assert np.array_equal(got, orc_encode(wl, x))
    ctx.close()


# ------------------------------------------------------------------ classical training
def gpu_classical(ctx, hv_d, y, acc=None, cn=None):
    yd = torch.from_numpy(y).cuda()
    acc = torch.zeros((ctx.C, ctx.D), dtype=torch.int32, device="cuda") if acc is None else acc
    cn = torch.zeros(ctx.C, dtype=torch.int64, device="cuda") if cn is None else cn
    ctx.hdc_train_classical(hv_d, yd, acc, cn)
    torch.cuda.synchronize()
    return acc, cn


# up to 8192 rows one fused launch does everything; up to 32768 one block groups the rows; beyond,
# grouping runs over many blocks
@pytest.mark.parametrize("D,C,N", [(1024, 5, 2000), (10000, 26, 6238), (10000, 2, 9000),
                                   (33, 1, 10), (2049, 7, 4100), (10000, 100, 700),
                                   (10000, 2, 70001), (4000, 26, 40000), (64, 1000, 50000),
                                   (2000, 1, 40001), (512, 3, 150000), (320, 2, 300007),
                                   (3000, 4, 260000), (10000, 5, 33000), (9000, 2, 8193),
                                   # rows of more than 320 words and up to four classes: column slices of up to 320
                                   # words, a pass each (two slices; three; four of 256; a last slice of few words;
                                   # the widest rows of this path); more classes or wider rows: grouped rows, a slice
                                   # of 64 words per wave
                                   (12000, 2, 40000), (20000, 3, 20001), (10400, 1, 9000), (10272, 4, 9001), (16384, 2, 30000),
                                   (32768, 4, 12000), (30001, 2, 9000), (20512, 3, 8200), (65536, 2, 8300), (65600, 2, 8300),
                                   (20000, 5, 9000), (16384, 26, 9000),
                                   # slices that do not fill the last block of sixteen
                                   (40000, 5, 9000), (34000, 26, 8200), (100000, 3, 8193),
                                   # the fused launch at its row limit: everything in one or two classes,
                                   # many classes, a dimension count that is no multiple of 4, very wide rows
                                   (10000, 1, 8192), (10000, 2, 8192), (1024, 1000, 8000), (10001, 3, 5000),
                                   (70000, 2, 300), (31, 4, 8192), (10000, 26, 8193)])
def test_classical_accumulate_and_binarize_bit_exact(D, C, N):
    rng = np.random.default_rng(D + C)
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    hv = rand_hv(rng, N, D)
    y = rng.integers(0, C, N).astype(np.int32)
    if C > 2:
        y[y == 1] = 0                                        # class 1 stays empty
    y[::50] = C + 3                                          # out-of-range labels are skipped
    y[1::50] = -1
    ctx = make_ctx(wl)
    hv_d = dev_u32(hv)
    acc, cn = gpu_classical(ctx, hv_d, y)
    want_acc, want_cn = oracle.train_classical(hv, y, D, C)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    assert np.array_equal(cn.cpu().numpy(), want_cn)
    m = torch.empty((C, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_binarize_classical(acc, cn, m)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(m), oracle.binarize_classical(want_acc, want_cn, wl.tie))
    # chunks compose: second half added onto the first gives the same sums
    h = N // 3
    a2, n2 = gpu_classical(ctx, hv_d[:h].contiguous(), y[:h])
    a2, n2 = gpu_classical(ctx, hv_d[h:].contiguous(), y[h:], a2, n2)
    assert torch.equal(a2, acc) and torch.equal(n2, cn)
    ctx.close()


# ------------------------------------------------------------------------------ search
@pytest.mark.parametrize("D,C,N", [(1024, 5, 500), (10000, 26, 1559), (10000, 2, 3001),
                                   (10000, 10, 1000), (10000, 6, 2947), (33, 1, 7), (31, 17, 66),
                                   (2049, 16, 129), (20000, 33, 50), (32768, 3, 20), (10000, 100, 64),
                                   # from 8192 queries on: the kernel that stages the class vectors in LDS
                                   (10000, 26, 9000), (2049, 16, 8193), (20000, 33, 8192), (31, 17, 20000),
                                   # class vectors larger than LDS: read from global memory at any N
                                   (10000, 200, 8200), (4096, 1024, 8192),
                                   # rows longer than a wave's registers hold
                                   (40000, 5, 50), (33000, 26, 9), (100000, 3, 8200)])
def test_search_bit_exact(D, C, N):
    rng = np.random.default_rng(D * 7 + C)
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    cls = rand_hv(rng, C, D)
    # queries: noisy copies of class vectors, so minima are meaningful, plus exact ties
    src = rng.integers(0, C, N)
    q_bits = oracle.unpack(cls, D)[src]
    flips = rng.random((N, D)) < 0.3
    q_bits = q_bits ^ flips.astype(np.uint8)
    q = pack_bits_lsb(q_bits)
    if C > 2:
        cls[2] = cls[0]                                      # duplicate class: argmin must pick 0
    ctx = make_ctx(wl)
    qd, cd = dev_u32(q), dev_u32(cls)
    dist = torch.empty((N, C), dtype=torch.int32, device="cuda")
    pred = torch.empty(N, dtype=torch.int32, device="cuda")
    ctx.hdc_search(qd, cd, pred, dist)
    torch.cuda.synchronize()
    want_d, want_p = oracle.search(q, cls, D)
    assert np.array_equal(host_u32(dist), want_d)
    assert np.array_equal(pred.cpu().numpy(), want_p)
    pred2 = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    ctx.hdc_search(qd, cd, pred2, None)                      # predictions only
    torch.cuda.synchronize()
    assert torch.equal(pred2, pred)
    ctx.close()


# Long query streams whose rows fill 16 lanes with 16-byte pieces take a kernel with one row per 16
# lanes: every size of its piece count, rows ending 1, 2, 3 or 4 words into the last piece, rows
# whose last word is partial, class counts on both sides of each group width, a ragged last tile.
@pytest.mark.parametrize("D,C,N", [(2048, 3, 8193), (1761, 9, 8195), (3900, 2, 8194), (6000, 17, 8192),
                                   (8001, 8, 8197), (10000, 10, 8195), (10240, 1, 8193), (12000, 26, 8194),
                                   (16384, 16, 8195), (24000, 5, 8193), (31000, 4, 8194), (32768, 2, 8195),
                                   (10000, 40, 8193),
                                   # from 8192 queries on with 13 to 31 classes, from 20480 on with 9 to 12, D up
                                   # to 10240: the matrix-core kernel (64 rows per block at a time, a row split in
                                   # two halves, every half in eight slices); around it the shapes that just miss it
                                   (10000, 26, 8192), (10000, 26, 8191), (10000, 13, 8193), (10000, 12, 20480), (10000, 12, 20479),
                                   (10000, 26, 32771), (10000, 12, 32833), (2049, 31, 32768), (128, 19, 40001),
                                   (20000, 12, 32770), (4127, 16, 32801), (7000, 11, 32769), (10000, 32, 32768), (10000, 8, 32768), (10000, 9, 32768), (6400, 31, 32770), (10030, 13, 32785), (10240, 20, 32768), (10241, 20, 32768),
                                   # more than 31 classes: up to four passes over the class slots; 125 miss it
                                   (10000, 62, 8195), (10000, 63, 8193), (9000, 93, 8194), (10000, 94, 8200), (10000, 124, 8199),
                                   (10000, 125, 8192), (10000, 64, 8195), (10000, 128, 8193), (10000, 129, 8192), (5000, 96, 8194), (10000, 33, 8193), (2049, 50, 16390), (400, 100, 16411), (6000, 77, 8193),
                                   # D above 10240: a tile of 32 rows per block at a time, every count of slices
                                   (10272, 9, 20481), (14000, 31, 8193), (12288, 26, 8195), (14336, 13, 8193), (14337, 13, 8193), (13000, 40, 8194), (11000, 32, 8200), (18000, 13, 8195), (23000, 16, 8197), (26000, 14, 8194),
                                   (30000, 13, 8193), (32768, 20, 8193), (32737, 31, 8225), (32800, 14, 8192), (16384, 40, 8200)])
def test_search_long_streams_bit_exact(D, C, N):
    rng = np.random.default_rng(D + 13 * C)
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    W = (D + 31) // 32
    tail = np.uint32((1 << (D - 32 * (W - 1))) - 1) if D % 32 else np.uint32(0xffffffff)

    def rand_rows(n):
        r = rng.integers(0, 2 ** 32, size=(n, W), dtype=np.uint64).astype(np.uint32)
        r[:, -1] &= tail
        return r
    cls = rand_rows(C)
    q = rand_rows(N)
    # every third query: a class vector with a few words disturbed (a clear nearest class); some exact
    near = np.arange(0, N, 3)
    q[near] = cls[rng.integers(0, C, near.size)]
    q[near[::2], rng.integers(0, W, near[::2].size)] ^= np.uint32(0x00f0f00f) & (tail if W == 1 else np.uint32(0xffffffff))
    q[:, -1] &= tail
    if C > 2:
        cls[2] = cls[0]                                      # duplicate class: argmin must pick 0
    ctx = make_ctx(wl)
    qd, cd = dev_u32(q), dev_u32(cls)
    dist = torch.full((N, C), -1, dtype=torch.int32, device="cuda")
    pred = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    ctx.hdc_search(qd, cd, pred, dist)
    torch.cuda.synchronize()
    want_d, want_p = oracle.search(q, cls, D)
    assert np.array_equal(host_u32(dist), want_d)
    assert np.array_equal(pred.cpu().numpy(), want_p)
    pred2 = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    ctx.hdc_search(qd, cd, pred2, None)
    torch.cuda.synchronize()
    assert torch.equal(pred2, pred)
    ctx.close()


# Level tables decide which dimensions encode to a per-model constant (every level vector has the
# same bit there).  The library then encodes only the other dimensions and spreads the result:
# the output must not depend on how many dimensions vary, nor on where they sit.
@pytest.mark.parametrize("D,F,L,N,vary", [
    (10000, 617, 64, 300, 1.0),      # every dimension varies: nothing to leave out
    (10000, 617, 64, 300, 0.80),     # too few invariant dimensions to bother
    (10000, 617, 64, 300, 0.74),     # just enough
    (10000, 128, 16, 200, 0.10),     # almost everything is a constant
    (10000, 33, 5, 100, 0.0),        # identical level vectors: the whole hypervector is a constant
    (10000, 61, 1, 50, 1.0),         # one level: same thing
    (4097, 100, 8, 120, 0.5), (33, 7, 4, 40, 0.5), (64, 8, 4, 40, 0.03), (2048, 64, 256, 65, 0.6),
    (20000, 40, 3, 30, 0.33)])
def test_encode_any_pattern_of_level_invariant_dimensions(D, F, L, N, vary):
    rng = np.random.default_rng(int(D + 7 * F + 13 * L + 1000 * vary))
    wl = make_workload(1, D=D, F=F, L=L)
    lv = np.repeat(rng.integers(0, 2, size=(1, D), dtype=np.uint8), L, axis=0)
    cols = np.flatnonzero(rng.random(D) < vary)              # scattered, not a prefix
    if L > 1 and cols.size:
        lv[:, cols] = rng.integers(0, 2, size=(L, cols.size), dtype=np.uint8)
        lv[1, cols] = lv[0, cols] ^ 1                        # each chosen dimension really varies
    wl.level = pack_bits_lsb(lv)
    x, _ = wl.train(N)
    ctx = make_ctx(wl)
    got = host_u32(gpu_encode(ctx, x))
    assert np.array_equal(got, orc_encode(wl, x))
    # what the library says it bundles: everything, or just the varying dimensions
    varying = int(cols.size) if L > 1 else 0
    want_words = ctx.W if 4 * varying > 3 * D else (varying + 31) // 32
    assert ctx.hdc_encoded_words() == want_words
    ctx.close()


# --------------------------------------------------------------------- online training
def rel_err(got, want):
    scale = np.maximum(np.abs(want), 1e-3 * np.abs(want).max() + 1e-30)
    return float(np.max(np.abs(got - want) / scale))


@pytest.mark.parametrize("D,C,N,epochs,lr", [(1024, 5, 600, 2, 1.0), (10000, 6, 1500, 3, 1.0),
                                             (10000, 26, 300, 1, 0.5), (33, 1, 20, 2, 1.0),
                                             (2049, 3, 100, 1, 0.0), (32768, 2, 40, 1, 1.0),
                                             # more samples than one prepared chunk (16384), two epochs
                                             (1024, 3, 20000, 2, 1.0),
                                             # 12 < C: the kernel with a butterfly per value; C > 80: accumulators in memory
                                             (1024, 20, 300, 1, 1.0), (512, 100, 120, 1, 1.0)])
def test_online_training_matches_oracle(D, C, N, epochs, lr):
    rng = np.random.default_rng(D + C + N)
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    protos = rng.integers(0, 2, size=(C, D), dtype=np.uint8)
    y = rng.integers(0, C, N).astype(np.int32)
    bits = protos[y] ^ (rng.random((N, D)) < 0.35).astype(np.uint8)
    hv = pack_bits_lsb(bits)
    y[N // 2] = C                                            # one out-of-range label: skipped
    ctx = make_ctx(wl)
    acc = torch.zeros((C, D), dtype=torch.float32, device="cuda")
    ctx.hdc_train_online(dev_u32(hv), torch.from_numpy(y).cuda(), acc, epochs=epochs, lr=lr)
    torch.cuda.synchronize()
    want = oracle.train_online(hv, y, D, C, epochs=epochs, lr=lr)
    got = acc.cpu().numpy()
    assert rel_err(got, want) < 1e-4
    m = torch.empty((C, ctx.W), dtype=torch.int32, device="cuda")
    acc_same = torch.from_numpy(want).cuda()                 # binarise identical inputs
    acc_same[0, :7] = 0.0                                    # exact zeros take the tie bit
    ctx.hdc_binarize_online(acc_same, m)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(m), oracle.binarize_online(acc_same.cpu().numpy(), wl.tie))
    # continuing from a non-zero model: a second call equals one more epoch
    if epochs == 1:
        ctx.hdc_train_online(dev_u32(hv), torch.from_numpy(y).cuda(), acc, epochs=1, lr=lr)
        torch.cuda.synchronize()
        want2 = oracle.train_online(hv, y, D, C, epochs=2, lr=lr)
        assert rel_err(acc.cpu().numpy(), want2) < 1e-4
    ctx.close()


# -------------------------------------------------------------------------- end to end
@pytest.mark.parametrize("cfg,ntr,nte", [(1, 2000, 500), (2, 6238, 1559), (3, 2500, 1000), (4, 2000, 800)])
def test_end_to_end_pipeline_matches_oracle(cfg, ntr, nte):
    wl = make_workload(cfg)
    xt, yt = wl.train(ntr)
    xs, ys = wl.test(nte)
    ctx = make_ctx(wl)
    ht, hs = gpu_encode(ctx, xt), gpu_encode(ctx, xs)
    o_ht, o_hs = orc_encode(wl, xt), orc_encode(wl, xs)
    assert np.array_equal(host_u32(ht), o_ht) and np.array_equal(host_u32(hs), o_hs)
    m = torch.empty((wl.C, ctx.W), dtype=torch.int32, device="cuda")
    if wl.mode == "classical":
        acc, cn = gpu_classical(ctx, ht, yt)
        ctx.hdc_binarize_classical(acc, cn, m)
        o_acc, o_cn = oracle.train_classical(o_ht, yt, wl.D, wl.C)
        assert np.array_equal(acc.cpu().numpy(), o_acc)
        o_m = oracle.binarize_classical(o_acc, o_cn, wl.tie)
    else:
        acc = torch.zeros((wl.C, wl.D), dtype=torch.float32, device="cuda")
        ctx.hdc_train_online(ht, torch.from_numpy(yt).cuda(), acc, epochs=wl.epochs, lr=wl.lr)
        ctx.hdc_binarize_online(acc, m)
        o_acc = oracle.train_online(o_ht, yt, wl.D, wl.C, epochs=wl.epochs, lr=wl.lr)
        torch.cuda.synchronize()
        assert rel_err(acc.cpu().numpy(), o_acc) < 1e-4
        o_m = oracle.binarize_online(o_acc, wl.tie)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(m), o_m)
    dist = torch.empty((nte, wl.C), dtype=torch.int32, device="cuda")
    pred = torch.empty(nte, dtype=torch.int32, device="cuda")
    ctx.hdc_search(hs, m, pred, dist)
    torch.cuda.synchronize()
    o_dist, o_pred = oracle.search(o_hs, o_m, wl.D)
    assert np.array_equal(host_u32(dist), o_dist) and np.array_equal(pred.cpu().numpy(), o_pred)
    assert (o_pred == ys).mean() > 0.5
    ctx.close()


# ----------------------------------------------------------------------- error handling
def test_argument_errors_are_reported_not_faulted():
    b = _binding()
    wl = make_workload(1, D=64, F=4, L=4, C=2)
    bad_tie = wl.tie.copy()
    with pytest.raises(b.HdcError) as e:
        b.Context(63, wl.F, wl.L, wl.C, wl.item, wl.level, bad_tie | np.uint32(0x80000000),
                  wl.lo, wl.scale)                           # pad bit set
    assert e.value.code == b.HDC_EINVAL
    with pytest.raises(b.HdcError):
        b.Context(wl.D, wl.F, 300, wl.C, wl.item, np.zeros((300, 2), np.uint32), wl.tie, wl.lo, wl.scale)
    ctx = make_ctx(wl)
    hv = torch.zeros((4, ctx.W), dtype=torch.int32, device="cuda")
    assert b.lib.hdc_search(ctx._h, hv.data_ptr(), 4, None, None, None, None) == b.HDC_EINVAL
    assert b.lib.hdc_encode(ctx._h, None, 4, hv.data_ptr(), None) == b.HDC_EINVAL
    assert b.lib.hdc_encode(ctx._h, None, -1, None, None) == b.HDC_EINVAL
    assert b.lib.hdc_train_online(ctx._h, hv.data_ptr(), hv.data_ptr(), 4, -1, 1.0, hv.data_ptr(), None) \
        == b.HDC_EINVAL
    assert b.lib.hdc_encode(ctx._h, None, 0, None, None) == b.HDC_OK      # N == 0 is a no-op
    ctx.close()


def test_online_training_beyond_the_register_resident_dimensions():
    # D > 32768: the per-sample trainer hands over to the batched one with batches of one sample
    rng = np.random.default_rng(3)
    D, C, N = 40000, 3, 24
    wl = make_workload(1, D=D, C=C, F=3, L=2)
    hv_h = rand_hv(rng, N, D)
    y = rng.integers(0, C, N).astype(np.int32)
    ctx = make_ctx(wl)
    acc = torch.zeros((C, D), dtype=torch.float32, device="cuda")
    ctx.hdc_train_online(dev_u32(hv_h), torch.from_numpy(y).cuda(), acc, 2, 1.0)
    torch.cuda.synchronize()
    want = oracle.train_online(hv_h, y, D, C, 2, 1.0)
    got = acc.cpu().numpy()
    assert np.max(np.abs(got - want)) <= 1e-4 * np.max(np.abs(want))
    ctx.close()


# ------------------------------------------------- full sizes of the benchmark configurations
def test_config3_full_size_classical_pipeline():
    """MNIST-shaped config at its full size (60000 train / 10000 test, u8 features, L=256)."""
    wl = make_workload(3)
    xt, yt = wl.train()
    xs, ys = wl.test()
    ctx = make_ctx(wl)
    ht, hs = gpu_encode(ctx, xt), gpu_encode(ctx, xs)
    acc, cn = gpu_classical(ctx, ht, yt)
    m = torch.empty((wl.C, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_binarize_classical(acc, cn, m)
    pred = torch.empty(xs.shape[0], dtype=torch.int32, device="cuda")
    dist = torch.empty((xs.shape[0], wl.C), dtype=torch.int32, device="cuda")
    ctx.hdc_search(hs, m, pred, dist)
    torch.cuda.synchronize()
    o_ht, o_hs = orc_encode(wl, xt), orc_encode(wl, xs)
    assert np.array_equal(host_u32(ht), o_ht) and np.array_equal(host_u32(hs), o_hs)
    o_acc, o_cn = oracle.train_classical(o_ht, yt, wl.D, wl.C)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(cn.cpu().numpy(), o_cn)
    o_m = oracle.binarize_classical(o_acc, o_cn, wl.tie)
    assert np.array_equal(host_u32(m), o_m)
    o_dist, o_pred = oracle.search(o_hs, o_m, wl.D)
    assert np.array_equal(host_u32(dist), o_dist) and np.array_equal(pred.cpu().numpy(), o_pred)
    ctx.close()


def test_config4_full_size_online_pipeline():
    """UCIHAR-shaped config at its full size: 7352 samples, 3 epochs, fixed order."""
    wl = make_workload(4)
    xt, yt = wl.train()
    xs, _ = wl.test()
    ctx = make_ctx(wl)
    ht, hs = gpu_encode(ctx, xt), gpu_encode(ctx, xs)
    acc = torch.zeros((wl.C, wl.D), dtype=torch.float32, device="cuda")
    ctx.hdc_train_online(ht, torch.from_numpy(yt).cuda(), acc, epochs=wl.epochs, lr=wl.lr)
    m = torch.empty((wl.C, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_binarize_online(acc, m)
    pred = torch.empty(xs.shape[0], dtype=torch.int32, device="cuda")
    ctx.hdc_search(hs, m, pred, None)
    torch.cuda.synchronize()
    o_ht, o_hs = orc_encode(wl, xt), orc_encode(wl, xs)
    assert np.array_equal(host_u32(ht), o_ht)
    o_acc, o_pred_log, margin = oracle.train_online(o_ht, yt, wl.D, wl.C, epochs=wl.epochs, lr=wl.lr, log=True)
    assert rel_err(acc.cpu().numpy(), o_acc) < 1e-4
    # where the sign of an accumulator is not within rounding of zero the class bits must agree
    o_m = oracle.binarize_online(o_acc, wl.tie)
    safe = np.abs(o_acc) > 1e-3 * np.abs(o_acc).max()
    got_bits, want_bits = oracle.unpack(host_u32(m), wl.D), oracle.unpack(o_m, wl.D)
    assert np.array_equal(got_bits[safe], want_bits[safe])
    if np.array_equal(host_u32(m), o_m):
        _, o_pred = oracle.search(o_hs, o_m, wl.D)
        assert np.array_equal(pred.cpu().numpy(), o_pred)
    ctx.close()


def test_config5_full_stream_invariants_and_sampled_parity():
    """CHB-MIT-shaped stream at its full size: 5,000,000 windows in five 1M-window chunks are
    encoded, accumulated and searched.  The oracle is far too slow for 5M encodes, so it checks
    sampled windows one by one (from its own inputs only); integer invariants cover the rest."""
    wl = make_workload(5)
    ctx = make_ctx(wl)
    chunk, nchunks, nsub = 1_000_000, 5, 5000
    acc = torch.zeros((wl.C, wl.D), dtype=torch.int32, device="cuda")
    cn = torch.zeros(wl.C, dtype=torch.int64, device="cuda")
    hv_all, y_all, samples = [], [], []
    o_m_sub = None
    for ci in range(nchunks):
        x, y = wl.train(chunk, start=ci * chunk)
        hv = gpu_encode(ctx, x)
        # sampled parity of the encoder: a prefix and a random scatter of every chunk
        rows = np.unique(np.concatenate([np.arange(300), np.random.default_rng(ci).choice(chunk, 300)]))
        o_rows = orc_encode(wl, x[rows])
        assert np.array_equal(host_u32(hv[torch.from_numpy(rows).cuda()]), o_rows)
        samples.append((ci * chunk + rows, o_rows))
        if ci == 0:   # a subset small enough for the oracle to train on
            o_hv = orc_encode(wl, x[:nsub])
            assert np.array_equal(host_u32(hv[:nsub]), o_hv)
            a_s, n_s = gpu_classical(ctx, hv[:nsub].contiguous(), y[:nsub])
            o_a, o_n = oracle.train_classical(o_hv, y[:nsub], wl.D, wl.C)
            assert np.array_equal(a_s.cpu().numpy(), o_a) and np.array_equal(n_s.cpu().numpy(), o_n)
            o_m_sub = oracle.binarize_classical(o_a, o_n, wl.tie)
        acc, cn = gpu_classical(ctx, hv, y, acc, cn)
        hv_all.append(hv)
        y_all.append(y)
        del x
    hv_cat = torch.cat(hv_all)
    del hv_all
    y_cat = np.concatenate(y_all)
    N = hv_cat.shape[0]
    assert N == 5_000_000
    # chunked == unchunked (integer sums compose in any order); counts match the labels
    acc1, cn1 = gpu_classical(ctx, hv_cat, y_cat)
    assert torch.equal(acc1, acc) and torch.equal(cn1, cn)
    assert np.array_equal(cn.cpu().numpy(), np.bincount(y_cat, minlength=wl.C))
    # sum over dimensions of acc[c] == total popcount of the class's vectors; the popcounts come
    # from a different kernel: Hamming distance to the all-zero vector
    zero = torch.zeros((wl.C, ctx.W), dtype=torch.int32, device="cuda")
    pc = torch.empty((N, wl.C), dtype=torch.int32, device="cuda")
    pr = torch.empty(N, dtype=torch.int32, device="cuda")
    ctx.hdc_search(hv_cat, zero, pr, pc)
    torch.cuda.synchronize()
    yd = torch.from_numpy(y_cat).cuda()
    for c in range(wl.C):
        assert int(acc[c].sum(dtype=torch.int64)) == int(pc[yd == c, 0].sum(dtype=torch.int64))
    assert int((pr != 0).sum()) == 0                       # equal distances: lowest class wins
    # class vectors of the full stream obey the majority rule (checked with plain tensor ops)
    m = torch.empty((wl.C, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_binarize_classical(acc, cn, m)
    torch.cuda.synchronize()
    tie_bits = np.unpackbits(wl.tie.view(np.uint8), bitorder="little")[:wl.D]
    a_h, n_h = acc.cpu().numpy().astype(np.int64), cn.cpu().numpy()
    want = np.where(2 * a_h > n_h[:, None], 1, np.where(2 * a_h < n_h[:, None], 0, tie_bits[None, :]))
    got = np.unpackbits(host_u32(m).view(np.uint8), axis=1, bitorder="little")[:, :wl.D]
    assert np.array_equal(got, want)
    # search of all 5M windows against the oracle-trained subset model: sampled rows one by one
    dist = torch.empty((N, wl.C), dtype=torch.int32, device="cuda")
    ctx.hdc_search(hv_cat, dev_u32(o_m_sub), pr, dist)
    torch.cuda.synchronize()
    assert int(dist.min()) >= 0 and int(dist.max()) <= wl.D
    for rows, o_rows in samples:
        o_d, o_p = oracle.search(o_rows, o_m_sub, wl.D)
        idx = torch.from_numpy(rows).cuda()
        assert np.array_equal(host_u32(dist[idx]), o_d) and np.array_equal(pr[idx].cpu().numpy(), o_p)
    ctx.close()
