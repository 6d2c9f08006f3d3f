"""GPU parity of the stand-alone primitives (Sec. IV-B: pack, unpack, horizontal and vertical
summation) and of cosine-similarity inference (Sec. III) against the CPU oracle, through the C
ABI.  Integer results bit-exact; cosines within 1e-6 (fp64 on both sides, fp32 output), and
predictions compared wherever the oracle's best two cosines are further apart than that."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload, pack_bits_lsb  # noqa: E402

from test_gpu_parity import dev_u32, gpu_classical, gpu_encode, host_u32, make_ctx, orc_encode  # noqa: E402


def ctx_for(D, C=2):
    return make_ctx(make_workload(1, D=D, C=C, F=3, L=2))


# D % 16 == 0 takes the vector path when the matrix is 16-byte aligned; the others the byte path
@pytest.mark.parametrize("D,N", [(10000, 700), (10016, 33), (1, 5), (31, 9), (32, 8), (33, 70), (4097, 41),
                                 (16, 1000), (48, 257), (32768, 19)])
def test_pack_and_unpack_bit_exact(D, N):
    rng = np.random.default_rng(D + N)
    bits = rng.integers(0, 2, size=(N, D), dtype=np.uint8)
    loud = bits * rng.integers(1, 256, size=(N, D)).astype(np.uint8)   # any non-zero byte is a 1
    ctx = ctx_for(D)
    want = oracle.pack(loud)
    assert np.array_equal(want, pack_bits_lsb(bits))
    for src in (bits, loud):
        hv = torch.full((N, ctx.W), -1, dtype=torch.int32, device="cuda")
        ctx.hdc_pack(torch.from_numpy(src).cuda(), hv)
        torch.cuda.synchronize()
        assert np.array_equal(host_u32(hv), want)
    back = torch.full((N, D), 7, dtype=torch.uint8, device="cuda")
    ctx.hdc_unpack(dev_u32(want), back)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy(), oracle.unpack(want, D))
    assert np.array_equal(back.cpu().numpy(), bits)
    ctx.close()


def test_pack_and_unpack_unaligned_matrix():
    # a byte matrix that starts 1 byte into an allocation: the byte path, same result
    D, N = 10000, 50
    rng = np.random.default_rng(1)
    bits = rng.integers(0, 2, size=(N, D), dtype=np.uint8)
    ctx = ctx_for(D)
    buf = torch.zeros(N * D + 1, dtype=torch.uint8, device="cuda")
    view = buf[1:].view(N, D)
    view.copy_(torch.from_numpy(bits))
    hv = torch.empty((N, ctx.W), dtype=torch.int32, device="cuda")
    ctx.hdc_pack(view, hv)
    out = torch.zeros(N * D + 1, dtype=torch.uint8, device="cuda")
    ctx.hdc_unpack(hv, out[1:].view(N, D))
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(hv), oracle.pack(bits))
    assert np.array_equal(out[1:].view(N, D).cpu().numpy(), bits) and int(out[0]) == 0
    ctx.close()


@pytest.mark.parametrize("D,N", [(10000, 5000), (33, 7), (1, 3), (2049, 130), (32768, 65), (10000, 70001),
                                 (16384, 9000), (20000, 20001), (10272, 8193), (65536, 300), (70000, 100)])
def test_hsum_and_vsum_bit_exact(D, N):
    rng = np.random.default_rng(D * 3 + N)
    dens = rng.random(N)[:, None]                              # rows of very different weight
    hv = pack_bits_lsb((rng.random((N, D)) < dens).astype(np.uint8))
    ctx = ctx_for(D)
    hd = dev_u32(hv)
    h = torch.full((N,), -1, dtype=torch.int32, device="cuda")
    v = torch.full((D,), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_hsum(hd, h)
    ctx.hdc_vsum(hd, v)
    torch.cuda.synchronize()
    assert np.array_equal(h.cpu().numpy(), oracle.hsum(hv, D))
    assert np.array_equal(v.cpu().numpy(), oracle.vsum(hv, D))
    ctx.hdc_vsum(hd[:0], v)                                    # no rows: zeros
    torch.cuda.synchronize()
    assert int(v.abs().sum()) == 0
    ctx.close()


def test_vsum_leaves_classical_training_intact():
    # both use the context's grouping scratch, one after the other on one stream
    wl = make_workload(2)
    x, y = wl.train(3000)
    ctx = make_ctx(wl)
    hv = gpu_encode(ctx, x)
    o_hv = orc_encode(wl, x)
    v = torch.empty(wl.D, dtype=torch.int32, device="cuda")
    ctx.hdc_vsum(hv, v)
    acc, cn = gpu_classical(ctx, hv, y)
    ctx.hdc_vsum(hv, v)
    torch.cuda.synchronize()
    o_acc, o_cn = oracle.train_classical(o_hv, y, wl.D, wl.C)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(cn.cpu().numpy(), o_cn)
    assert np.array_equal(v.cpu().numpy(), oracle.vsum(o_hv, wl.D))
    ctx.close()


@pytest.mark.parametrize("D,C,N", [(10000, 6, 2947), (1024, 5, 500), (10000, 26, 1559), (33, 1, 7),
                                   (2049, 3, 129), (32768, 2, 40), (4096, 300, 100), (1000, 3, 9000)])
def test_cosine_inference_matches_oracle(D, C, N):
    rng = np.random.default_rng(D + 7 * C + N)
    m = rng.standard_normal((C, D)).astype(np.float32) * rng.uniform(0.1, 50.0, size=(C, 1)).astype(np.float32)
    if C > 2:
        m[1] = 0.0                                             # an all-zero row scores 0
    protos = (m > 0).astype(np.uint8)
    y = rng.integers(0, C, N)
    hv = pack_bits_lsb(protos[y] ^ (rng.random((N, D)) < 0.4).astype(np.uint8))
    ctx = ctx_for(D, C)
    cos = torch.empty((N, C), dtype=torch.float32, device="cuda")
    pred = torch.full((N,), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_search_cosine(dev_u32(hv), torch.from_numpy(m).cuda(), pred, cos)
    torch.cuda.synchronize()
    o_cos, o_pred = oracle.search_cosine(hv, m, D)
    assert np.max(np.abs(cos.cpu().numpy() - o_cos)) < 1e-6
    top2 = np.sort(o_cos, axis=1)[:, -2:] if C > 1 else None
    clear = np.ones(N, bool) if C == 1 else (top2[:, 1] - top2[:, 0] > 1e-9)
    assert clear.mean() > 0.9
    assert np.array_equal(pred.cpu().numpy()[clear], o_pred[clear])
    pred2 = torch.full((N,), -1, dtype=torch.int32, device="cuda")
    ctx.hdc_search_cosine(dev_u32(hv), torch.from_numpy(m).cuda(), pred2, None)   # predictions only
    torch.cuda.synchronize()
    assert torch.equal(pred2, pred)
    ctx.close()


def test_cosine_inference_on_bipolar_rows_ranks_like_hamming():
    # class rows of +-1: cosine = 1 - 2 hamming / D exactly, so both searches agree bit for bit
    rng = np.random.default_rng(9)
    D, C, N = 10000, 26, 1559
    cbits = rng.integers(0, 2, size=(C, D), dtype=np.uint8)
    hv = pack_bits_lsb(cbits[rng.integers(0, C, N)] ^ (rng.random((N, D)) < 0.45).astype(np.uint8))
    ctx = ctx_for(D, C)
    hd = dev_u32(hv)
    pc = torch.empty(N, dtype=torch.int32, device="cuda")
    ph = torch.empty(N, dtype=torch.int32, device="cuda")
    cos = torch.empty((N, C), dtype=torch.float32, device="cuda")
    dist = torch.empty((N, C), dtype=torch.int32, device="cuda")
    ctx.hdc_search_cosine(hd, torch.from_numpy(2.0 * cbits - 1.0).float().cuda(), pc, cos)
    ctx.hdc_search(hd, dev_u32(pack_bits_lsb(cbits)), ph, dist)
    torch.cuda.synchronize()
    o_dist, o_pred = oracle.search(hv, pack_bits_lsb(cbits), D)
    assert np.array_equal(ph.cpu().numpy(), o_pred) and np.array_equal(pc.cpu().numpy(), o_pred)
    want = (1.0 - 2.0 * o_dist.astype(np.float64) / D).astype(np.float32)
    assert np.array_equal(cos.cpu().numpy(), want)
    ctx.close()


def test_primitive_argument_errors():
    from paper_2206_04746_amd import binding as b
    ctx = ctx_for(64)
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    for f in (b.lib.hdc_pack, b.lib.hdc_unpack, b.lib.hdc_hsum):
        assert f(ctx._h, None, 4, t.data_ptr(), None) == b.HDC_EINVAL
        assert f(ctx._h, t.data_ptr(), -1, t.data_ptr(), None) == b.HDC_EINVAL
        assert f(ctx._h, None, 0, None, None) == b.HDC_OK
    assert b.lib.hdc_vsum(ctx._h, None, 4, t.data_ptr(), None) == b.HDC_EINVAL
    assert b.lib.hdc_vsum(ctx._h, t.data_ptr(), 4, None, None) == b.HDC_EINVAL
    assert b.lib.hdc_search_cosine(ctx._h, t.data_ptr(), 4, None, None, t.data_ptr(), None) == b.HDC_EINVAL
    assert b.lib.hdc_search_cosine(ctx._h, None, 0, None, None, None, None) == b.HDC_OK
    ctx.close()
