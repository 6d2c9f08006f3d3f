"""Pins for the CPU oracle: hand-worked fixtures, closed forms, brute force on tiny
inputs, library special cases and invariants.  None of these tests touches the GPU
library.  Citations are to arXiv 2206.04746: Sec. III (Eqs. 1-3) and Sec. IV-B."""
import itertools
import os

import numpy as np
import pytest

import oracle
from workloads import make_workload, pack_bits_lsb

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_bits(rng, *shape):
    return rng.integers(0, 2, size=shape, dtype=np.uint8)


def bits_of(s):
    return np.array([int(ch) for ch in s], dtype=np.uint8)


# --------------------------------------------------------------------- pack / unpack
def test_pack_is_lsb_first_with_zero_pad():
    # Sec. IV-B1: bits go into 32-bit integers; dimension d is bit d%32 of word d//32.
    D = 70
    for d, (word, value) in {0: (0, 1), 5: (0, 32), 31: (0, 0x80000000), 32: (1, 1),
                             69: (2, 1 << 5)}.items():
        b = np.zeros((1, D), dtype=np.uint8)
        b[0, d] = 1
        w = oracle.pack(b)
        assert w.shape == (1, 3) and w.dtype == np.uint32
        expect = np.zeros(3, dtype=np.uint32)
        expect[word] = value
        assert np.array_equal(w[0], expect)
    ones = oracle.pack(np.ones((1, D), dtype=np.uint8))
    assert ones[0].tolist() == [0xFFFFFFFF, 0xFFFFFFFF, 0x3F]  # pad bits 70..95 stay zero


@pytest.mark.parametrize("D", [1, 31, 32, 33, 64, 1000])
def test_pack_matches_numpy_packbits_and_roundtrips(D):
    rng = np.random.default_rng(D)
    b = rand_bits(rng, 7, D)
    w = oracle.pack(b)
    assert np.array_equal(w, pack_bits_lsb(b))          # numpy.packbits(bitorder="little")
    assert np.array_equal(oracle.unpack(w, D), b)


# ------------------------------------------------------------------------- quantiser
def test_quantiser_edges_f32():
    L = 16
    lo = np.array([0.0, -1.0], dtype=np.float32)
    hi = np.array([1.0, 1.0])
    scale = (L / (hi - lo)).astype(np.float32)
    x = np.array([[0.0, -1.0],        # x == lo  -> bin 0
                  [1.0, 1.0],         # x == hi  -> last bin
                  [-3.0, -1.5],       # below    -> 0
                  [7.0, 1.0001],      # above    -> L-1
                  [np.nan, np.nan],   # NaN      -> 0
                  [np.inf, -np.inf],
                  [0.5, 0.0],         # exact bin edge k/L -> bin k
                  [0.49999997, -1e-7]], dtype=np.float32)
    q = oracle.quantize(x, L, lo, scale)
    assert q.tolist() == [[0, 0], [15, 15], [0, 0], [15, 15], [0, 0], [15, 0], [8, 8], [7, 7]]


def test_quantiser_bin_edges_exact_and_monotone():
    # [0,1) in L=16 equal bins: every k/16 is exact in fp32 and opens bin k.
    L = 16
    lo, scale = np.zeros(1, np.float32), np.full(1, 16.0, np.float32)
    edges = (np.arange(L) / L).astype(np.float32)[:, None]
    assert oracle.quantize(edges, L, lo, scale)[:, 0].tolist() == list(range(L))
    just_below = np.nextafter(edges[1:], np.float32(-1))
    assert oracle.quantize(just_below, L, lo, scale)[:, 0].tolist() == list(range(L - 1))
    xs = np.sort(np.random.default_rng(0).uniform(-0.2, 1.2, 5000)).astype(np.float32)[:, None]
    q = oracle.quantize(xs, L, lo, scale)[:, 0]
    assert np.all(np.diff(q) >= 0) and q.min() == 0 and q.max() == L - 1
    # equal-width: inside the range the bin is floor((x-lo)/(hi-lo)*L) (floor, not round)
    inside = (xs[:, 0] >= 0) & (xs[:, 0] < 1)
    assert np.array_equal(q[inside], np.floor(xs[inside, 0].astype(np.float64) * L).astype(int))


def test_quantiser_u8():
    x = np.arange(256, dtype=np.uint8)[:, None]
    assert np.array_equal(oracle.quantize(x, 256)[:, 0], np.arange(256))        # identity
    assert np.array_equal(oracle.quantize(x, 64)[:, 0], np.arange(256) // 4)    # 4 values per bin
    assert np.array_equal(oracle.quantize(x, 2)[:, 0], (np.arange(256) >= 128).astype(int))
    q100 = oracle.quantize(x, 100)[:, 0]
    assert q100[0] == 0 and q100[255] == 99 and np.all(np.diff(q100) >= 0)


# -------------------------------------------------------------------------- encoding
def test_encode_hand_case_from_golden_file():
    ids, levels, tie, cases = [], [], None, []
    for line in open(os.path.join(GOLDEN, "encode_hand_case.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "id":
            ids.append(bits_of(t[1]))
        elif t[0] == "level":
            levels.append(bits_of(t[1]))
        elif t[0] == "tie":
            tie = bits_of(t[1])
        elif t[0] == "q":
            cases.append(([int(v) for v in t[1:5]], bits_of(t[6])))
    q = np.array([c[0] for c in cases], dtype=np.int32)
    hv = oracle.encode_bits(q, np.array(ids), np.array(levels), tie)
    assert np.array_equal(hv, np.array([c[1] for c in cases]))


def test_encode_single_feature_is_the_bound_vector():
    # F = 1: the "majority" of one vector is the vector: H = ID_0 xor V_q (Eq. 1).
    rng = np.random.default_rng(1)
    D, L = 77, 5
    item, level, tie = rand_bits(rng, 1, D), rand_bits(rng, L, D), rand_bits(rng, D)
    q = np.arange(L, dtype=np.int32)[:, None]
    hv = oracle.encode_bits(q, item, level, tie)
    assert np.array_equal(hv, item[0][None, :] ^ level)
    # XOR is self-inverse: binding the result with the level again gives the ID back.
    assert np.array_equal(hv ^ level, np.repeat(item, L, axis=0))


def test_encode_two_and_three_features_closed_forms():
    rng = np.random.default_rng(2)
    D, L = 130, 4
    level, tie = rand_bits(rng, L, D), rand_bits(rng, D)
    for F in (2, 3):
        item = rand_bits(rng, F, D)
        q = rng.integers(0, L, size=(9, F)).astype(np.int32)
        hv = oracle.encode_bits(q, item, level, tie)
        for n in range(q.shape[0]):
            b = [item[f] ^ level[q[n, f]] for f in range(F)]
            if F == 3:   # majority of three = (a&b)|(a&c)|(b&c)
                want = (b[0] & b[1]) | (b[0] & b[2]) | (b[1] & b[2])
            else:        # two votes: agree -> that bit, disagree (tie) -> tie vector
                want = (b[0] & b[1]) | ((b[0] ^ b[1]) & tie)
            assert np.array_equal(hv[n], want)


@pytest.mark.parametrize("D,F,L", [(1, 1, 2), (31, 2, 2), (33, 4, 3), (64, 5, 16), (40, 100, 16)])
def test_encode_brute_force_per_bit(D, F, L):
    rng = np.random.default_rng(D * 1000 + F)
    item, level, tie = rand_bits(rng, F, D), rand_bits(rng, L, D), rand_bits(rng, D)
    q = rng.integers(0, L, size=(6, F)).astype(np.int32)
    hv = oracle.encode_bits(q, item, level, tie)
    for n in range(6):
        for d in range(D):
            votes = sum(int(item[f, d]) != int(level[q[n, f], d]) for f in range(F))
            want = 1 if 2 * votes > F else 0 if 2 * votes < F else int(tie[d])
            assert hv[n, d] == want, (n, d)


def test_encode_tie_vector_equals_extra_vote_when_F_even():
    # With F even, breaking ties by T is the same as letting T cast an (F+1)-th vote.
    rng = np.random.default_rng(3)
    D, F, L = 96, 6, 4
    item, level, tie = rand_bits(rng, F, D), rand_bits(rng, L, D), rand_bits(rng, D)
    q = rng.integers(0, L, size=(20, F)).astype(np.int32)
    hv = oracle.encode_bits(q, item, level, tie)
    level_x = np.vstack([level, np.zeros((1, D), np.uint8)])      # extra level: all zero
    item_x = np.vstack([item, tie[None, :]])                      # extra feature: ID = T
    q_x = np.hstack([q, np.full((20, 1), L, np.int32)])
    hv_x = oracle.encode_bits(q_x, item_x, level_x, rand_bits(rng, D))  # odd F: tie unused
    assert np.array_equal(hv, hv_x)


def test_encode_complementing_levels_complements_output_for_odd_F():
    rng = np.random.default_rng(4)
    D, F, L = 50, 7, 3
    item, level, tie = rand_bits(rng, F, D), rand_bits(rng, L, D), rand_bits(rng, D)
    q = rng.integers(0, L, size=(10, F)).astype(np.int32)
    a = oracle.encode_bits(q, item, level, tie)
    b = oracle.encode_bits(q, item, level ^ 1, tie)
    assert np.array_equal(a ^ 1, b)


def test_encode_packed_path_pad_bits_and_structure_with_linear_levels():
    # End to end through packed tables (config 1 shapes, D cut to a non-multiple of 32).
    wl = make_workload(1, D=1000, n_train=64)
    x, _ = wl.train(64)
    hv = oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)
    assert hv.shape == (64, 32) and hv.dtype == np.uint32
    assert np.all(hv[:, -1] >> (1000 - 31 * 32) == 0)                 # pad bits zero
    # Linear-scaling level table: Hamming(V_i, V_j) = |i-j| * b exactly (closed form).
    lv = oracle.unpack(wl.level, wl.D).astype(int)
    b = wl.D // (2 * (wl.L - 1))
    for i, j in itertools.combinations(range(wl.L), 2):
        assert np.sum(lv[i] != lv[j]) == (j - i) * b
    # Dimensions no level ever flips carry the same bound bits for every sample, so the
    # encoded bit there cannot depend on the sample.
    never = np.all(lv == lv[0], axis=0)
    assert never.sum() == wl.D - (wl.L - 1) * b
    bits = oracle.unpack(hv, wl.D)
    assert np.all(bits[:, never] == bits[0, never])
    assert not np.all(bits[:, ~never] == bits[0, ~never])


def test_encode_vs_numpy_column_sums():
    wl = make_workload(2, D=257, F=33, L=8, n_train=40)
    x, _ = wl.train(40)
    hv = oracle.unpack(oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale), wl.D)
    q = oracle.quantize(x, wl.L, wl.lo, wl.scale)
    it, lv, tie = (oracle.unpack(a, wl.D) for a in (wl.item, wl.level, wl.tie))
    for n in range(40):
        cnt = (it ^ lv[q[n]]).sum(axis=0)                              # library reduction
        want = np.where(2 * cnt > wl.F, 1, np.where(2 * cnt < wl.F, 0, tie))
        assert np.array_equal(hv[n], want)


# ----------------------------------------------------------------- classical training
def _rand_hv(rng, N, D):
    return pack_bits_lsb(rand_bits(rng, N, D))


def test_classical_column_and_row_sum_identities():
    rng = np.random.default_rng(5)
    N, D, C = 300, 203, 4
    hv, y = _rand_hv(rng, N, D), rng.integers(0, C, N).astype(np.int32)
    acc, cn = oracle.train_classical(hv, y, D, C)
    bits = np.unpackbits(hv.view(np.uint8), axis=1, bitorder="little")[:, :D].astype(np.int64)
    assert np.array_equal(cn, np.bincount(y, minlength=C))
    assert np.array_equal(acc.sum(axis=0), bits.sum(axis=0))          # over classes = all rows
    for c in range(C):
        assert acc[c].sum() == bits[y == c].sum()                     # total popcount of class
        assert np.array_equal(acc[c], bits[y == c].sum(axis=0))


def test_classical_chunking_order_and_repeat():
    rng = np.random.default_rng(6)
    N, D, C = 120, 64, 3
    hv, y = _rand_hv(rng, N, D), rng.integers(0, C, N).astype(np.int32)
    tie = _rand_hv(rng, 1, D)[0]
    acc, cn = oracle.train_classical(hv, y, D, C)
    a1, n1 = oracle.train_classical(hv[:50], y[:50], D, C)
    a2, n2 = oracle.train_classical(hv[50:], y[50:], D, C, a1, n1)
    assert np.array_equal(a2, acc) and np.array_equal(n2, cn)         # chunks compose
    p = rng.permutation(N)
    ap, _ = oracle.train_classical(hv[p], y[p], D, C)
    assert np.array_equal(ap, acc)                                     # order-free
    ad, nd = oracle.train_classical(hv, y, D, C, acc, cn)
    assert np.array_equal(ad, 2 * acc) and np.array_equal(nd, 2 * cn)  # twice the data
    assert np.array_equal(oracle.binarize_classical(ad, nd, tie),
                          oracle.binarize_classical(acc, cn, tie))     # same class vectors


def test_classical_majority_special_cases():
    rng = np.random.default_rng(7)
    D = 90
    tie = _rand_hv(rng, 1, D)[0]
    hv = _rand_hv(rng, 6, D)
    # one sample per class -> class vector is that sample
    acc, cn = oracle.train_classical(hv[:3], np.arange(3, dtype=np.int32), D, 3)
    assert np.array_equal(oracle.binarize_classical(acc, cn, tie), hv[:3])
    # three samples -> bitwise majority; two samples -> agree or tie vector; empty -> tie
    y = np.array([0, 0, 0, 1, 1, 7], dtype=np.int32)                  # label 7 is out of range
    acc, cn = oracle.train_classical(hv, y, D, 3)
    assert cn.tolist() == [3, 2, 0]
    m = oracle.binarize_classical(acc, cn, tie)
    a, b, c = hv[0], hv[1], hv[2]
    assert np.array_equal(m[0], (a & b) | (a & c) | (b & c))
    assert np.array_equal(m[1], (hv[3] & hv[4]) | ((hv[3] ^ hv[4]) & tie))
    assert np.array_equal(m[2], tie)


# ---------------------------------------------------------------------------- search
def test_search_basic_identities():
    rng = np.random.default_rng(8)
    D, N = 333, 40
    x = _rand_hv(rng, N, D)
    mask = pack_bits_lsb(np.ones(D, dtype=np.uint8))
    dist, pred = oracle.search(x, x, D)
    assert np.all(np.diag(dist) == 0) and np.array_equal(dist, dist.T)      # d(x,x)=0, symmetric
    assert np.array_equal(pred, np.arange(N))
    dc, _ = oracle.search(x, (~x) & mask, D)
    assert np.all(np.diag(dc) == D)                                          # complement: D
    pc = np.array([bin(int(v)).count("1") for v in x.ravel()]).reshape(N, -1).sum(axis=1)
    assert np.all((dist - (pc[:, None] + pc[None, :])) % 2 == 0)             # parity rule
    assert dist.max() <= D
    for i, j, k in itertools.product(range(6), repeat=3):
        assert dist[i, k] <= dist[i, j] + dist[j, k]                         # triangle
    # library special case: count of unequal unpacked bits
    ub = np.unpackbits(x.view(np.uint8), axis=1, bitorder="little")[:, :D]
    assert np.array_equal(dist, (ub[:, None, :] != ub[None, :, :]).sum(axis=2))


def test_search_argmin_tie_goes_to_lowest_class():
    D = 40
    q = pack_bits_lsb(np.zeros((1, D), np.uint8))
    cls = np.zeros((4, D), np.uint8)
    cls[0, :5] = 1
    cls[1, 5:8] = 1     # distance 3
    cls[2, 30:33] = 1   # distance 3 as well
    cls[3, :] = 1
    dist, pred = oracle.search(q, pack_bits_lsb(cls), D)
    assert dist.tolist() == [[5, 3, 3, 40]] and pred.tolist() == [1]


def test_search_distance_to_noisy_copy_is_number_of_flips():
    rng = np.random.default_rng(9)
    D = 500
    base = rand_bits(rng, 3, D)
    qs, want = [], []
    for c, k in [(0, 0), (1, 17), (2, 249), (1, 1)]:
        v = base[c].copy()
        v[rng.choice(D, k, replace=False)] ^= 1
        qs.append(v)
        want.append((c, k))
    dist, pred = oracle.search(pack_bits_lsb(np.array(qs)), pack_bits_lsb(base), D)
    for i, (c, k) in enumerate(want):
        assert dist[i, c] == k and pred[i] == c


# -------------------------------------------------------------------- online training
def _load_online_case():
    hs, ys, after = [], [], []
    for line in open(os.path.join(GOLDEN, "online_hand_case.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "h":
            hs.append(bits_of(t[1]))
            ys.append(int(t[2]))
        elif t[0] == "after":
            after.append((int(t[1]), int(t[3]), [float(v) for v in t[5:9]], [float(v) for v in t[10:14]]))
    return pack_bits_lsb(np.array(hs)), np.array(ys, dtype=np.int32), after


def test_online_hand_case_from_golden_file():
    hv, y, after = _load_online_case()
    for k, pred_k, m0, m1 in after:
        acc, pred, _ = oracle.train_online(hv[:k], y[:k], 4, 2, epochs=1, lr=1.0, log=True)
        assert pred[k - 1] == pred_k
        np.testing.assert_allclose(acc, np.array([m0, m1]), rtol=0, atol=2e-7)


def test_online_learning_rate_scales_only_the_subtraction():
    hv, y, _ = _load_online_case()
    # lr = 0: step 2 mispredicts but class 0 must stay untouched; class 1 still gets the sample
    acc = oracle.train_online(hv[:2], y[:2], 4, 2, lr=0.0)
    assert acc.tolist() == [[1, 1, -1, -1], [1, -1, 1, -1]]
    acc = oracle.train_online(hv[:2], y[:2], 4, 2, lr=0.25)
    assert acc.tolist() == [[0.75, 1.25, -1.25, -0.75], [1, -1, 1, -1]]


def test_online_first_step_repeat_and_complement():
    rng = np.random.default_rng(10)
    D, C = 10000, 3                                   # sqrt(D) = 100 exactly
    h = rand_bits(rng, 1, D)
    s = 2.0 * h[0] - 1.0
    hv = pack_bits_lsb(h)
    mask = pack_bits_lsb(np.ones(D, np.uint8))
    for y in range(C):
        lab = np.array([y], dtype=np.int32)
        acc = oracle.train_online(hv, lab, D, C)
        want = np.zeros((C, D), np.float32)
        want[y] = s
        # first sample of an all-zero model: cosine 0, weight 1 -> acc[y] = s exactly; the
        # all-zero model predicts class 0, which is "wrong" for y > 0 but subtracts from a
        # zero row with weight lr*(1-0): acc[0] = -s.
        if y != 0:
            want[0] = -s
        assert np.array_equal(acc, want)
    lab = np.array([0], dtype=np.int32)
    acc1 = oracle.train_online(hv, lab, D, C)
    acc2, pred, margin = oracle.train_online(hv, lab, D, C, acc=acc1, log=True)
    assert np.array_equal(acc2, acc1) and pred[0] == 0 and margin[0] == 1.0   # cos = 1, weight 0
    acc3 = oracle.train_online((~hv) & mask, lab, D, C, acc=acc1)
    # cos_0 = -1 -> weight 2: acc[0] = s - 2s = -s; the zero rows (cosine 0) now beat
    # class 0, the lowest of them (class 1) is the wrong prediction and loses 1 * (-s).
    assert np.array_equal(acc3[0], -s) and np.array_equal(acc3[1], s) and not acc3[2].any()
    # epochs = 2 on one sample equals two calls
    assert np.array_equal(oracle.train_online(hv, lab, D, C, epochs=2), acc2)


def test_online_single_class_never_subtracts():
    rng = np.random.default_rng(11)
    D, N = 64, 30
    hv = _rand_hv(rng, N, D)
    y = np.zeros(N, dtype=np.int32)
    a = oracle.train_online(hv, y, D, 1, epochs=2, lr=0.0)
    b = oracle.train_online(hv, y, D, 1, epochs=2, lr=1000.0)
    assert np.array_equal(a, b)


def test_online_matches_independent_float64_rederivation_on_small_cases():
    # Cross-check (not a pin): the same steps written with numpy on +-1 vectors.
    rng = np.random.default_rng(12)
    D, C, N = 48, 4, 60
    h = rand_bits(rng, N, D)
    y = rng.integers(0, C, N).astype(np.int32)
    acc, pred, _ = oracle.train_online(pack_bits_lsb(h), y, D, C, epochs=2, lr=0.7, log=True)
    m = np.zeros((C, D), np.float32)
    k = 0
    for _ in range(2):
        for n in range(N):
            s = (2.0 * h[n] - 1.0)
            md = m.astype(np.float64)
            nrm = np.sqrt((md * md).sum(axis=1))
            cos = np.where(nrm == 0, 0.0, (md @ s) / np.where(nrm == 0, 1, nrm * np.sqrt(D)))
            p = int(np.argmax(cos))
            assert p == pred[k]
            k += 1
            wy = np.float32(1.0 - cos[y[n]])
            wp = np.float32(np.float32(0.7).astype(np.float64) * (1.0 - cos[p]))
            m[y[n]] = m[y[n]] + wy * s.astype(np.float32)
            if p != y[n]:
                m[p] = m[p] - wp * s.astype(np.float32)
    np.testing.assert_allclose(acc, m, rtol=1e-6, atol=1e-6)


def test_online_binarise_sign_and_tie():
    D = 6
    tie = pack_bits_lsb(bits_of("010101"))
    acc = np.array([[1.5, -2.0, 0.0, 0.0, -0.0, 1e-30],
                    [0, 0, 0, 0, 0, 0]], dtype=np.float32)
    m = oracle.unpack(oracle.binarize_online(acc, tie), D)
    assert m.tolist() == [[1, 0, 0, 1, 0, 1], [0, 1, 0, 1, 0, 1]]


# ------------------------------------------------------------------------ end to end
def test_config1_end_to_end_is_accurate_on_separated_clusters():
    wl = make_workload(1, n_train=600, n_test=200)
    xt, yt = wl.train()
    xs, ys = wl.test()
    enc = lambda x: oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)
    ht, hs = enc(xt), enc(xs)
    acc, cn = oracle.train_classical(ht, yt, wl.D, wl.C)
    m = oracle.binarize_classical(acc, cn, wl.tie)
    _, pred = oracle.search(hs, m, wl.D)
    assert (pred == ys).mean() > 0.9          # smoke level only; the paper's accuracies are in a lost figure
    acc_o = oracle.train_online(ht, yt, wl.D, wl.C, epochs=2)
    _, pred_o = oracle.search(hs, oracle.binarize_online(acc_o, wl.tie), wl.D)
    assert (pred_o == ys).mean() > 0.9


# ------------------------------------------------------- batched online training (Sec. VI-D2)
def test_online_batched_hand_case_from_golden_file():
    hs, ys, after, batch = [], [], [], None
    for line in open(os.path.join(GOLDEN, "online_batched_hand_case.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "h":
            hs.append(bits_of(t[1]))
            ys.append(int(t[2]))
        elif t[0] == "batch":
            batch = int(t[1])
        elif t[0] == "after":
            after.append((int(t[1]), [float(v) for v in t[3:7]], [float(v) for v in t[8:12]]))
    hv, y = pack_bits_lsb(np.array(hs)), np.array(ys, dtype=np.int32)
    for k, m0, m1 in after:
        acc = oracle.train_online_batched(hv[:k], y[:k], 4, 2, batch)
        np.testing.assert_allclose(acc, np.array([m0, m1]), rtol=0, atol=2e-7)


def test_online_batched_whole_set_from_zero_model_closed_form():
    # One batch over everything, zero start: every cosine is 0, every prediction is class 0, all
    # weights are 1 (lr for the subtraction): acc[c] = sum of s over class c, and class 0
    # additionally loses lr * (sum of s over all other classes).  Small integers: exact.
    rng = np.random.default_rng(20)
    D, C, N, lr = 96, 4, 50, 0.5
    h = rand_bits(rng, N, D)
    y = rng.integers(0, C, N).astype(np.int32)
    s = 2.0 * h - 1.0
    acc = oracle.train_online_batched(pack_bits_lsb(h), y, D, C, batch=N, lr=lr)
    want = np.zeros((C, D))
    for c in range(C):
        want[c] = s[y == c].sum(axis=0)
    want[0] -= lr * s[y != 0].sum(axis=0)
    assert np.array_equal(acc, want.astype(np.float32))
    # a batch larger than the set is the same thing; two epochs = two such batches
    assert np.array_equal(oracle.train_online_batched(pack_bits_lsb(h), y, D, C, batch=10 * N, lr=lr), acc)


def test_online_batched_with_batch_one_is_plain_online_training():
    rng = np.random.default_rng(21)
    D, C, N = 64, 3, 40
    hv = _rand_hv(rng, N, D)
    y = rng.integers(0, C, N).astype(np.int32)
    a = oracle.train_online(hv, y, D, C, epochs=2, lr=0.8)
    b = oracle.train_online_batched(hv, y, D, C, batch=1, epochs=2, lr=0.8)
    np.testing.assert_allclose(b, a, rtol=1e-6, atol=1e-6)


def test_online_batched_order_inside_a_batch_does_not_matter_but_batches_do():
    rng = np.random.default_rng(22)
    D, C, N, B = 80, 3, 24, 8
    hv = _rand_hv(rng, N, D)
    y = rng.integers(0, C, N).astype(np.int32)
    a = oracle.train_online_batched(hv, y, D, C, batch=B)
    p = np.concatenate([b0 + rng.permutation(B) for b0 in range(0, N, B)])     # shuffle inside batches
    b = oracle.train_online_batched(hv[p], y[p], D, C, batch=B)
    np.testing.assert_allclose(b, a, rtol=1e-6, atol=1e-6)
    c = oracle.train_online_batched(hv, y, D, C, batch=N)                      # different batching
    assert not np.allclose(c, a)


# ------------------------------------- stand-alone summations (Sec. IV-B2), cosine inference
def test_hsum_and_vsum_are_row_and_column_sums():
    rng = np.random.default_rng(30)
    N, D = 37, 203
    bits = rand_bits(rng, N, D)
    hv = pack_bits_lsb(bits)
    assert np.array_equal(oracle.hsum(hv, D), bits.sum(axis=1))
    assert np.array_equal(oracle.vsum(hv, D), bits.sum(axis=0))
    # the two agree on the grand total, and an all-ones / all-zero row counts D / 0
    assert oracle.hsum(hv, D).sum() == oracle.vsum(hv, D).sum()
    ends = pack_bits_lsb(np.stack([np.ones(D, np.uint8), np.zeros(D, np.uint8)]))
    assert oracle.hsum(ends, D).tolist() == [D, 0]
    assert oracle.vsum(ends, D).tolist() == [1] * D


def test_hsum_of_xor_is_the_hamming_distance_and_vsum_is_the_class_accumulator():
    rng = np.random.default_rng(31)
    N, D, C = 25, 130, 3
    q, cls = _rand_hv(rng, N, D), _rand_hv(rng, C, D)
    dist, _ = oracle.search(q, cls, D)
    for c in range(C):
        assert np.array_equal(oracle.hsum(q ^ cls[c], D), dist[:, c])
    y = rng.integers(0, C, N).astype(np.int32)
    acc, _ = oracle.train_classical(q, y, D, C)
    for c in range(C):
        assert np.array_equal(oracle.vsum(q[y == c], D), acc[c])


def test_cosine_inference_closed_forms():
    rng = np.random.default_rng(32)
    N, D, C = 20, 96, 4
    bits = rand_bits(rng, N, D)
    hv = pack_bits_lsb(bits)
    s = 2.0 * bits - 1.0
    # rows that are themselves +-1 vectors: cosine = 1 - 2 hamming / D (both sides exact in fp64)
    cbits = rand_bits(rng, C, D)
    m = (2.0 * cbits - 1.0).astype(np.float32)
    cosv, pred = oracle.search_cosine(hv, m, D)
    dist, hpred = oracle.search(hv, pack_bits_lsb(cbits), D)
    np.testing.assert_allclose(cosv, 1.0 - 2.0 * dist / D, rtol=0, atol=1e-15)
    assert np.array_equal(pred, hpred)
    # a sample against itself / its complement / a zero row; scaling a row changes nothing
    m2 = np.stack([s[0], -s[0], np.zeros(D), 7.5 * s[0]]).astype(np.float32)
    c2, p2 = oracle.search_cosine(hv[:1], m2, D)
    np.testing.assert_allclose(c2[0], [1.0, -1.0, 0.0, 1.0], rtol=0, atol=1e-15)
    assert p2[0] == 0                                        # the lowest of the equal best
    # general rows: the definition, written with numpy
    m3 = rng.standard_normal((C, D)).astype(np.float32)
    c3, p3 = oracle.search_cosine(hv, m3, D)
    want = (s @ m3.astype(np.float64).T) / (np.linalg.norm(m3.astype(np.float64), axis=1) * np.sqrt(D))
    np.testing.assert_allclose(c3, want, rtol=1e-12, atol=1e-15)
    assert np.array_equal(p3, want.argmax(axis=1))


def test_cosine_scores_are_the_ones_online_training_uses():
    # one online step from a trained model: the weights it applies follow from search_cosine
    rng = np.random.default_rng(33)
    D, C, N = 64, 3, 30
    hv = _rand_hv(rng, N, D)
    y = rng.integers(0, C, N).astype(np.int32)
    acc = oracle.train_online(hv, y, D, C)
    cosv, pred = oracle.search_cosine(hv[:1], acc, D)
    nxt = oracle.train_online(hv[:1], y[:1], D, C, acc=acc)
    s = 2.0 * oracle.unpack(hv[:1], D)[0] - 1.0
    want = acc.astype(np.float64).copy()
    want[y[0]] += np.float32(1.0 - cosv[0, y[0]]) * s
    if pred[0] != y[0]:
        want[pred[0]] -= np.float32(1.0 - cosv[0, pred[0]]) * s
    np.testing.assert_allclose(nxt, want.astype(np.float32), rtol=1e-6, atol=1e-6)


def test_online_exact_tie_between_proportional_rows_goes_to_the_lowest_class():
    """Two class rows that are exact multiples of one another score every sample identically: in
    exact arithmetic the two best cosines tie.  With a power-of-two factor the fp64 sums are
    scaled exactly, the oracle's margin is exactly 0 and the lowest class wins (reading Q12); the
    step then subtracts from class 0 because the label is 1.  With the factor 3 the tie holds in
    exact arithmetic only: the logged margin stays within rounding of 0 (far below the 1e-9 below
    which parity tests do not compare trajectories), whichever way rounding decides it."""
    D = 16
    rng = np.random.default_rng(5)
    s = rng.integers(0, 2, D).astype(np.uint8)
    t = s.copy()
    t[:5] ^= 1                                     # a sample that is neither s nor its complement
    row = (2.0 * s - 1.0).astype(np.float32)
    hv = pack_bits_lsb(t[None, :])
    y = np.array([1], dtype=np.int32)
    acc0 = np.stack([row, 2.0 * row]).astype(np.float32)
    acc, pred, margin = oracle.train_online(hv, y, D, 2, 1, 1.0, acc=acc0, log=True)
    assert margin[0] == 0.0 and pred[0] == 0
    cos = float(np.dot(row, 2.0 * t - 1.0)) / (np.sqrt(float(D)) * np.sqrt(float(D)))
    w = np.float32(1.0 - cos)
    assert np.array_equal(acc[1], (2.0 * row + w * (2.0 * t - 1.0)).astype(np.float32))
    assert np.array_equal(acc[0], (row - w * (2.0 * t - 1.0)).astype(np.float32))
    acc3 = np.stack([row, 3.0 * row]).astype(np.float32)
    _, _, margin3 = oracle.train_online(hv, y, D, 2, 1, 1.0, acc=acc3, log=True)
    assert abs(margin3[0]) < 1e-12
