"""Pins for the oracle's density routing (Sec. 3.4) and dense copy: the break-even of the cost model
(Eq. (1)/(2): X(rho) = 1/(3 rho) crosses 1 at rho = 1/3; with 2-byte indices at rho = 1/2), slot order,
capacity, and the round trip of a mixed sparse / dense update."""
import numpy as np
import pytest

import oracle


def test_break_even_density_follows_the_cost_model():
    be, total, cap = 3000, 9000, 3000
    for bpp, frac in ((6, 1 / 3), (4, 1 / 2)):
        edge = int(np.ceil(2 * be / bpp))                    # smallest count whose payload is not smaller than dense
        assert abs(edge / be - frac) < 1e-3                  # X = b_v / (rho (b_i + b_v)) = 1
        counts = np.array([edge - 1, edge, edge + 1], np.uint32)
        slot, sc, db, nd, dropped = oracle.route(counts, be, total, cap, bytes_per_pair=bpp)
        assert slot.tolist() == [-1, 0, 1] and nd == 2 and dropped == 0
        assert sc.tolist() == [edge - 1, 0, 0] and db[:2].tolist() == [1, 2]
        # brute force: payload bytes against dense bytes
        for c in range(0, be + 1, 7):
            s1 = oracle.route(np.array([c], np.uint32), be, be, cap, bytes_per_pair=bpp)[0][0]
            assert (s1 == 0) == (c > 0 and c * bpp >= 2 * be)


def test_overflowing_and_short_buckets():
    be, total, cap = 100, 560, 50
    counts = np.array([0, 10, 34, 33, 1000, 5, 0], np.uint32)[:6]
    slot, sc, db, nd, dropped = oracle.route(counts, be, total, cap)
    assert slot.tolist() == [-1, -1, 0, -1, 1, -1]           # 34*6 >= 200; 1000 > cap; last bucket has 60 elements
    assert sc.tolist() == [0, 10, 0, 33, 0, 5] and nd == 2
    # a short last bucket goes dense earlier: 20*6 = 120 >= 2*60
    slot2 = oracle.route(np.array([0, 0, 0, 0, 0, 20], np.uint32), be, total, cap)[0]
    assert slot2.tolist() == [-1] * 5 + [0]
    # not enough dense slots: the surplus stays sparse, truncated, and is reported
    slot3, sc3, db3, nd3, dropped3 = oracle.route(counts, be, total, cap, max_dense=1)
    assert slot3.tolist() == [-1, -1, 0, -1, -1, -1] and nd3 == 1 and dropped3 == 1 and sc3[4] == cap


def test_mixed_sparse_and_dense_round_trip():
    rng = np.random.default_rng(4)
    numel = [5000, 300, 300, 12000, 77]                      # two small "adapter-like" tensors that change everywhere
    be = 2048
    olds = [rng.integers(0, 1 << 16, size=m, dtype=np.uint16) for m in numel]
    news = [o.copy() for o in olds]
    for k, w in enumerate(news):
        p = 1.0 if k in (1, 2) else 0.01
        m = rng.random(w.size) < p
        w[m] ^= 0x11
    total = sum(numel)
    cap = 400
    I, V, c, _ = oracle.extract_multi([o.copy() for o in olds], news, numel, be, cap=cap)
    slot, sc, db, nd, dropped = oracle.route(c, be, total, cap)
    assert nd >= 1 and dropped == 0
    dense = np.zeros(nd * be, np.uint16)
    oracle.copy_dense_multi(news, numel, be, db, nd, dense, pack=True)
    # the dense body of a bucket is exactly that slice of the packed new weights
    packed = np.concatenate(news)
    for s in range(nd):
        b = db[s]
        want = packed[b * be:(b + 1) * be]
        assert np.array_equal(dense[s * be:s * be + want.size], want)
    roll = [o.copy() for o in olds]
    oracle.apply_multi(roll, numel, be, I, V, sc)             # sparse buckets only
    oracle.copy_dense_multi(roll, numel, be, db, nd, dense, pack=False)
    assert all(np.array_equal(r, w) for r, w in zip(roll, news))
    # without routing the overflowing buckets would have been truncated
    roll2 = [o.copy() for o in olds]
    oracle.apply_multi(roll2, numel, be, I, V, c)
    assert (c > cap).any() and not all(np.array_equal(r, w) for r, w in zip(roll2, news))
