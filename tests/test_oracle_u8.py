"""Pins for the one-byte (FP8 synchronisation precision, Sec. 2.1) functions of the CPU oracle.

Alg. 1-3 do not depend on the width of an element, so the pins are those of the 16-bit functions:
brute force over every change mask of tiny tensors, a Python loop, numpy's flatnonzero / fancy indexing,
the round trip, identical -> empty, all-changed -> dense, capacity clipping, bad indices.  One pin is
specific to this width: byte patterns widened to 16 bits must give, through the separately written 16-bit
functions, the same indices and counts and the widened values.
"""
import itertools

import numpy as np
import pytest

import oracle


def rnd_u8(rng, n):
    return rng.integers(0, 256, size=n, dtype=np.uint8)


def flip(a, idx, rng):
    b = a.copy()
    delta = rng.integers(1, 256, size=len(idx), dtype=np.uint32)
    b[idx] = ((a[idx].astype(np.uint32) + delta) & 0xFF).astype(np.uint8)
    assert np.all(b[idx] != a[idx])
    return b


def split(rng, n, parts):
    cuts = np.sort(rng.integers(0, n + 1, size=parts - 1))
    return np.diff(np.concatenate([[0], cuts, [n]])).astype(int).tolist()


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 10])
def test_every_mask_every_bucket_size(n):
    rng = np.random.default_rng(100 + n)
    base = rnd_u8(rng, n)
    for bits in itertools.product([0, 1], repeat=n):
        pos = [i for i in range(n) if bits[i]]
        new = flip(base, np.array(pos, dtype=np.int64), rng) if pos else base.copy()
        for be in range(1, n + 2):
            old = base.copy()
            I, V, counts, ovf = oracle.extract_u8(old, new, be)
            nb = -(-n // be)
            assert counts.shape == (nb,) and ovf == 0 and V.dtype == np.uint8
            for b in range(nb):
                want = [i for i in pos if b * be <= i < (b + 1) * be]
                assert counts[b] == len(want)
                assert I[b, :len(want)].tolist() == want
                assert V[b, :len(want)].tolist() == [int(new[i]) for i in want]
            assert np.array_equal(old, new)
            # the list form on the same data cut into two tensors: index = packed position mod be
            for cut in range(n + 1):
                olds = [base[:cut].copy(), base[cut:].copy()]
                I2, V2, c2, _ = oracle.extract_multi_u8(olds, [new[:cut].copy(), new[cut:].copy()], [cut, n - cut], be)
                assert np.array_equal(c2, counts) and np.array_equal(V2, V)
                for b in range(nb):
                    assert (I2[b, :counts[b]] + b * be).tolist() == I[b, :counts[b]].tolist()
                assert np.array_equal(np.concatenate(olds), new)


@pytest.mark.parametrize("n,be", [(1000, 64), (4097, 1000), (70001, 8192), (65536, 65536)])
def test_against_numpy(n, be):
    rng = np.random.default_rng(n)
    old = rnd_u8(rng, n)
    pos = np.flatnonzero(rng.random(n) < 0.03)
    new = flip(old, pos, rng)
    snap = old.copy()
    I, V, counts, ovf = oracle.extract_u8(snap, new, be)
    changed = np.flatnonzero(old != new)                     # numpy's statement of the same definition
    assert np.array_equal(changed, pos) and ovf == 0
    assert int(counts.sum()) == changed.size
    flatI = np.concatenate([I[b, :counts[b]] for b in range(counts.size)])
    flatV = np.concatenate([V[b, :counts[b]] for b in range(counts.size)])
    assert np.array_equal(flatI, changed) and np.array_equal(flatV, new[changed])
    assert np.array_equal(np.bincount(changed // be, minlength=counts.size), counts)
    assert np.array_equal(snap, new)
    roll = old.copy()
    assert oracle.apply_u8(roll, be, I, V, counts) == oracle.OK
    assert np.array_equal(roll, new)
    want = old.copy(); want[changed] = new[changed]          # fancy-index scatter
    assert np.array_equal(roll, want)
    # a second extract against the refreshed snapshot is empty
    _, _, c2, _ = oracle.extract_u8(snap, new, be)
    assert not c2.any()


def test_identical_empty_and_all_changed_dense():
    rng = np.random.default_rng(5)
    a = rnd_u8(rng, 5000)
    I, V, counts, _ = oracle.extract_u8(a.copy(), a.copy(), 1024)
    assert not counts.any() and (I == -1).all() and (V == 0xFF).all()
    b = (a ^ 0x80).astype(np.uint8)
    I, V, counts, _ = oracle.extract_u8(a.copy(), b, 1024)
    assert counts.tolist() == [1024, 1024, 1024, 1024, 904]
    assert np.array_equal(np.concatenate([I[k, :counts[k]] for k in range(5)]), np.arange(5000))
    assert np.array_equal(np.concatenate([V[k, :counts[k]] for k in range(5)]), b)


def test_widened_patterns_agree_with_the_16_bit_functions():
    rng = np.random.default_rng(6)
    numel = [1, 777, 4096, 3, 12345]
    olds = [rnd_u8(rng, m) for m in numel]
    news = [flip(o, np.flatnonzero(rng.random(o.size) < 0.05), rng) for o in olds]
    be = 3000
    I8, V8, c8, _ = oracle.extract_multi_u8([o.copy() for o in olds], news, numel, be)
    wide = lambda xs: [x.astype(np.uint16) * 257 for x in xs]            # byte b -> pattern 0xbbbb, injective
    I16, V16, c16, _ = oracle.extract_multi(wide(olds), wide(news), numel, be)
    assert np.array_equal(c8, c16)
    for b in range(c8.size):
        assert np.array_equal(I8[b, :c8[b]], I16[b, :c8[b]])
        assert np.array_equal(V8[b, :c8[b]].astype(np.uint16) * 257, V16[b, :c8[b]])


def test_list_round_trip_and_python_walk():
    rng = np.random.default_rng(7)
    numel = split(rng, 50000, 9)
    olds = [rnd_u8(rng, m) for m in numel]
    news = [flip(o, np.flatnonzero(rng.random(o.size) < 0.02), rng) for o in olds]
    be = 4099
    snaps = [o.copy() for o in olds]
    I, V, counts, ovf = oracle.extract_multi_u8(snaps, news, numel, be)
    assert ovf == 0
    flat_old, flat_new = np.concatenate(olds), np.concatenate(news)
    changed = np.flatnonzero(flat_old != flat_new)
    assert np.array_equal(np.bincount(changed // be, minlength=counts.size), counts)
    for b in range(counts.size):
        sel = changed[(changed // be) == b]
        assert np.array_equal(I[b, :counts[b]], sel - b * be) and np.array_equal(V[b, :counts[b]], flat_new[sel])
    for s, w in zip(snaps, news):
        assert np.array_equal(s, w)
    rolls = [o.copy() for o in olds]
    assert oracle.apply_multi_u8(rolls, numel, be, I, V, counts) == oracle.OK
    for r, w in zip(rolls, news):
        assert np.array_equal(r, w)


def test_refresh_off_capacity_and_bad_index():
    rng = np.random.default_rng(8)
    old = rnd_u8(rng, 3000)
    new = flip(old, np.arange(0, 3000, 3), rng)
    keep = old.copy()
    I, V, counts, ovf = oracle.extract_u8(keep, new, 1000, cap=100, refresh=False)
    assert np.array_equal(keep, old)                                      # snapshot left alone
    assert ovf == 3 and counts.tolist() == [334, 333, 333]                # true counts above cap
    assert I[0].tolist() == list(range(0, 300, 3)) and (I[1] >= 1000).all()
    w = old.copy()
    assert oracle.apply_u8(w, 1000, I, V, counts) == oracle.OK           # counts above cap read as cap
    assert np.array_equal(np.flatnonzero(w != old), np.concatenate([I[0], I[1], I[2]]))
    I[1, 5] = 999                                                         # belongs to bucket 0, stored in bucket 1
    w2 = old.copy()
    assert oracle.apply_u8(w2, 1000, I, V, counts) == oracle.BAD_INDEX
    assert w2[999] == old[999]
    with pytest.raises(ValueError):
        oracle.extract_u8(old.copy(), new, 0)
