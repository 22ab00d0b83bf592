"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle itself.

The oracle states Alg. 1's changed-index set (bitwise), Alg. 2's V = W[I] with sorted int32 I,
and Alg. 3's scatter, per fixed-size bucket.  None of the expected values below comes from the
oracle or from the GPU library: they are brute-force enumerations written out in Python, the
generator's own change mask, numpy's flatnonzero / fancy indexing, and the cost model of
Eq. (1)/(2) with the numbers the paper prints (tests/golden/payload_cost_model.txt).
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd_u16(rng, n):
    return rng.integers(0, 1 << 16, size=n, dtype=np.uint16)


def flip(a, idx, rng):
    """Return a copy of a whose elements at idx all differ bitwise from a."""
    b = a.copy()
    delta = rng.integers(1, 1 << 16, size=len(idx), dtype=np.uint32)
    b[idx] = ((a[idx].astype(np.uint32) + delta) & 0xFFFF).astype(np.uint16)
    assert np.all(b[idx] != a[idx])
    return b


# ---------------------------------------------------------------------------------------------
# brute force on tiny tensors: every change mask, every bucket size
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 10])
def test_every_mask_every_bucket_size(n):
    rng = np.random.default_rng(n)
    base = rnd_u16(rng, n)
    for bits in itertools.product([0, 1], repeat=n):
        pos = [i for i in range(n) if bits[i]]
        new = flip(base, np.array(pos, dtype=np.int64), rng) if pos else base.copy()
        for be in range(1, n + 2):
            old = base.copy()
            I, V, counts, ovf = oracle.extract(old, new, be)
            nb = -(-n // be)
            assert counts.shape == (nb,) and ovf == 0
            for b in range(nb):
                want = [i for i in pos if b * be <= i < (b + 1) * be]      # ascending by construction
                assert counts[b] == len(want)
                assert I[b, :len(want)].tolist() == want
                assert V[b, :len(want)].tolist() == [int(new[i]) for i in want]
            assert np.array_equal(old, new)                                  # snapshot refreshed


@pytest.mark.parametrize("n", [7, 9, 63, 64, 65, 255, 256, 257, 1000])
def test_counts_and_order_against_python_loop(n):
    rng = np.random.default_rng(1000 + n)
    for be in sorted({1, 2, 3, 7, 8, 64, n - 1, n, n + 1} - {0}):
        base = rnd_u16(rng, n)
        pos = np.flatnonzero(rng.random(n) < 0.3)
        new = flip(base, pos, rng)
        old = base.copy()
        I, V, counts, _ = oracle.extract(old, new, be)
        got = []
        for b in range(len(counts)):
            row = I[b, :counts[b]].tolist()
            assert all(x < y for x, y in zip(row, row[1:]))                  # strictly ascending
            assert all(b * be <= x < min(n, (b + 1) * be) for x in row)
            got += row
        assert got == pos.tolist()
        assert int(counts.sum()) == len(pos)


# ---------------------------------------------------------------------------------------------
# invariants the paper fixes (goal G1; the Sec. 4.2 bit-exact protocol)
# ---------------------------------------------------------------------------------------------

def test_round_trip_single_full_config0():
    wl = synth.workload(0)
    a = synth.WeightSet(wl, "cpu"); b = synth.WeightSet(wl, "cpu")
    synth.fill_base(a, 0)
    nchanged, masks = synth.make_update(b, a, 0, want_masks=True)
    old, new = a.to_numpy_u16()[0], b.to_numpy_u16()[0]
    roll = old.copy()
    I, V, counts, ovf = oracle.extract(old, new, wl.bucket_elems)
    assert ovf == 0 and counts.shape == (4,)
    # generator ground truth: every masked position was forced to differ, nothing else changed
    truth = np.flatnonzero(masks[0].numpy())
    got = np.concatenate([I[b_, :counts[b_]] for b_ in range(4)])
    assert np.array_equal(got, truth) and int(counts.sum()) == nchanged
    assert oracle.apply(roll, wl.bucket_elems, I, V, counts) == oracle.OK
    assert np.array_equal(roll, new)
    assert np.array_equal(old, new)
    # a repeated extract finds nothing
    I2, V2, c2, _ = oracle.extract(old, new, wl.bucket_elems)
    assert int(c2.sum()) == 0 and np.all(I2 == -1)


def test_identical_inputs_give_empty_payload():
    rng = np.random.default_rng(5)
    a = rnd_u16(rng, 5000)
    I, V, counts, _ = oracle.extract(a.copy(), a.copy(), 777)
    assert counts.tolist() == [0] * 7
    assert np.all(I == -1) and np.all(V == 0xFFFF)                          # slots untouched


def test_all_changed_gives_dense_payload():
    rng = np.random.default_rng(6)
    n, be = 5000, 777
    a = rnd_u16(rng, n)
    b = flip(a, np.arange(n), rng)
    I, V, counts, _ = oracle.extract(a.copy(), b, be)
    assert counts.tolist() == [777] * 6 + [5000 - 6 * 777]
    for k in range(7):
        lo, hi = k * be, min(n, (k + 1) * be)
        assert np.array_equal(I[k, :hi - lo], np.arange(lo, hi))
        assert np.array_equal(V[k, :hi - lo], b[lo:hi])


def test_comparison_is_on_bit_patterns():
    # +0 -> -0 is a change; a NaN keeping its pattern is not; a NaN changing payload is; Inf, subnormals
    old = np.array([0x0000, 0x7FC0, 0x7FC0, 0x7F80, 0x0001, 0x8000, 0x3F80], np.uint16)
    new = np.array([0x8000, 0x7FC0, 0x7FC1, 0xFF80, 0x0002, 0x8000, 0x3F80], np.uint16)
    I, V, counts, _ = oracle.extract(old.copy(), new, 100)
    assert counts.tolist() == [4]
    assert I[0, :4].tolist() == [0, 2, 3, 4]
    assert V[0, :4].tolist() == [0x8000, 0x7FC1, 0xFF80, 0x0002]


def test_values_are_the_new_ones_not_the_old():
    old = np.array([1, 2, 3, 4], np.uint16); new = np.array([1, 9, 3, 8], np.uint16)
    I, V, c, _ = oracle.extract(old.copy(), new, 4)
    assert V[0, :2].tolist() == [9, 8] and I[0, :2].tolist() == [1, 3]
    w = np.array([1, 2, 3, 4], np.uint16)
    oracle.apply(w, 4, I, V, c)
    assert w.tolist() == [1, 9, 3, 8]


def test_chain_of_updates_reproduces_final_weights():
    rng = np.random.default_rng(7)
    n, be = 30000, 4096
    snap = rnd_u16(rng, n); roll = snap.copy(); cur = snap.copy()
    for step in range(5):
        cur = flip(cur, np.flatnonzero(rng.random(n) < 0.01), rng)
        I, V, c, _ = oracle.extract(snap, cur, be)
        oracle.apply(roll, be, I, V, c)
        assert np.array_equal(roll, cur) and np.array_equal(snap, cur)


# ---------------------------------------------------------------------------------------------
# library reduction: numpy states the same definition in one line each
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n,be", [(100003, 4096), (65536, 65536), (65537, 65536), (12345, 100000)])
def test_matches_numpy_flatnonzero_and_fancy_indexing(n, be):
    rng = np.random.default_rng(n)
    old = rnd_u16(rng, n)
    new = flip(old, np.flatnonzero(rng.random(n) < 0.02), rng)
    ref_I = np.flatnonzero(old != new)
    ref_V = new[ref_I]
    I, V, counts, _ = oracle.extract(old.copy(), new, be)
    cat_I = np.concatenate([I[b, :counts[b]] for b in range(len(counts))])
    cat_V = np.concatenate([V[b, :counts[b]] for b in range(len(counts))])
    assert np.array_equal(cat_I, ref_I) and np.array_equal(cat_V, ref_V)
    assert np.array_equal(counts, np.bincount(ref_I // be, minlength=len(counts)))
    w = old.copy(); w2 = old.copy()
    w2[ref_I] = ref_V
    oracle.apply(w, be, I, V, counts)
    assert np.array_equal(w, w2) and np.array_equal(w, new)


# ---------------------------------------------------------------------------------------------
# closed form: Eq. (1) / Eq. (2) and the numbers the paper prints
# ---------------------------------------------------------------------------------------------

def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "payload_cost_model.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_payload_bytes_follow_cost_model_with_paper_numbers():
    rng = np.random.default_rng(11)
    n, be = 1 << 20, 1 << 18
    base = rnd_u16(rng, n)
    for row in _golden_rows():
        if len(row) == 6:                     # label full_GB rho sparse_GB tol src
            full_gb, rho, want_gb, tol = map(float, row[1:5])
            k = round(rho * n)
            pos = np.sort(rng.choice(n, size=k, replace=False))
            I, V, counts, _ = oracle.extract(base.copy(), flip(base, pos, rng), be)
            payload = 4 * int(counts.sum()) + 2 * int(counts.sum())           # int32 + BF16 per pair
            frac = payload / (2 * n)                                            # of the dense BF16 bytes
            assert abs(full_gb * frac - want_gb) < tol + full_gb * 3 / n
        elif len(row) == 5:                   # label rho X tol src
            rho, want_x, tol = map(float, row[1:4])
            k = round(rho * n)
            pos = np.sort(rng.choice(n, size=k, replace=False))
            I, V, counts, _ = oracle.extract(base.copy(), flip(base, pos, rng), be)
            x = (2 * n) / (6 * int(counts.sum()))
            assert abs(x - want_x) < tol + 0.01


def test_payload_ratio_at_one_percent_is_one_over_three_rho():
    wl = synth.workload(0)
    a = synth.WeightSet(wl, "cpu"); b = synth.WeightSet(wl, "cpu")
    synth.fill_base(a, 3)
    synth.make_update(b, a, 3)
    old, new = a.to_numpy_u16()[0], b.to_numpy_u16()[0]
    _, _, counts, _ = oracle.extract(old, new, wl.bucket_elems)
    n, p = wl.numel, 0.01
    sigma = (n * p * (1 - p)) ** 0.5
    assert abs(int(counts.sum()) - n * p) < 5 * sigma
    x = 2 * n / (6 * int(counts.sum()))
    assert abs(x - 1 / (3 * p)) < 1.0


# ---------------------------------------------------------------------------------------------
# tensor lists
# ---------------------------------------------------------------------------------------------

def _split(flat, numel):
    out, off = [], 0
    for m in numel:
        out.append(flat[off:off + m].copy()); off += m
    return out


@pytest.mark.parametrize("numel,be", [
    ([5, 1, 1, 20, 3], 7), ([5, 1, 1, 20, 3], 1), ([5, 1, 1, 20, 3], 30), ([5, 1, 1, 20, 3], 31),
    ([100, 0, 50, 0, 0, 25], 64), ([4096] * 5 + [1] + [70000], 8192), ([1], 1), ([3, 3, 3], 3),
])
def test_list_equals_single_over_concatenation(numel, be):
    rng = np.random.default_rng(sum(numel) + be)
    n = sum(numel)
    old = rnd_u16(rng, n)
    new = flip(old, np.flatnonzero(rng.random(n) < 0.25), rng)
    ref_I = np.flatnonzero(old != new)
    olds, news = _split(old, numel), _split(new, numel)
    I, V, counts, ovf = oracle.extract_multi(olds, news, numel, be)
    nb = -(-n // be)
    assert counts.shape == (nb,) and ovf == 0
    for b in range(nb):
        want = ref_I[(ref_I >= b * be) & (ref_I < (b + 1) * be)]
        assert counts[b] == len(want)
        assert np.array_equal(I[b, :len(want)], want - b * be)               # position inside the bucket
        assert np.array_equal(V[b, :len(want)], new[want])
    for o, w in zip(olds, news):
        assert np.array_equal(o, w)
    roll = _split(old, numel)
    assert oracle.apply_multi(roll, numel, be, I, V, counts) == oracle.OK
    for r, w in zip(roll, news):
        assert np.array_equal(r, w)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_round_trip_tiny_model_shaped_lists(cfg):
    wl = synth.workload(cfg, tiny=True)
    a = synth.WeightSet(wl, "cpu", slab=False); b = synth.WeightSet(wl, "cpu", slab=False)
    synth.fill_base(a, cfg)
    nchanged, masks = synth.make_update(b, a, cfg, want_masks=True)
    olds, news = a.to_numpy_u16(), b.to_numpy_u16()
    roll = [o.copy() for o in olds]
    I, V, counts, ovf = oracle.extract_multi(olds, news, a.numels, wl.bucket_elems)
    assert ovf == 0 and int(counts.sum()) == nchanged
    truth = np.flatnonzero(torch.cat(masks).numpy())                         # packed positions
    got = np.concatenate([I[k, :counts[k]].astype(np.int64) + k * wl.bucket_elems for k in range(len(counts))])
    assert np.array_equal(got, truth)
    assert oracle.apply_multi(roll, a.numels, wl.bucket_elems, I, V, counts) == oracle.OK
    for r, w, o in zip(roll, news, olds):
        assert np.array_equal(r, w) and np.array_equal(o, w)
    if cfg == 3:                                                             # the skewed set has empty buckets
        assert (counts == 0).any()


def test_bucket_range_equals_slice_of_full_run():
    wl = synth.workload(2, tiny=True)
    a = synth.WeightSet(wl, "cpu", slab=False); b = synth.WeightSet(wl, "cpu", slab=False)
    synth.fill_base(a, 9); synth.make_update(b, a, 9)
    olds, news = a.to_numpy_u16(), b.to_numpy_u16()
    be = wl.bucket_elems
    I, V, counts, _ = oracle.extract_multi([o.copy() for o in olds], news, a.numels, be)
    lo, hi = 5, 11
    # tensors wholly outside the range are not needed at all
    starts = np.concatenate([[0], np.cumsum(a.numels)])
    keep = [(starts[k + 1] > lo * be) and (starts[k] < hi * be) for k in range(len(olds))]
    o2 = [o.copy() if k else None for o, k in zip(olds, keep)]
    n2 = [w if k else None for w, k in zip(news, keep)]
    I2, V2, c2, _ = oracle.extract_multi(o2, n2, a.numels, be, b_lo=lo, b_hi=hi)
    assert np.array_equal(c2, counts[lo:hi]) and np.array_equal(I2, I[lo:hi]) and np.array_equal(V2, V[lo:hi])
    # only positions inside the range were refreshed
    for k, (o, w, orig) in enumerate(zip(o2, news, olds)):
        if o is None:
            continue
        g = np.arange(starts[k], starts[k + 1])
        inside = (g >= lo * be) & (g < hi * be)
        assert np.array_equal(o[inside], w[inside]) and np.array_equal(o[~inside], orig[~inside])
    roll = [o.copy() if k else None for o, k in zip(olds, keep)]
    assert oracle.apply_multi(roll, a.numels, be, I2, V2, c2, b_lo=lo, b_hi=hi) == oracle.OK
    for k, (r, w, orig) in enumerate(zip(roll, news, olds)):
        if r is None:
            continue
        g = np.arange(starts[k], starts[k + 1])
        inside = (g >= lo * be) & (g < hi * be)
        assert np.array_equal(r[inside], w[inside]) and np.array_equal(r[~inside], orig[~inside])


# ---------------------------------------------------------------------------------------------
# capacity and invalid payloads
# ---------------------------------------------------------------------------------------------

def test_capacity_overflow_keeps_true_count_and_first_pairs():
    rng = np.random.default_rng(21)
    n, be, cap = 1000, 256, 10
    old = rnd_u16(rng, n)
    pos = np.concatenate([np.arange(0, 10), np.arange(256, 256 + 11), np.arange(600, 640)])
    new = flip(old, pos, rng)
    I, V, counts, ovf = oracle.extract(old.copy(), new, be, cap=cap)
    assert counts.tolist() == [10, 11, 40, 0] and ovf == 2
    assert I[0].tolist() == list(range(10)) and I[1].tolist() == list(range(256, 266))
    assert I[2].tolist() == list(range(600, 610)) and V[2].tolist() == new[600:610].tolist()
    w = old.copy()
    oracle.apply(w, be, I, V, counts)                                        # counts above cap read as cap
    exp = old.copy(); exp[0:10] = new[0:10]; exp[256:266] = new[256:266]; exp[600:610] = new[600:610]
    assert np.array_equal(w, exp)


def test_apply_rejects_index_outside_its_bucket():
    w = np.zeros(100, np.uint16)
    I = np.array([[3, 60, -1], [50, 100, 99]], np.int32)                     # 60 is not in bucket 0, 100 is past the end
    V = np.array([[7, 8, 9], [1, 2, 3]], np.uint16)
    c = np.array([3, 3], np.uint32)
    assert oracle.apply(w, 50, I, V, c) == oracle.BAD_INDEX
    exp = np.zeros(100, np.uint16); exp[3] = 7; exp[50] = 1; exp[99] = 3
    assert np.array_equal(w, exp)
    ws = [np.zeros(60, np.uint16), np.zeros(40, np.uint16)]
    I = np.array([[3, 50, 49], [10, 49, 0]], np.int32)                       # bucket-local: 50 is out of a 50-wide bucket
    assert oracle.apply_multi(ws, [60, 40], 50, I, V, c) == oracle.BAD_INDEX
    assert ws[0][3] == 7 and ws[0][49] == 9 and ws[1][0] == 1 and ws[1][39] == 2 and ws[0][50] == 3


def test_bad_arguments():
    a = np.zeros(4, np.uint16)
    with pytest.raises(ValueError):
        oracle.extract(a.copy(), a, 0)
    with pytest.raises(ValueError):
        oracle.extract(a.copy(), a, 4, cap=0)
    with pytest.raises(ValueError):
        oracle.extract(a.copy(), a, 1 << 31)
    I, V, c, _ = oracle.extract(np.zeros(0, np.uint16), np.zeros(0, np.uint16), 8)
    assert c.size == 0


# ---------------------------------------------------------------------------------------------
# the per-tensor view of a list payload is the paper's own index: flatnonzero taken tensor by tensor (Alg. 2)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("numel,be", [([5, 1, 1, 20, 3], 7), ([100, 0, 50, 0, 0, 25], 64), ([4096] * 3 + [1, 70000], 8192),
                                      ([40000, 7, 40000, 9, 16385], 16384), ([3, 3, 3], 1)])
def test_per_tensor_view_is_flatnonzero_per_tensor(numel, be):
    rng = np.random.default_rng(sum(numel) * 31 + be)
    olds = [rnd_u16(rng, m) for m in numel]
    news = [flip(o, np.flatnonzero(rng.random(o.size) < 0.2), rng) if o.size else o.copy() for o in olds]
    I, V, counts, _ = oracle.extract_multi([o.copy() for o in olds], news, numel, be)
    tid, tix, rc = oracle.tensor_indices(I, counts, numel, be)
    assert rc == oracle.OK
    # gather the view in payload order (bucket by bucket), then split by tensor: order inside a tensor is preserved
    ids = np.concatenate([tid[b, :counts[b]] for b in range(counts.size)]) if counts.size else np.zeros(0, np.uint32)
    idx = np.concatenate([tix[b, :counts[b]] for b in range(counts.size)]) if counts.size else np.zeros(0, np.int32)
    val = np.concatenate([V[b, :counts[b]] for b in range(counts.size)]) if counts.size else np.zeros(0, np.uint16)
    assert np.all(ids[1:] >= ids[:-1])                                    # tensors appear in list order
    for k, (o, w) in enumerate(zip(olds, news)):
        want = np.flatnonzero(o != w)
        assert np.array_equal(idx[ids == k], want), f"tensor {k}"
        assert np.array_equal(val[ids == k], w[want]), f"tensor {k}"
    # untouched slots keep the wrapper's fill; a position outside its bucket is reported
    for b in range(counts.size):
        assert (tid[b, counts[b]:] == 0xFFFFFFFF).all() and (tix[b, counts[b]:] == -1).all()
    if counts.size and counts[-1]:
        bad = I.copy(); bad[-1, 0] = be
        assert oracle.tensor_indices(bad, counts, numel, be)[2] == oracle.BAD_INDEX
