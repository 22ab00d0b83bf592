"""Pins for the oracle's index delta coding (Sec. 3.3): numpy's diff / cumsum state the same transform,
the 16-bit width rule, the anchors, and the per-element wire size the paper prints."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "payload_cost_model.txt")


def payload(rng, n, be, p):
    old = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    new = old.copy()
    pos = np.flatnonzero(rng.random(n) < p)
    new[pos] ^= 1
    I, V, c, _ = oracle.extract(old, new, be)
    return I, V, c, pos


@pytest.mark.parametrize("n,be,p", [(100000, 30000, 0.01), (50000, 50000, 0.3), (4097, 2048, 1.0), (9000, 1000, 0.0)])
def test_differences_match_numpy_diff_with_zero_prepended(n, be, p):
    rng = np.random.default_rng(n)
    I, V, c, pos = payload(rng, n, be, p)
    D, mg, an = oracle.encode_indices(I, c, base_stride=be)
    for b in range(len(c)):
        loc = I[b, :c[b]].astype(np.int64) - b * be                     # positions inside the bucket
        want = np.diff(loc, prepend=0)                                  # first differences, zero prepended
        assert np.array_equal(D[b, :c[b]].astype(np.int64), want & 0xFFFF)
        assert mg[b] == (want.max() if c[b] else 0)
        assert np.array_equal(an[b, :(c[b] + 2047) // 2048], loc[::2048])
        assert np.all(D[b, c[b]:] == 0xFFFF) and np.all(an[b, (c[b] + 2047) // 2048:] == -1)
        # inverse = running sum
        assert np.array_equal(np.cumsum(D[b, :c[b]].astype(np.int64)), loc) or mg[b] >= 65536
    back = oracle.decode_indices(D, I, c, mg, base_stride=be)
    for b in range(len(c)):
        assert np.array_equal(back[b, :c[b]], I[b, :c[b]])


def test_list_payloads_use_positions_inside_the_bucket():
    rng = np.random.default_rng(3)
    numel = [5000, 17, 30000, 1, 9000]
    olds = [rng.integers(0, 1 << 16, size=m, dtype=np.uint16) for m in numel]
    news = [o.copy() for o in olds]
    for w in news:
        w[rng.random(w.size) < 0.05] ^= 3
    I, V, c, _ = oracle.extract_multi([o.copy() for o in olds], news, numel, 8192)
    D, mg, an = oracle.encode_indices(I, c)                              # base_stride 0
    for b in range(len(c)):
        assert np.array_equal(D[b, :c[b]].astype(np.int64), np.diff(I[b, :c[b]].astype(np.int64), prepend=0))
    back = oracle.decode_indices(D, np.zeros_like(I), c, mg)             # no wide bucket: I_wide never read
    assert all(np.array_equal(back[b, :c[b]], I[b, :c[b]]) for b in range(len(c)))
    roll = [o.copy() for o in olds]
    oracle.apply_multi(roll, numel, 8192, back, V, c)
    assert all(np.array_equal(r, w) for r, w in zip(roll, news))


def test_width_rule_at_two_to_the_fifteen():
    # gaps of 32767 fit, a gap of 32768 does not: that bucket keeps its 32-bit indices
    I = np.array([[5, 32772, 32780, -1], [32768, 32769, -1, -1], [0, 65535, 98302, 131069]], np.int32)
    c = np.array([3, 2, 4], np.uint32)
    D, mg, an = oracle.encode_indices(I, c)
    assert mg.tolist() == [32767, 32768, 65535]
    assert D[0, :3].tolist() == [5, 32767, 8] and D[1, :2].tolist() == [32768, 1]
    back = oracle.decode_indices(D, I, c, mg)
    assert back[0, :3].tolist() == [5, 32772, 32780]                     # decoded from differences
    assert back[1, :2].tolist() == [32768, 32769] and back[2].tolist() == I[2].tolist()   # taken from I
    poisoned = np.full_like(I, 7)
    back2 = oracle.decode_indices(D, poisoned, c, mg)
    assert back2[0, :3].tolist() == [5, 32772, 32780] and back2[1, :2].tolist() == [7, 7]


def test_unsorted_indices_are_rejected():
    I = np.array([[9, 3, 4]], np.int32)
    with pytest.raises(ValueError):
        oracle.encode_indices(I, np.array([3], np.uint32))


def test_iid_one_percent_gaps_are_far_below_the_limit_and_cost_two_bytes():
    rng = np.random.default_rng(11)
    n, be = 1 << 22, 1 << 20
    I, V, c, pos = payload(rng, n, be, 0.0062)
    D, mg, an = oracle.encode_indices(I, c, base_stride=be)
    assert int(mg.max()) < 32768 and int(mg.max()) > 200             # "maxima in the low thousands" (Sec. 3.3)
    changed = int(c.sum())
    index_bytes = D[:, 0].itemsize * changed                         # one 16-bit difference per changed element
    rows = [l.split() for l in open(GOLDEN) if l.startswith("worked_example_100x")]
    rho, b_i, alpha, per_elem, ratio, tol = map(float, rows[0][1:7])
    assert index_bytes == b_i * changed
    wire = index_bytes + alpha * 2 * changed                         # Eq. (3) with the paper's alpha for values
    assert abs(wire / changed - per_elem) < 1e-9
    assert abs(2 * n / wire - ratio) < tol + 100 * abs(changed / n - rho) / rho
    # without value coding (alpha = 1) the encoded payload is 4 B per pair: X = 1/(2 rho)
    assert abs(2 * n / (4 * changed) - 1 / (2 * changed / n)) < 1e-9
