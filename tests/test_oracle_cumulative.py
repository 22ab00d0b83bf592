"""Pins for the oracle's cumulative changed-index set (Alg. 1 as printed: the union over optimizer steps,
sent with the current values by Alg. 2)."""
import numpy as np
import pytest

import oracle


def split(flat, numel):
    out, off = [], 0
    for m in numel:
        out.append(flat[off:off + m].copy()); off += m
    return out


def bits_to_set(bitmap, total):
    return {g for g in range(total) if (bitmap[g >> 5] >> (g & 31)) & 1}


@pytest.mark.parametrize("numel,be", [([50, 3, 0, 77, 1], 32), ([200], 64), ([33, 31, 64, 5], 1000)])
def test_union_over_steps_and_lossless_delivery(numel, be):
    rng = np.random.default_rng(sum(numel))
    total = sum(numel)
    synced = rng.integers(0, 1 << 16, size=total, dtype=np.uint16)        # what Rollout holds
    w = synced.copy()
    bitmap = np.zeros(oracle.bitmap_words(total), np.uint32)
    union = set()
    reverted = None
    for step in range(4):
        prev = w.copy()
        pos = np.flatnonzero(rng.random(total) < 0.1)
        w[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
        if step == 0 and pos.size:
            reverted = int(pos[0])
        if step == 1 and reverted is not None:
            w[reverted] = synced[reverted]                                    # changed, then changed back
        step_set = {int(i) for i in range(total) if prev[i] != w[i]}          # I_t, brute force
        union |= step_set
        oracle.mark_multi(split(prev, numel), split(w, numel), numel, bitmap)
        assert bits_to_set(bitmap, total) == union                            # I_cum = I_cum U I_t
    exact = {int(i) for i in range(total) if synced[i] != w[i]}
    assert exact <= union                                                     # a superset of the true delta
    I, V, c, ovf = oracle.extract_marked_multi(split(w, numel), numel, be, bitmap)
    got = [int(I[b, r]) + b * be for b in range(len(c)) for r in range(c[b])]
    assert got == sorted(union) and ovf == 0                                  # ascending per bucket, all of the set
    assert [int(V[b, r]) for b in range(len(c)) for r in range(c[b])] == [int(w[g]) for g in sorted(union)]
    if reverted is not None and reverted in union and reverted not in exact:
        assert int(w[reverted]) == int(synced[reverted])                      # a redundant pair carries the old value
    roll = split(synced, numel)
    assert oracle.apply_multi(roll, numel, be, I, V, c) == oracle.OK
    assert np.array_equal(np.concatenate(roll) if roll else synced, w)        # Rollout ends bit-identical


def test_cast_mark_equals_round_then_mark():
    rng = np.random.default_rng(8)
    numel = [300, 45, 1000]
    total = sum(numel)
    w0 = rng.integers(0, 1 << 16, size=total, dtype=np.uint16)
    master = rng.standard_normal(total).astype(np.float32)
    keep = rng.random(total) < 0.8
    master[keep] = (w0[keep].astype(np.uint32) << 16).view(np.float32)
    rounded = oracle.round_bf16(master)
    bm_ref = np.zeros(oracle.bitmap_words(total), np.uint32)
    oracle.mark_multi(split(w0, numel), split(rounded, numel), numel, bm_ref)
    ws = split(w0, numel)
    bm = np.zeros_like(bm_ref)
    oracle.cast_mark_multi(ws, split(master, numel), numel, bm)
    assert np.array_equal(bm, bm_ref)
    assert np.array_equal(np.concatenate(ws), rounded)
    # marking again with the same master weights adds nothing
    oracle.cast_mark_multi(ws, split(master, numel), numel, bm)
    assert np.array_equal(bm, bm_ref)


def test_capacity_and_empty_set():
    numel = [100]
    w = [np.arange(100, dtype=np.uint16)]
    bm = np.zeros(oracle.bitmap_words(100), np.uint32)
    I, V, c, ovf = oracle.extract_marked_multi(w, numel, 40, bm)
    assert c.tolist() == [0, 0, 0] and np.all(I == -1)
    bm[0] = 0xFFFFFFFF; bm[2] = 0x5
    I, V, c, ovf = oracle.extract_marked_multi(w, numel, 40, bm, cap=10)
    assert c.tolist() == [32, 2, 0] and ovf == 1
    assert I[0].tolist() == list(range(10)) and I[1, :2].tolist() == [24, 26] and V[1, :2].tolist() == [64, 66]
