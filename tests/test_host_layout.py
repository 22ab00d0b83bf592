"""Host logic of the library that needs no GPU: the bucket packer's tables (segments, tiles, the
workgroup-to-bucket interleave) checked against a re-derivation in Python."""
import numpy as np
import pytest

from paper_2605_07330_amd import srs, synth


def reference_segments(numel, be):
    out, g = [], 0
    for k, m in enumerate(numel):
        off = 0
        while off < m:
            pos = g + off
            b, boff = divmod(pos, be)
            ln = min(m - off, be - boff)
            out.append((b, boff, ln, k, off))
            off += ln
        g += m
    return out


@pytest.mark.parametrize("numel,be,tile,il", [
    ([5, 1, 1, 20, 3], 7, 4096, 3), ([100, 0, 50, 0, 0, 25], 64, 4096, 1), ([4096] * 5 + [1] + [70000], 8192, 4096, 1024),
    ([40000, 7, 40000, 9, 16385], 16384, 16384, 2), ([37] * 1000 + [5000], 20000, 8192, 4),
])
def test_tables_partition_the_packed_space(numel, be, tile, il):
    L = srs.plan_layout(numel, be, tile, il)
    total = sum(numel)
    nb = -(-total // be)
    assert L["nbuckets"] == nb
    ref = reference_segments(numel, be)
    segs = L["segs"]
    assert len(segs) == len(ref)
    for s, (b, boff, ln, k, off) in zip(segs, ref):
        assert s.tolist() == [boff, ln, k, off]
    # seg_begin delimits each bucket's segments
    for b in range(nb):
        mine = [i for i, r in enumerate(ref) if r[0] == b]
        assert L["seg_begin"][b] == mine[0] and L["seg_begin"][b + 1] == mine[-1] + 1
    # tiles: never longer than `tile`, never across a segment end, and together they cover every element once
    covered = np.zeros(total, np.int32)
    starts = np.concatenate([[0], np.cumsum(numel)])
    bf = L["bucket_first"]
    for b in range(nb):
        for t in L["tiles"][bf[b]:bf[b + 1]]:
            k, toff, boff, ln = map(int, t)
            assert 1 <= ln <= tile and toff + ln <= numel[k] and boff + ln <= be
            g = starts[k] + toff
            assert g // be == b and g % be == boff and (g + ln - 1) // be == b
            covered[g:g + ln] += 1
    assert np.all(covered == 1)
    # every bucket is served by exactly as many workgroups as it has tiles; inside a group of `il` buckets
    # consecutive workgroups rotate over the buckets that still have tiles
    wg = L["wg_bucket"]
    assert np.array_equal(np.bincount(wg, minlength=nb), np.diff(bf))
    assert np.all(np.diff(wg // il) >= 0)
    for g0 in range(0, nb, il):
        sel = wg[(wg >= g0) & (wg < g0 + il)]
        left = np.diff(bf)[g0:g0 + il].astype(np.int64).copy()
        want = []
        while left.sum():
            for j in range(len(left)):
                if left[j]:
                    want.append(g0 + j); left[j] -= 1
        assert sel.tolist() == want


def test_benchmark_workload_counts():
    wl = synth.workload(2)
    L = srs.plan_layout([t.numel for t in wl.tensors], wl.bucket_elems)
    assert L["nbuckets"] == 910 and len(L["tiles"]) == 931760 and len(L["segs"]) == 19438
    assert int(L["tiles"][:, 3].astype(np.int64).sum()) == wl.numel
    assert np.all(L["tiles"][:, 3] == 32768)                  # every tensor of the set is a multiple of a tile
    L2 = srs.plan_layout([t.numel for t in wl.tensors], wl.bucket_elems, tile_elems=16384, interleave=1024)
    assert len(L2["tiles"]) == 1863520 and np.array_equal(L2["segs"], L["segs"])
    assert np.all(L["tiles"][:, 1] % 8 == 0)                  # 16-byte aligned tile starts: the vector path


def test_invalid_layout_arguments():
    with pytest.raises(srs.SrsError):
        srs.plan_layout([10], 0)
    with pytest.raises(srs.SrsError):
        srs.plan_layout([10], 8, tile_elems=1000)
    with pytest.raises(srs.SrsError):
        srs.plan_layout([1 << 31], 8)
