"""srs_extract_noalloc (static scratch, never allocates) against srs_extract, through the C ABI, bit for bit:
indices, values, counts, untouched payload slots and the refreshed snapshot.  Two calls in a row on one context,
the second with a smaller input (the static array still holds the first call's status words and tickets), then
one more with many small buckets (ticket counters packed 4 bytes apart) and the size limits."""
import numpy as np
import pytest
import torch

import oracle
from util import from_u16, payload_to_host, u16

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _pair(n, density, seed):
    rng = np.random.default_rng(seed)
    old = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    new = old.copy()
    pos = np.flatnonzero(rng.random(n) < density)
    if pos.size:
        delta = rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint32)
        new[pos] = ((old[pos].astype(np.uint32) + delta) & 0xFFFF).astype(np.uint16)
    return old, new


def _both_ways(srs, ctx, n, be, density, seed, cap=None):
    old_h, new_h = _pair(n, density, seed)
    cap = be if cap is None else cap
    nb = (n + be - 1) // be
    got = []
    for call in (ctx.extract, ctx.extract_noalloc):
        d_old, d_new = from_u16(old_h, DEV), from_u16(new_h, DEV)
        I, V, counts = srs.alloc_payload(nb, cap, DEV)
        print(f"{call.__name__}: n={n} be={be} density={density} seed={seed}", flush=True)
        call(d_old, d_new, be, I, V, counts, cap)
        assert ctx.status() == 0
        got.append((payload_to_host(I, V, counts), u16(d_old)))
    (pa, sa), (pb, sb) = got
    for x, y, what in zip(pa, pb, ("indices", "values", "counts")):
        assert np.array_equal(x, y), f"{what} differ between srs_extract and srs_extract_noalloc"
    assert np.array_equal(sa, sb) and np.array_equal(sb, new_h), "snapshot"
    # and both against the oracle, so that agreement is not agreement in error
    wI, wV, wc, wold = oracle.extract(old_h, new_h, be, cap=cap)
    assert np.array_equal(pb[2], wc) and np.array_equal(pb[0], wI) and np.array_equal(pb[1], wV)
    return int(pb[2].sum())


def test_noalloc_matches_extract_on_two_calls_in_a_row_then_many_buckets():
    from paper_2605_07330_amd import srs
    ctx = srs.Context(0)
    try:
        # several tiles per bucket, ragged tail; then a smaller input right after it
        big = _both_ways(srs, ctx, n=3_000_017, be=700_001, density=0.01, seed=11)
        small = _both_ways(srs, ctx, n=70_001, be=33_000, density=0.02, seed=12)
        assert big > small > 0
        # more buckets than fit 256 bytes apart in the static array: counters 4 bytes apart
        _both_ways(srs, ctx, n=20_003, be=3, density=0.3, seed=13)
        # identical inputs: empty payload, slots untouched
        assert _both_ways(srs, ctx, n=100_000, be=40_000, density=0.0, seed=14) == 0
    finally:
        ctx.close()


def test_noalloc_refuses_sizes_beyond_its_static_array():
    from paper_2605_07330_amd import srs
    ctx = srs.Context(0)
    try:
        n = (1 << 18) + 1                       # one bucket per element: more buckets than ticket counters
        d_old = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
        d_new = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
        I, V, counts = srs.alloc_payload(n, 1, DEV)
        counts.fill_(7)
        with pytest.raises(srs.SrsError) as e:
            ctx.extract_noalloc(d_old, d_new, 1, I, V, counts, 1)
        assert e.value.code == srs.ERR_TOO_LARGE
        torch.cuda.synchronize()
        assert int(counts.min()) == 7 and int(counts.max()) == 7, "nothing may be launched on an error"
        ctx.extract(d_old, d_new, 1, I, V, counts, 1)          # the allocating entry point takes the same input
        assert ctx.status() == 0 and int(counts.sum()) == 0
    finally:
        ctx.close()


def test_noalloc_first_call_under_graph_capture_then_replays():
    """What the entry point is for: a fresh context whose very first extract of this size is recorded into a HIP
    graph (where the runtime forbids allocation and synchronisation), followed by the scatter; every replay, with the
    program's own eager work in between, must equal the oracle on the data of that replay."""
    from paper_2605_07330_amd import srs
    n, be = 1_200_003, 400_001
    nb = (n + be - 1) // be
    cap = be
    ctx = srs.Context(0)
    try:
        base_h, _ = _pair(n, 0.0, 30)
        d_base = from_u16(base_h, DEV)
        d_old = d_base.clone(); d_new = d_base.clone(); d_roll = d_base.clone()
        I, V, counts = srs.alloc_payload(nb, cap, DEV)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        print("capturing srs_extract_noalloc + srs_apply", flush=True)
        with torch.cuda.graph(g):
            ctx.extract_noalloc(d_old, d_new, be, I, V, counts, cap)
            ctx.apply(d_roll, be, I, V, counts, cap)
        for rep in range(4):
            _, new_h = _pair(n, 0.01 * (rep + 1), 30)           # same old values (same seed), denser update every time
            d_old.copy_(d_base); d_roll.copy_(d_base); d_new.copy_(from_u16(new_h, DEV))
            I.fill_(-1); V.fill_(-1); counts.zero_()
            torch.cuda.synchronize()
            print(f"replay {rep}", flush=True)
            g.replay()
            torch.cuda.synchronize()
            assert ctx.status() == 0
            wI, wV, wc, _ = oracle.extract(base_h.copy(), new_h, be, cap=cap)
            gI, gV, gc = payload_to_host(I, V, counts)
            assert np.array_equal(gc, wc) and np.array_equal(gI, wI) and np.array_equal(gV, wV), f"replay {rep}"
            assert np.array_equal(u16(d_old), new_h) and np.array_equal(u16(d_roll), new_h), f"replay {rep}: weights"
    finally:
        ctx.close()
