"""GPU parity of the rotating-snapshot contract (SRS_OPT_SNAPSHOT = 1).

Extract leaves the snapshot alone and the caller swaps roles: the new weights of one synchronisation are
the snapshot of the next, and the Trainer's next cast overwrites the buffer that held the old snapshot.
The payload is Alg. 2's, so it is compared element by element with the oracle's (whose own snapshot is
refreshed the paper's way, by a copy); on top of that the snapshot buffer must come back bit for bit
untouched, and a chain of synchronisations over two alternating buffers must keep the rollout copy equal
to the Trainer's weights.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth
from util import assert_payload_equal, from_u16, payload_to_host, u16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def srs():
    from paper_2605_07330_amd import srs as m
    return m


def next_version(rng, cur, density):
    """What a Trainer step leaves in the other buffer: the current patterns with a few of them replaced."""
    new = cur.copy()
    pos = np.flatnonzero(rng.random(cur.size) < density)
    if pos.size:
        delta = rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint32)
        new[pos] = ((cur[pos].astype(np.uint32) + delta) & 0xFFFF).astype(np.uint16)
    return new


@pytest.mark.parametrize("tile", [4096, 16384, 32768])
@pytest.mark.parametrize("n,be,density", [(1, 1, 1.0), (70001, 1000, 0.02), (300007, 65536, 0.01),
                                          ((1 << 20) + 5, (1 << 18) + 3, 0.01), (100003, 100003, 0.0),
                                          (100003, 20000, 1.0)])
def test_single_tensor_chain(srs, tile, n, be, density):
    print(f"case rotate single n={n} be={be} density={density} tile={tile}", flush=True)
    rng = np.random.default_rng(n + tile)
    ctx = srs.Context(0)
    try:
        ctx.set_option(srs.OPT_TILE_ELEMS, tile)
        ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_ROTATE)
        nb = (n + be - 1) // be
        cur_h = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
        bufs = [from_u16(cur_h, DEV), from_u16(np.zeros(n, np.uint16), DEV)]
        roll = from_u16(cur_h, DEV)
        I, V, counts = srs.alloc_payload(nb, be, DEV)
        for step in range(3):
            new_h = next_version(rng, cur_h, density)
            snap, new = bufs[step % 2], bufs[(step + 1) % 2]
            new.view(torch.int16).copy_(torch.from_numpy(new_h.view(np.int16)))          # the Trainer's write
            I.fill_(-1); V.fill_(-1)
            ctx.extract(snap, new, be, I, V, counts, be)
            ctx.apply(roll, be, I, V, counts, be)
            assert ctx.status() == 0
            wI, wV, wc, ovf = oracle.extract(cur_h.copy(), new_h, be, cap=be)
            assert ovf == 0
            assert_payload_equal(payload_to_host(I, V, counts), (wI, wV, wc), f"step {step}")
            assert np.array_equal(u16(snap), cur_h), "the snapshot buffer was written"
            assert np.array_equal(u16(new), new_h), "the new weights were written"
            assert np.array_equal(u16(roll), new_h), "reconstruction differs"
            cur_h = new_h
    finally:
        ctx.close()


@pytest.mark.parametrize("cfg,misalign", [(2, 0), (2, 1), (3, 0)])
def test_tensor_list_chain(srs, cfg, misalign):
    print(f"case rotate list cfg={cfg} misalign={misalign}", flush=True)
    wl = synth.workload(cfg, tiny=True)
    A = synth.WeightSet(wl, DEV, misalign=misalign); B = synth.WeightSet(wl, DEV, misalign=misalign)
    R = synth.WeightSet(wl, DEV, misalign=misalign)
    synth.fill_base(A, cfg)
    R.copy_from(A)
    ctx = srs.Context(0)
    try:
        ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_ROTATE)
        ctx.set_option(srs.OPT_TILE_ELEMS, 4096)
        plan = ctx.plan(A.numels, wl.bucket_elems)
        cap = wl.bucket_elems
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        bufs = [A, B]
        for step in range(4):
            snap, new = bufs[step % 2], bufs[(step + 1) % 2]
            nchanged, _ = synth.make_update(new, snap, cfg, step=step + 1)       # overwrites the stale buffer
            snap_h, new_h = snap.to_numpy_u16(), new.to_numpy_u16()
            I.fill_(-1); V.fill_(-1)
            ctx.extract_multi(plan, snap.tensors, new.tensors, I, V, counts, cap)
            ctx.apply_multi(plan, R.tensors, I, V, counts, cap)
            assert ctx.status() == 0
            wI, wV, wc, ovf = oracle.extract_multi([x.copy() for x in snap_h], new_h, A.numels, wl.bucket_elems, cap=cap)
            assert ovf == 0 and int(wc.sum()) == nchanged
            assert_payload_equal(payload_to_host(I, V, counts), (wI, wV, wc), f"step {step}")
            for x, y in zip(snap.to_numpy_u16(), snap_h):
                assert np.array_equal(x, y), "the snapshot buffers were written"
            assert R.equal(new), "reconstruction differs"
        plan.close()
    finally:
        ctx.close()


def test_option_range(srs):
    ctx = srs.Context(0)
    try:
        with pytest.raises(srs.SrsError):
            ctx.set_option(srs.OPT_SNAPSHOT, 3)
        ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_REFRESH)
    finally:
        ctx.close()
