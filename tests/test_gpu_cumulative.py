"""GPU parity for the cumulative changed-index set (Alg. 1 as printed): srs_mark_multi,
srs_cast_mark_multi and srs_extract_marked_multi against the oracle, bit for bit."""
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


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
@pytest.mark.parametrize("tile", [4096, 16384])
@pytest.mark.parametrize("slab,misalign", [(True, 0), (False, 1)])
def test_three_steps_then_sync(srs, cfg, tile, slab, misalign):
    print(f"case cfg={cfg} tile={tile} slab={slab}", flush=True)
    wl = synth.workload(cfg, tiny=True)
    cur = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign)
    nxt = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign * 2)
    roll = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign * 3)
    synth.fill_base(cur, cfg + 50)
    roll.copy_from(cur)
    synced = cur.to_numpy_u16()
    words = oracle.bitmap_words(wl.numel)
    bm_ref = np.zeros(words, np.uint32)
    c = srs.Context(0)
    try:
        c.set_option(srs.OPT_TILE_ELEMS, tile)
        plan = c.plan(cur.numels, wl.bucket_elems)
        bitmap = torch.zeros(srs.bitmap_words(wl.numel), dtype=torch.int32, device=DEV)
        for step in range(1, 4):
            synth.make_update(nxt, cur, cfg + 50, step=step)
            if step == 2:                                     # undo part of step 1: changed and changed back
                for a, s0 in zip(nxt.tensors[:3], synced[:3]):
                    a[: a.numel() // 2].copy_(from_u16(s0[: a.numel() // 2], DEV))
            oracle.mark_multi(cur.to_numpy_u16(), nxt.to_numpy_u16(), cur.numels, bm_ref)
            c.mark_multi(plan, cur.tensors, nxt.tensors, bitmap)
            cur.copy_from(nxt)
            assert np.array_equal(bitmap.cpu().numpy().view(np.uint32), bm_ref), f"bitmap after step {step}"
        cap = wl.bucket_elems
        want = oracle.extract_marked_multi(cur.to_numpy_u16(), cur.numels, wl.bucket_elems, bm_ref)[:3]
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        c.extract_marked_multi(plan, cur.tensors, bitmap, I, V, counts, cap)
        c.apply_multi(plan, roll.tensors, I, V, counts, cap)
        assert c.status() == 0
        plan.close()
    finally:
        c.close()
    assert_payload_equal(payload_to_host(I, V, counts), want, "marked")
    assert roll.equal(cur), "rollout is not bit-identical after the cumulative update"
    exact = sum(int((a != b).sum()) for a, b in zip(synced, cur.to_numpy_u16()))
    assert int(want[2].sum()) >= exact                       # superset of the true delta


@pytest.mark.parametrize("cfg", [2, 4])
def test_cast_mark_steps(srs, cfg):
    print(f"case cast-mark cfg={cfg}", flush=True)
    wl = synth.workload(cfg, tiny=True)
    W = synth.WeightSet(wl, DEV, slab=False, misalign=1)
    tmp = synth.WeightSet(wl, DEV)
    roll = synth.WeightSet(wl, DEV)
    synth.fill_base(W, cfg + 70)
    roll.copy_from(W)
    master_flat = torch.empty(wl.numel, dtype=torch.float32, device=DEV)
    masters, off = [], 0
    for t in wl.tensors:
        masters.append(master_flat[off:off + t.numel]); off += t.numel
    bm_ref = np.zeros(oracle.bitmap_words(wl.numel), np.uint32)
    ws_ref = W.to_numpy_u16()
    c = srs.Context(0)
    try:
        plan = c.plan(W.numels, wl.bucket_elems)
        bitmap = torch.zeros(srs.bitmap_words(wl.numel), dtype=torch.int32, device=DEV)
        for step in range(1, 4):
            cur_slab = synth.WeightSet(wl, DEV); cur_slab.copy_from(W)
            synth.make_update(tmp, cur_slab, cfg + 70, step=step)
            synth.master_from_(master_flat, tmp.flat, cfg, salt=step)
            oracle.cast_mark_multi(ws_ref, [m.cpu().numpy() for m in masters], W.numels, bm_ref)
            c.cast_mark_multi(plan, W.tensors, masters, bitmap)
            assert np.array_equal(bitmap.cpu().numpy().view(np.uint32), bm_ref), f"bitmap after step {step}"
            assert all(np.array_equal(x, y) for x, y in zip(W.to_numpy_u16(), ws_ref)), "parameters after the cast"
        cap = wl.bucket_elems
        want = oracle.extract_marked_multi(ws_ref, W.numels, wl.bucket_elems, bm_ref)[:3]
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        c.extract_marked_multi(plan, W.tensors, bitmap, I, V, counts, cap)
        c.apply_multi(plan, roll.tensors, I, V, counts, cap)
        assert c.status() == 0
        plan.close()
    finally:
        c.close()
    assert_payload_equal(payload_to_host(I, V, counts), want, "cast-marked")
    assert roll.equal(W)


def test_odd_shapes_and_capacity(srs):
    numel = [5, 1, 1, 20, 3, 0, 4099, 37, 70000]
    be = 4100
    rng = np.random.default_rng(2)
    prev = [rng.integers(0, 1 << 16, size=m, dtype=np.uint16) for m in numel]
    cur = [p.copy() for p in prev]
    for w in cur:
        w[rng.random(w.size) < 0.3] ^= 0x00F0
    bm_ref = np.zeros(oracle.bitmap_words(sum(numel)), np.uint32)
    oracle.mark_multi(prev, cur, numel, bm_ref)
    cap = 500
    wI, wV, wc, ovf = oracle.extract_marked_multi(cur, numel, be, bm_ref, cap=cap)
    assert ovf > 0
    c = srs.Context(0)
    try:
        plan = c.plan(numel, be)
        d_prev = [from_u16(p, DEV) for p in prev]; d_cur = [from_u16(w, DEV) for w in cur]
        bitmap = torch.zeros(srs.bitmap_words(sum(numel)), dtype=torch.int32, device=DEV)
        c.mark_multi(plan, d_prev, d_cur, bitmap)
        assert np.array_equal(bitmap.cpu().numpy().view(np.uint32), bm_ref)
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        c.extract_marked_multi(plan, d_cur, bitmap, I, V, counts, cap)
        assert c.status() == srs.FLAG_OVERFLOW
        plan.close()
    finally:
        c.close()
    assert_payload_equal(payload_to_host(I, V, counts), (wI, wV, wc), "marked, overflow")


@pytest.mark.parametrize("tile", [4096, 8192, 16384, 32768])
@pytest.mark.parametrize("density", [0.0, 0.003, 0.2, 1.0])
def test_bitmap_gather_every_tile_size(srs, tile, density):
    """The bitmap is given directly (any set of positions is a valid index set): empty, sparse, dense enough for
    several staging rounds per tile, and all ones; odd tensor sizes put tile starts at every bit offset of a word."""
    print(f"case bitmap gather tile={tile} density={density}", flush=True)
    numel = [33, 70001, 1, 0, 131072, 4097, 95, 262144 + 17]
    total, be = sum(numel), 150000
    rng = np.random.default_rng(int(density * 1000) + tile)
    cur = [rng.integers(0, 1 << 16, size=m, dtype=np.uint16) for m in numel]
    bits = (rng.random(total) < density) if density < 1.0 else np.ones(total, bool)
    words = oracle.bitmap_words(total)
    padded = np.zeros(words * 32, bool); padded[:total] = bits
    bm = np.packbits(padded.reshape(-1, 32), axis=1, bitorder="little").view(np.uint32).reshape(-1).copy()
    cap = be
    wI, wV, wc, ovf = oracle.extract_marked_multi(cur, numel, be, bm, cap=cap)
    assert ovf == 0 and int(wc.sum()) == int(bits.sum())
    c = srs.Context(0)
    try:
        c.set_option(srs.OPT_TILE_ELEMS, tile)
        plan = c.plan(numel, be)
        d_cur = [from_u16(w, DEV) for w in cur]
        bitmap = torch.from_numpy(bm.view(np.int32)).to(DEV)
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        c.extract_marked_multi(plan, d_cur, bitmap, I, V, counts, cap)
        assert c.status() == 0
        plan.close()
    finally:
        c.close()
    assert_payload_equal(payload_to_host(I, V, counts), (wI, wV, wc), "bitmap gather")
