"""GPU parity for the fused cast + diff (srs_extract_cast*) against the oracle, bit for bit."""
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


def make_case(n, seed, frac_same=0.97):
    rng = np.random.default_rng(seed)
    w = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    master = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)        # any binary32 pattern
    keep = rng.random(n) < frac_same
    # master weights that round back to the current parameter: same upper half, lower half below the tie
    master[keep] = (w[keep].astype(np.uint32) << 16) | rng.integers(0, 0x7FFF, size=int(keep.sum()), dtype=np.uint32)
    nan_w = ((w & 0x7F80) == 0x7F80) & ((w & 0x7F) != 0)
    master[keep & nan_w] = 0x7FC00000                                                   # NaN parameters: NaN master
    return w, master


@pytest.mark.parametrize("tile", [4096, 16384, 32768])
@pytest.mark.parametrize("n,be,offset", [(1, 1, 0), (9, 4, 0), (2049, 2048, 0), (100003, 33000, 0), (100003, 33000, 1),
                                          (300000, 65536, 3), (1 << 20, 1 << 18, 0), ((1 << 20) + 5, (1 << 18) + 3, 0)])
def test_single_tensor_cast_matches_oracle(srs, tile, n, be, offset):
    print(f"case tile={tile} n={n} be={be} offset={offset}", flush=True)
    c = srs.Context(0)
    try:
        c.set_option(srs.OPT_TILE_ELEMS, tile)
        w_h, m_h = make_case(n, seed=n + tile)
        w_ref = w_h.copy()
        want = oracle.extract_cast(w_ref, m_h, be)[:3]
        d_w = from_u16(np.concatenate([np.zeros(offset, np.uint16), w_h]), DEV)[offset:]
        d_m = torch.from_numpy(np.concatenate([np.zeros(offset, np.uint32), m_h]).view(np.int32)).to(DEV).view(torch.float32)[offset:]
        d_roll = from_u16(w_h, DEV)
        nb = (n + be - 1) // be
        I, V, counts = srs.alloc_payload(nb, be, DEV)
        c.extract_cast(d_w, d_m, be, I, V, counts, be)
        c.apply(d_roll, be, I, V, counts, be)
        assert c.status() == 0
        assert_payload_equal(payload_to_host(I, V, counts), want, "cast")
        assert np.array_equal(u16(d_w), w_ref), "model parameters are not the rounded master weights"
        assert np.array_equal(u16(d_roll), w_ref), "rollout reconstruction differs"
    finally:
        c.close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
@pytest.mark.parametrize("slab", [True, False])
def test_tensor_lists_cast(srs, cfg, slab):
    print(f"case cfg={cfg} slab={slab}", flush=True)
    wl = synth.workload(cfg, tiny=True)
    a = synth.WeightSet(wl, DEV, slab=slab, misalign=0 if slab else 1)
    b = synth.WeightSet(wl, DEV, slab=True)
    r = synth.WeightSet(wl, DEV, slab=slab)
    synth.fill_base(a, cfg + 30)
    nchanged, _ = synth.make_update(b, a, cfg + 30)
    r.copy_from(a)
    master_flat = torch.empty(wl.numel, dtype=torch.float32, device=DEV)
    synth.master_from_(master_flat, b.flat, cfg)
    masters, off = [], 0
    for t in wl.tensors:
        masters.append(master_flat[off:off + t.numel]); off += t.numel
    ws = a.to_numpy_u16()
    ms = [m.cpu().numpy() for m in masters]
    want = oracle.extract_cast_multi(ws, ms, a.numels, wl.bucket_elems)[:3]
    c = srs.Context(0)
    try:
        plan = c.plan(a.numels, wl.bucket_elems)
        cap = wl.bucket_elems
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        c.extract_cast_multi(plan, a.tensors, masters, I, V, counts, cap)
        c.apply_multi(plan, r.tensors, I, V, counts, cap)
        assert c.status() == 0
        plan.close()
    finally:
        c.close()
    got = payload_to_host(I, V, counts)
    assert_payload_equal(got, want, f"cast cfg {cfg}")
    assert int(got[2].sum()) == nchanged
    assert a.equal(b), "model parameters are not the rounded master weights"
    assert r.equal(b), "rollout reconstruction differs"
