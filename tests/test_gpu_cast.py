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


def test_rounding_equals_the_frameworks_device_cast_nan_included(srs):
    """The Trainer's cast runs on the GPU (Alg. 1, Sec. 3.4: the optimizer's FP32 -> BF16 copy of the training
    stack).  On this platform PyTorch's device cast is that routine: it must give what the oracle's rounding and the
    fused kernel give on every class of binary32 pattern -- including the NaN patterns, where the paper is silent and
    CPU library casts differ (all of them map to the quiet NaN 0x7FC0 here)."""
    rng = np.random.default_rng(11)
    special = np.array([0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF800001, 0x7FFFFFFF, 0xFFFFFFFF, 0x7FA00000, 0x7F80FFFF,
                        0xFF812345, 0x7F800000, 0xFF800000, 0x00000000, 0x80000000, 0x00000001, 0x807FFFFF,
                        0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x7F7FFFFF, 0xFF7F8000], dtype=np.uint32)
    nan_hi = (0x7F800001 + rng.integers(0, 0x7FFFFF, size=50000, dtype=np.uint32)) | (rng.integers(0, 2, size=50000, dtype=np.uint32) << 31)
    m_h = np.concatenate([special, nan_hi, rng.integers(0, 1 << 32, size=400000, dtype=np.uint64).astype(np.uint32)])
    n = m_h.size
    d_m = torch.from_numpy(m_h.view(np.int32).copy()).to(DEV).view(torch.float32)
    framework = u16(d_m.to(torch.bfloat16))
    assert np.array_equal(oracle.round_bf16(m_h.view(np.float32)), framework), "oracle rounding differs from the device cast"
    is_nan = (m_h & 0x7FFFFFFF) > 0x7F800000
    assert is_nan.sum() > 50000 and np.all(framework[is_nan] == 0x7FC0)
    # the fused kernel: parameters that differ from the rounded master everywhere, so that every element is emitted
    w_h = (~framework).astype(np.uint16)
    d_w = from_u16(w_h, DEV)
    c = srs.Context(0)
    try:
        I, V, counts = srs.alloc_payload(1, n, DEV)
        c.extract_cast(d_w, d_m, n, I, V, counts, n)
        assert c.status() == 0
        assert int(counts[0].item()) == n
        assert np.array_equal(V[0].cpu().numpy().view(np.uint16), framework)
        assert np.array_equal(u16(d_w), framework)
    finally:
        c.close()
