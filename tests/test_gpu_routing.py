"""GPU parity for density routing and the dense (full-copy) route against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth
from util import from_u16, u16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def srs():
    from paper_2605_07330_amd import srs as m
    return m


@pytest.fixture(scope="module")
def ctx(srs):
    c = srs.Context(0)
    yield c
    c.close()


def route_buffers(nb, max_dense):
    return (torch.full((nb,), -9, dtype=torch.int32, device=DEV), torch.full((nb,), 12345, dtype=torch.int32, device=DEV),
            torch.full((max(max_dense, 1),), -1, dtype=torch.int32, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV))


@pytest.mark.parametrize("nb,be,total,cap,bpp,max_dense", [
    (6, 100, 560, 50, 6, 6), (6, 100, 560, 50, 4, 6), (6, 100, 560, 50, 6, 1), (1000, 64, 63990, 64, 6, 1000),
    (1000, 64, 63990, 64, 4, 10), (1, 5, 5, 5, 6, 1), (700, 33554432, 700 * 33554432 - 5, 423528, 6, 64),
])
def test_route_matches_oracle(srs, ctx, nb, be, total, cap, bpp, max_dense):
    rng = np.random.default_rng(nb + be + bpp + max_dense)
    counts = rng.integers(0, min(be, 2**31 - 1) + 1, size=nb, dtype=np.uint64)
    counts[rng.random(nb) < 0.7] //= 50                          # most buckets sparse
    counts = counts.astype(np.uint32)
    want = oracle.route(counts, be, total, cap, bytes_per_pair=bpp, max_dense=max_dense)
    d_counts = torch.from_numpy(counts.view(np.int32)).to(DEV)
    slot, sc, db, nd = route_buffers(nb, max_dense)
    ctx.route(d_counts, nb, be, total, cap, bpp, max_dense, slot, sc, db, nd)
    flags = ctx.status()
    assert flags == (srs.FLAG_OVERFLOW if want[4] else 0)
    assert np.array_equal(slot.cpu().numpy(), want[0])
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), want[1])
    assert int(nd.item()) == want[3]
    assert np.array_equal(db.cpu().numpy()[:want[3]], want[2][:want[3]])


@pytest.mark.parametrize("slab,misalign", [(True, 0), (False, 0), (False, 1)])
def test_mixed_update_round_trip(srs, ctx, slab, misalign):
    """A tiny MoE-shaped list where two layers' routers and some experts change everywhere (adapter-like),
    the rest at 1 %: sparse buckets through apply, dense buckets through pack / unpack."""
    wl = synth.workload(2, tiny=True)
    a = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign)
    b = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign * 2)
    r = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign * 3)
    synth.fill_base(a, 21)
    synth.make_update(b, a, 21)
    for k, spec in enumerate(wl.tensors):                       # make some tensors change on every element
        if spec.kind == "router" or (spec.kind == "expert" and spec.expert in (3, 4)):
            b.tensors[k].view(torch.int16).bitwise_xor_(1)
    r.copy_from(a)
    olds, news = a.to_numpy_u16(), b.to_numpy_u16()
    be, cap = wl.bucket_elems, 600
    wI, wV, wc, ovf = oracle.extract_multi([o.copy() for o in olds], news, a.numels, be, cap=cap)
    w_slot, w_sc, w_db, w_nd, _ = oracle.route(wc, be, wl.numel, cap)
    assert w_nd >= 2 and ovf >= 1
    w_dense = np.zeros(w_nd * be, np.uint16)
    oracle.copy_dense_multi(news, a.numels, be, w_db, w_nd, w_dense, pack=True)

    plan = ctx.plan(a.numels, be)
    I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
    max_dense = plan.nbuckets
    slot, sc, db, nd = route_buffers(plan.nbuckets, max_dense)
    dense = torch.zeros(max_dense * be, dtype=torch.int16, device=DEV)
    pairs = ctx.bind_pairs(plan, a.tensors, b.tensors)
    ctx.extract_multi(plan, None, None, I, V, counts, cap, pairs=pairs)
    assert ctx.status() == srs.FLAG_OVERFLOW                     # the dense tensors overflowed their slots
    ctx.route(counts, plan.nbuckets, be, wl.numel, cap, 6, max_dense, slot, sc, db, nd)
    ctx.pack_dense_multi(plan, None, None, db, nd, max_dense, dense, pairs=pairs)
    ctx.apply_multi(plan, r.tensors, I, V, sc, cap)
    ctx.unpack_dense_multi(plan, r.tensors, db, nd, max_dense, dense)
    assert ctx.status() == 0
    plan.close()
    assert np.array_equal(slot.cpu().numpy(), w_slot) and int(nd.item()) == w_nd
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), w_sc)
    got_dense = dense.cpu().numpy().view(np.uint16)
    assert np.array_equal(got_dense[:w_nd * be], w_dense), "dense bodies differ"
    assert not got_dense[w_nd * be:].any(), "slots beyond n_dense were written"
    assert a.equal(b), "snapshot not refreshed"
    assert r.equal(b), "mixed sparse + dense reconstruction differs"
