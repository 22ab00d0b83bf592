"""GPU parity for the 16-bit index coding (Sec. 3.3): srs_encode_indices and the encoded apply calls
against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth
from util import from_u16, payload_to_host, u16

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


def sparse_pair(n, positions, seed):
    rng = np.random.default_rng(seed)
    old = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    new = old.copy()
    new[positions] ^= 0x0101
    return old, new


def encoded_to_host(D, mg, an):
    return D.cpu().numpy().view(np.uint16), mg.cpu().numpy().view(np.uint32), an.cpu().numpy()


def check_encoded(got, want, counts, nchunk):
    gD, gm, ga = got
    wD, wm, wa = want
    assert np.array_equal(gm, wm), "max_gap"
    assert np.array_equal(gD, wD), "differences (including untouched slots)"
    assert np.array_equal(ga.reshape(-1)[:wa.size].reshape(wa.shape), wa), "anchors"


@pytest.mark.parametrize("n,be,cap,kind", [
    (300000, 100000, 100000, "iid1"), (300000, 100000, 100000, "iid30"), (300000, 100000, 100000, "dense"),
    (300000, 100000, 100000, "empty"), (300000, 100000, 100000, "wide"), (300000, 100000, 100000, "edge"),
    (70001, 7000, 7000, "iid1"), (1 << 20, 1 << 18, 5000, "iid1"), (5000, 5000, 4999, "iid30"),
    (1500 * 3000 + 11, 3000, 3000, "iid30"),            # 1501 buckets: two groups of the bucket interleave
])
def test_single_tensor_encode_and_encoded_apply(srs, ctx, n, be, cap, kind):
    print(f"case n={n} be={be} cap={cap} kind={kind}", flush=True)
    rng = np.random.default_rng(n + be + len(kind))
    if kind == "iid1":
        pos = np.flatnonzero(rng.random(n) < 0.01)
    elif kind == "iid30":
        pos = np.flatnonzero(rng.random(n) < 0.3)
    elif kind == "dense":
        pos = np.arange(n)
    elif kind == "empty":
        pos = np.zeros(0, np.int64)
    elif kind == "wide":      # bucket 0: one gap of exactly 32768; bucket 1: gaps of at most 32767; bucket 2: first gap wide
        pos = np.array([10, 10 + 32768, 50000, be + 32767, be + 2 * 32767, 2 * be + 40000, 2 * be + 40001])
    else:                     # "edge": first and last element of buckets and of 2048-pair chunks
        pos = np.unique(np.concatenate([[0, be - 1, be, 2 * be - 1, n - 1], np.arange(be + 100, be + 100 + 2 * 2048 + 1)]))
    old_h, new_h = sparse_pair(n, pos, seed=n)
    nb = (n + be - 1) // be
    wI, wV, wc, _ = oracle.extract(old_h.copy(), new_h, be, cap=cap)
    try:
        want = oracle.encode_indices(wI, wc, base_stride=be)
    except ValueError:
        pytest.skip("oracle rejects this payload")
    d_old, d_new, d_roll = from_u16(old_h, DEV), from_u16(new_h, DEV), from_u16(old_h, DEV)
    I, V, counts = srs.alloc_payload(nb, cap, DEV)
    D, mg, an = srs.alloc_encoded(nb, cap, DEV)
    ctx.extract(d_old, d_new, be, I, V, counts, cap)
    ctx.encode_indices(I, counts, nb, cap, be, D, mg, an)
    flags = ctx.status()
    assert flags in (0, srs.FLAG_OVERFLOW)
    check_encoded(encoded_to_host(D, mg, an), want, wc, (cap + 2047) // 2048)
    if kind == "wide":
        assert want[1].tolist() == [32768, 32767, 40000]
    # the receiver only has I for the wide buckets: poison the rest
    I_wide = I.clone()
    narrow = (mg.to(torch.int64) < 32768)
    I_wide[narrow] = -12345
    ctx.apply_encoded(d_roll, be, D, I_wide, V, counts, mg, an, cap)
    assert ctx.status() == 0
    exp = old_h.copy()
    oracle.apply(exp, be, oracle.decode_indices(want[0], wI, wc, want[1], base_stride=be), wV, wc)
    assert np.array_equal(u16(d_roll), exp)
    if int(wc.max()) <= cap:
        assert np.array_equal(exp, new_h)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
@pytest.mark.parametrize("slab", [True, False])
def test_tensor_lists_encoded_round_trip(srs, ctx, cfg, slab):
    print(f"case cfg={cfg} slab={slab}", flush=True)
    wl = synth.workload(cfg, tiny=True)
    a = synth.WeightSet(wl, DEV, slab=slab, misalign=0 if slab else 1)
    b = synth.WeightSet(wl, DEV, slab=slab, misalign=0 if slab else 2)
    r = synth.WeightSet(wl, DEV, slab=slab, misalign=0 if slab else 3)
    synth.fill_base(a, cfg + 10)
    synth.make_update(b, a, cfg + 10)
    r.copy_from(a)
    olds, news = a.to_numpy_u16(), b.to_numpy_u16()
    cap = wl.bucket_elems
    wI, wV, wc, _ = oracle.extract_multi(olds, news, a.numels, wl.bucket_elems, cap=cap)
    want = oracle.encode_indices(wI, wc)
    plan = ctx.plan(a.numels, wl.bucket_elems)
    I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
    D, mg, an = srs.alloc_encoded(plan.nbuckets, cap, DEV)
    ctx.extract_multi(plan, a.tensors, b.tensors, I, V, counts, cap)
    ctx.encode_indices(I, counts, plan.nbuckets, cap, 0, D, mg, an)
    assert ctx.status() == 0
    check_encoded(encoded_to_host(D, mg, an), want, wc, (cap + 2047) // 2048)
    I_wide = I.clone()
    I_wide[mg.to(torch.int64) < 32768] = -777
    ctx.apply_multi_encoded(plan, r.tensors, D, I_wide, V, counts, mg, an, cap)
    assert ctx.status() == 0
    plan.close()
    assert r.equal(b), "reconstruction from the encoded payload differs"


def test_unsorted_payload_is_flagged_and_kept_wide(srs, ctx):
    I = torch.tensor([[9, 3, 4, -1]], dtype=torch.int32, device=DEV)
    counts = torch.tensor([3], dtype=torch.int32, device=DEV)
    D, mg, an = srs.alloc_encoded(1, 4, DEV)
    ctx.encode_indices(I, counts, 1, 4, 0, D, mg, an)
    assert ctx.status() == srs.FLAG_BAD_INDEX
    assert int(mg.cpu().numpy().view(np.uint32)[0]) >= 32768


def test_full_size_bucket_shape(srs, ctx):
    """One 64 MiB bucket pair at 1 %: 335 k pairs, 164 chunks; everything narrow; 4 B per pair."""
    n = 2 * 33_554_432
    be = 33_554_432
    g = torch.Generator(device=DEV); g.manual_seed(5)
    old = torch.randint(-32768, 32767, (n,), dtype=torch.int16, device=DEV, generator=g).view(torch.bfloat16)
    mask = torch.rand(n, device=DEV, generator=g) < 0.01
    new = torch.where(mask, (old.view(torch.int16) ^ 1), old.view(torch.int16)).view(torch.bfloat16)
    roll = old.clone()
    old_h, new_h = u16(old), u16(new)
    cap = 423528
    wI, wV, wc, _ = oracle.extract(old_h.copy(), new_h, be, cap=cap)
    want = oracle.encode_indices(wI, wc, base_stride=be)
    I, V, counts = srs.alloc_payload(2, cap, DEV)
    D, mg, an = srs.alloc_encoded(2, cap, DEV)
    ctx.extract(old, new, be, I, V, counts, cap)
    ctx.encode_indices(I, counts, 2, cap, be, D, mg, an)
    ctx.apply_encoded(roll, be, D, torch.full_like(I, -5), V, counts, mg, an, cap)
    assert ctx.status() == 0
    check_encoded(encoded_to_host(D, mg, an), want, wc, (cap + 2047) // 2048)
    assert int(want[1].max()) < 32768
    assert np.array_equal(u16(roll), new_h)
