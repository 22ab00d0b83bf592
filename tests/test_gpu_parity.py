"""GPU parity: libsrs.so (through the C ABI) against the CPU oracle, element by element, tolerance 0.

No arithmetic is done on weight values, so the bar is bit-exact: indices, values, per-bucket counts,
the untouched payload slots, the refreshed snapshot and the reconstructed weights.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth
from util import assert_payload_equal, from_u16, payload_to_host, u16

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TILES = [4096, 8192, 16384, 32768]


@pytest.fixture(scope="module")
def srs():
    from paper_2605_07330_amd import srs as m
    return m


@pytest.fixture(scope="module")
def ctx(srs):
    c = srs.Context(0)
    yield c
    c.close()


def make_pair(n, density, seed, pattern="iid"):
    """Host uint16 old/new with the requested change pattern."""
    rng = np.random.default_rng(seed)
    old = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    new = old.copy()
    if pattern == "iid":
        pos = np.flatnonzero(rng.random(n) < density)
    elif pattern == "edges":          # first / last element of tensor, and around vector, wave and tile boundaries
        cand = [0, 1, 7, 8, 9, 511, 512, 513, 4095, 4096, 4097, 16383, 16384, 16385, 32767, 32768, n - 2, n - 1]
        pos = np.array(sorted({c for c in cand if 0 <= c < n}), dtype=np.int64)
    elif pattern == "runs":           # long runs of consecutive changes (row clusters)
        pos = np.concatenate([np.arange(a, min(n, a + 5000)) for a in range(100, n, 40000)]) if n > 100 else np.arange(n)
    else:
        raise ValueError(pattern)
    if pos.size:
        delta = rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint32)
        new[pos] = ((old[pos].astype(np.uint32) + delta) & 0xFFFF).astype(np.uint16)
    return old, new


def run_single(srs, ctx, old_h, new_h, be, cap=None, offset=0):
    """extract + apply on the GPU; returns host payload, snapshot and reconstructed weights."""
    n = old_h.size
    cap = be if cap is None else cap
    nb = (n + be - 1) // be
    # offset > 0 shifts the device buffers by that many elements: 2-byte-aligned base pointers
    d_old = from_u16(np.concatenate([np.zeros(offset, np.uint16), old_h]), DEV)[offset:]
    d_new = from_u16(np.concatenate([np.zeros(offset, np.uint16), new_h]), DEV)[offset:]
    d_roll = from_u16(np.concatenate([np.zeros(offset, np.uint16), old_h]), DEV)[offset:]
    I, V, counts = srs.alloc_payload(nb, cap, DEV)
    ctx.extract(d_old, d_new, be, I, V, counts, cap)
    ctx.apply(d_roll, be, I, V, counts, cap)
    flags = ctx.status()
    return payload_to_host(I, V, counts), u16(d_old), u16(d_roll), flags


SINGLE_CASES = [
    # n, bucket_elems, density, pattern
    (1, 1, 1.0, "iid"), (7, 3, 0.5, "iid"), (8, 8, 0.5, "iid"), (9, 4, 0.5, "iid"),
    (63, 64, 0.3, "iid"), (64, 64, 0.3, "iid"), (65, 64, 0.3, "iid"), (255, 100, 0.3, "iid"),
    (2047, 2047, 0.1, "iid"), (2048, 1024, 0.1, "iid"), (2049, 2048, 0.1, "iid"),
    (16383, 16384, 0.05, "iid"), (16384, 16384, 0.05, "iid"), (16385, 16384, 0.05, "iid"),
    (100003, 4096, 0.01, "iid"), (100003, 33000, 0.01, "iid"), (100003, 100003, 0.0, "iid"),
    (100003, 20000, 1.0, "iid"), (300000, 65536, 0.01, "edges"), (300000, 100000, 0.01, "runs"),
    (1 << 20, 1 << 18, 0.01, "iid"), ((1 << 20) + 5, (1 << 18) + 3, 0.01, "iid"),
    (1 << 20, 1 << 20, 0.3, "iid"), (70001, 1000, 0.02, "iid"),
    # more than 1024 buckets: apply's bucket-interleaved order has a full group and a ragged one; 3 chunks per bucket
    (3000017, 1000, 0.02, "iid"), (2500 * 5000 + 7, 5000, 1.0, "iid"),
]


@pytest.mark.parametrize("n,be,density,pattern", SINGLE_CASES)
def test_single_tensor_matches_oracle(srs, ctx, n, be, density, pattern):
    print(f"case n={n} be={be} density={density} pattern={pattern}", flush=True)
    old_h, new_h = make_pair(n, density, seed=n * 31 + be, pattern=pattern)
    want = oracle.extract(old_h.copy(), new_h, be)[:3]
    got, snap, roll, flags = run_single(srs, ctx, old_h, new_h, be)
    assert flags == 0
    assert_payload_equal(got, want, "single")
    assert np.array_equal(snap, new_h), "snapshot not refreshed"
    assert np.array_equal(roll, new_h), "reconstruction differs from the trainer's weights"


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("offset", [0, 1, 3, 8])
def test_single_tensor_tile_sizes_and_misaligned_bases(srs, tile, offset):
    print(f"case tile={tile} offset={offset}", flush=True)
    c = srs.Context(0)
    try:
        c.set_option(srs.OPT_TILE_ELEMS, tile)
        n, be = 200003, 70001
        old_h, new_h = make_pair(n, 0.02, seed=tile + offset)
        want = oracle.extract(old_h.copy(), new_h, be)[:3]
        got, snap, roll, flags = run_single(srs, c, old_h, new_h, be, offset=offset)
        assert flags == 0
        assert_payload_equal(got, want, f"tile {tile} offset {offset}")
        assert np.array_equal(snap, new_h) and np.array_equal(roll, new_h)
    finally:
        c.close()


@pytest.mark.parametrize("interleave", [1, 3, 1024])
@pytest.mark.parametrize("rg", [0, 8])
def test_interleave_and_refresh_granularity_options(srs, interleave, rg):
    """Every workgroup-to-bucket interleave and every snapshot-refresh granularity gives the same bits."""
    print(f"case interleave={interleave} rg={rg}", flush=True)
    c = srs.Context(0)
    try:
        c.set_option(srs.OPT_INTERLEAVE, interleave)
        c.set_option(srs.OPT_REFRESH_GROUP, rg)
        c.set_option(srs.OPT_TILE_ELEMS, 4096)
        # single tensor: 11 buckets, the last one short (5 tiles instead of 9)
        n, be = 10 * 36000 + 17000, 36000
        old_h, new_h = make_pair(n, 0.03, seed=interleave * 10 + rg)
        want = oracle.extract(old_h.copy(), new_h, be)[:3]
        got, snap, roll, flags = run_single(srs, c, old_h, new_h, be)
        assert flags == 0
        assert_payload_equal(got, want, "single")
        assert np.array_equal(snap, new_h) and np.array_equal(roll, new_h)
        # tensor list
        wl = synth.workload(2, tiny=True)
        a = synth.WeightSet(wl, DEV); b = synth.WeightSet(wl, DEV); r = synth.WeightSet(wl, DEV)
        synth.fill_base(a, 3); synth.make_update(b, a, 3); r.copy_from(a)
        olds, news = a.to_numpy_u16(), b.to_numpy_u16()
        want = oracle.extract_multi(olds, news, a.numels, wl.bucket_elems)[:3]
        got, flags = run_multi(srs, c, wl, a, b, r, wl.bucket_elems)
        assert flags == 0
        assert_payload_equal(got, want, "list")
        assert a.equal(b) and r.equal(b)
    finally:
        c.close()


def test_bit_pattern_semantics(srs, ctx):
    old_h = np.array([0x0000, 0x7FC0, 0x7FC0, 0x7F80, 0x0001, 0x8000, 0x3F80] * 3, np.uint16)
    new_h = np.array([0x8000, 0x7FC0, 0x7FC1, 0xFF80, 0x0002, 0x8000, 0x3F80] * 3, np.uint16)
    want = oracle.extract(old_h.copy(), new_h, 10)[:3]
    got, snap, roll, flags = run_single(srs, ctx, old_h, new_h, 10)
    assert flags == 0
    assert_payload_equal(got, want, "bit patterns")
    assert np.array_equal(roll, new_h)


def test_config0_full_size_with_generator_ground_truth(srs, ctx):
    wl = synth.workload(0)
    a = synth.WeightSet(wl, DEV); b = synth.WeightSet(wl, DEV); r = synth.WeightSet(wl, DEV)
    for seed in (0, 1, 2):
        print(f"case config0 seed={seed}", flush=True)
        synth.fill_base(a, seed)
        nchanged, masks = synth.make_update(b, a, seed, want_masks=True)
        r.copy_from(a)
        old_h, new_h = u16(a.flat), u16(b.flat)
        want = oracle.extract(old_h.copy(), new_h, wl.bucket_elems, cap=synth.payload_capacity(wl))[:3]
        cap = synth.payload_capacity(wl)
        I, V, counts = srs.alloc_payload(wl.num_buckets, cap, DEV)
        ctx.extract(a.flat, b.flat, wl.bucket_elems, I, V, counts, cap)
        ctx.apply(r.flat, wl.bucket_elems, I, V, counts, cap)
        assert ctx.status() == 0
        got = payload_to_host(I, V, counts)
        assert_payload_equal(got, want, "config 0")
        assert int(got[2].sum()) == nchanged
        truth = torch.nonzero(masks[0]).flatten().cpu().numpy()
        cat = np.concatenate([got[0][k, :got[2][k]] for k in range(wl.num_buckets)])
        assert np.array_equal(cat, truth)
        assert a.equal(b) and r.equal(b)
        # a second extract right after finds nothing
        I2, V2, c2 = srs.alloc_payload(wl.num_buckets, cap, DEV)
        ctx.extract(a.flat, b.flat, wl.bucket_elems, I2, V2, c2, cap)
        assert ctx.status() == 0 and int(c2.sum().item()) == 0 and bool((I2 == -1).all().item())


def run_multi(srs, c, wl, a, b, r, cap):
    plan = c.plan(a.numels, wl.bucket_elems)
    I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
    c.extract_multi(plan, a.tensors, b.tensors, I, V, counts, cap)
    c.apply_multi(plan, r.tensors, I, V, counts, cap)
    flags = c.status()
    plan.close()
    return payload_to_host(I, V, counts), flags


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
@pytest.mark.parametrize("tile", [4096, 16384])
@pytest.mark.parametrize("slab,misalign", [(True, 0), (False, 0), (False, 1)])
def test_tensor_lists_tiny_model_shapes(srs, cfg, tile, slab, misalign):
    print(f"case cfg={cfg} tile={tile} slab={slab} misalign={misalign}", flush=True)
    wl = synth.workload(cfg, tiny=True)
    a = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign)
    b = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign * 2)      # old and new misaligned differently
    r = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign * 3)
    synth.fill_base(a, cfg)
    nchanged, _ = synth.make_update(b, a, cfg)
    r.copy_from(a)
    olds, news = a.to_numpy_u16(), b.to_numpy_u16()
    want = oracle.extract_multi(olds, news, a.numels, wl.bucket_elems)[:3]
    c = srs.Context(0)
    try:
        c.set_option(srs.OPT_TILE_ELEMS, tile)
        got, flags = run_multi(srs, c, wl, a, b, r, wl.bucket_elems)
    finally:
        c.close()
    assert flags == 0
    assert_payload_equal(got, want, f"cfg {cfg}")
    assert int(got[2].sum()) == nchanged
    assert a.equal(b), "snapshot not refreshed"
    assert r.equal(b), "reconstruction differs"
    # the oracle's own reconstruction from the GPU payload agrees as well
    roll = [o.copy() for o in olds]
    assert oracle.apply_multi(roll, a.numels, wl.bucket_elems, *got) == oracle.OK
    assert all(np.array_equal(x, y) for x, y in zip(roll, news))


@pytest.mark.parametrize("numel,be", [
    ([5, 1, 1, 20, 3], 7), ([5, 1, 1, 20, 3], 1), ([5, 1, 1, 20, 3], 31), ([100, 0, 50, 0, 0, 25], 64),
    ([4096] * 5 + [1] + [70000], 8192), ([1], 1), ([3, 3, 3], 3), ([40000, 7, 40000, 9, 16385], 16384),
    ([700001, 3, 1200000, 50, 999999], 1300),          # 2231 buckets: three groups of apply's bucket interleave
])
def test_tensor_lists_odd_shapes(srs, ctx, numel, be):
    print(f"case numel={numel} be={be}", flush=True)
    rng = np.random.default_rng(sum(numel) + be)
    olds, news = [], []
    for k, m in enumerate(numel):
        o, w = make_pair(m, 0.25, seed=1000 * k + m + be) if m else (np.zeros(0, np.uint16), np.zeros(0, np.uint16))
        olds.append(o); news.append(w)
    want = oracle.extract_multi([o.copy() for o in olds], news, numel, be)[:3]
    d_old = [from_u16(o, DEV) for o in olds]
    d_new = [from_u16(w, DEV) for w in news]
    d_roll = [from_u16(o, DEV) for o in olds]
    plan = ctx.plan(numel, be)
    I, V, counts = srs.alloc_payload(plan.nbuckets, be, DEV)
    ctx.extract_multi(plan, d_old, d_new, I, V, counts, be)
    ctx.apply_multi(plan, d_roll, I, V, counts, be)
    assert ctx.status() == 0
    plan.close()
    assert_payload_equal(payload_to_host(I, V, counts), want, "odd list")
    for o, r, w in zip(d_old, d_roll, news):
        assert np.array_equal(u16(o), w) and np.array_equal(u16(r), w)


def test_bucket_with_more_segments_than_the_lds_cache(srs, ctx):
    """1000 tensors of 37 elements share few buckets: apply's segment table does not fit its LDS cache."""
    numel = [37] * 1000 + [5000] + [1] * 300
    be = 20000
    rng = np.random.default_rng(12)
    olds = [rng.integers(0, 1 << 16, size=m, dtype=np.uint16) for m in numel]
    news = [o.copy() for o in olds]
    for w in news:
        w[rng.random(w.size) < 0.2] ^= 0x8001
    want = oracle.extract_multi([o.copy() for o in olds], news, numel, be)[:3]
    d_old = [from_u16(o, DEV) for o in olds]; d_new = [from_u16(w, DEV) for w in news]
    d_roll = [from_u16(o, DEV) for o in olds]; d_roll2 = [from_u16(o, DEV) for o in olds]
    plan = ctx.plan(numel, be)
    assert plan.nsegments > 1300
    I, V, counts = srs.alloc_payload(plan.nbuckets, be, DEV)
    ctx.extract_multi(plan, d_old, d_new, I, V, counts, be)
    ctx.apply_multi(plan, d_roll, I, V, counts, be)
    D, mg, an = srs.alloc_encoded(plan.nbuckets, be, DEV)
    ctx.encode_indices(I, counts, plan.nbuckets, be, 0, D, mg, an)
    ctx.apply_multi_encoded(plan, d_roll2, D, I, V, counts, mg, an, be)
    assert ctx.status() == 0
    plan.close()
    assert_payload_equal(payload_to_host(I, V, counts), want, "many segments")
    for o, r, r2, w in zip(d_old, d_roll, d_roll2, news):
        assert np.array_equal(u16(o), w) and np.array_equal(u16(r), w) and np.array_equal(u16(r2), w)


def test_capacity_overflow(srs, ctx):
    n, be, cap = 200000, 50000, 300
    old_h, new_h = make_pair(n, 0.01, seed=77)                  # ~500 changes per bucket > cap
    want_I, want_V, want_c, ovf = oracle.extract(old_h.copy(), new_h, be, cap=cap)
    assert ovf == 4
    got, snap, roll, flags = run_single(srs, ctx, old_h, new_h, be, cap=cap)
    assert flags == srs.FLAG_OVERFLOW
    assert_payload_equal(got, (want_I, want_V, want_c), "overflow")
    assert np.array_equal(snap, new_h)                          # snapshot refreshed all the same
    exp = old_h.copy()
    oracle.apply(exp, be, want_I, want_V, want_c)
    assert np.array_equal(roll, exp)                            # only the stored pairs were applied
    # exactly full is not an overflow
    cmax = int(want_c.max())
    got2, _, roll2, flags2 = run_single(srs, ctx, old_h, new_h, be, cap=cmax)
    assert flags2 == 0 and np.array_equal(roll2, new_h)


def test_apply_skips_and_flags_bad_indices(srs, ctx):
    n, be, cap = 100, 50, 3
    w = from_u16(np.zeros(n, np.uint16), DEV)
    I = torch.tensor([[3, 60, -1], [50, 100, 99]], dtype=torch.int32, device=DEV)
    V = torch.tensor([[7, 8, 9], [1, 2, 3]], dtype=torch.int16, device=DEV)
    counts = torch.tensor([3, 3], dtype=torch.int32, device=DEV)
    ctx.apply(w, be, I, V, counts, cap)
    assert ctx.status() == srs.FLAG_BAD_INDEX
    exp = np.zeros(n, np.uint16); exp[3] = 7; exp[50] = 1; exp[99] = 3
    assert np.array_equal(u16(w), exp)
    ws = [from_u16(np.zeros(60, np.uint16), DEV), from_u16(np.zeros(40, np.uint16), DEV)]
    plan = ctx.plan([60, 40], 50)
    I = torch.tensor([[3, 50, 49], [10, 49, 0]], dtype=torch.int32, device=DEV)
    ctx.apply_multi(plan, ws, I, V, counts, cap)
    assert ctx.status() == srs.FLAG_BAD_INDEX
    plan.close()
    e0 = np.zeros(60, np.uint16); e1 = np.zeros(40, np.uint16)
    e0[3] = 7; e0[49] = 9; e0[50] = 3; e1[0] = 1; e1[39] = 2
    assert np.array_equal(u16(ws[0]), e0) and np.array_equal(u16(ws[1]), e1)


def test_invalid_arguments_are_rejected_before_launch(srs, ctx):
    t = from_u16(np.zeros(64, np.uint16), DEV)
    I, V, counts = srs.alloc_payload(1, 64, DEV)
    for be, cap in [(0, 64), (64, 0), (1 << 31, 64)]:
        with pytest.raises(srs.SrsError) as e:
            ctx.extract(t, t.clone(), be, I, V, counts, cap)
        assert e.value.code == srs.ERR_INVALID
    with pytest.raises(srs.SrsError):
        ctx.plan([1 << 31], 64)
    with pytest.raises(srs.SrsError):
        ctx.set_option(srs.OPT_TILE_ELEMS, 1000)
    for opt, bad in [(srs.OPT_REFRESH_GROUP, 4), (srs.OPT_REFRESH_GROUP, 16), (srs.OPT_INTERLEAVE, 0), (srs.OPT_INTERLEAVE, 5000),
                     (srs.OPT_SNAPSHOT, 3), (srs.OPT_SPIN_LIMIT, 0), (99, 1)]:
        with pytest.raises(srs.SrsError) as e:
            ctx.set_option(opt, bad)
        assert e.value.code == srs.ERR_INVALID
    for opt, good in [(srs.OPT_REFRESH_GROUP, 0), (srs.OPT_REFRESH_GROUP, 8), (srs.OPT_SNAPSHOT, 0)]:
        ctx.set_option(opt, good)
    # empty inputs are fine and write nothing
    e = torch.empty(0, dtype=torch.bfloat16, device=DEV)
    ctx.extract(e, e.clone(), 64, I, V, counts, 64)
    plan = ctx.plan([], 64)
    assert plan.nbuckets == 0
    ctx.extract_multi(plan, [], [], I, V, counts, 64)
    ctx.apply_multi(plan, [], I, V, counts, 64)
    assert ctx.status() == 0 and bool((I == -1).all().item())
    plan.close()


def test_null_tensor_pointers_are_rejected_before_launch(srs, ctx):
    """A tensor with elements needs its pointers; one without elements may carry anything."""
    numel = [100, 0, 60]
    olds = [from_u16(np.zeros(m, np.uint16), DEV) for m in numel]
    news = [from_u16(np.ones(m, np.uint16), DEV) for m in numel]
    plan = ctx.plan(numel, 64)
    I, V, counts = srs.alloc_payload(plan.nbuckets, 64, DEV)
    pairs = ctx.bind_pairs(plan, olds, news)
    weights = ctx.bind_weights(plan, olds)
    pairs[1].old_snapshot = None; pairs[1].new_w = None; weights[1].weights = None     # the empty tensor
    ctx.extract_multi(plan, None, None, I, V, counts, 64, pairs=pairs)
    ctx.apply_multi(plan, None, I, V, counts, 64, tensors=weights)
    assert ctx.status() == 0 and counts.tolist() == [64, 64, 32]
    keep = pairs[2].new_w
    pairs[2].new_w = None
    with pytest.raises(srs.SrsError) as e:
        ctx.extract_multi(plan, None, None, I, V, counts, 64, pairs=pairs)
    assert e.value.code == srs.ERR_INVALID
    pairs[2].new_w = keep
    pairs[0].old_snapshot = None
    with pytest.raises(srs.SrsError) as e:
        ctx.extract_multi(plan, None, None, I, V, counts, 64, pairs=pairs)
    assert e.value.code == srs.ERR_INVALID
    weights[2].weights = None
    with pytest.raises(srs.SrsError) as e:
        ctx.apply_multi(plan, None, I, V, counts, 64, tensors=weights)
    assert e.value.code == srs.ERR_INVALID
    assert ctx.status() == 0
    plan.close()


def test_repeated_runs_are_bit_identical(srs, ctx):
    """The look-back chain is the only cross-workgroup interaction: 20 runs must agree exactly."""
    n, be = 3_000_017, 1_000_003
    old_h, new_h = make_pair(n, 0.01, seed=5)
    want = oracle.extract(old_h.copy(), new_h, be, cap=20000)[:3]
    d_new = from_u16(new_h, DEV)
    for it in range(20):
        d_old = from_u16(old_h, DEV)
        I, V, counts = srs.alloc_payload((n + be - 1) // be, 20000, DEV)
        ctx.extract(d_old, d_new, be, I, V, counts, 20000)
        assert ctx.status() == 0
        assert_payload_equal(payload_to_host(I, V, counts), want, f"run {it}")


def test_chain_of_updates(srs, ctx):
    wl = synth.workload(2, tiny=True)
    snap = synth.WeightSet(wl, DEV, slab=False); cur = synth.WeightSet(wl, DEV, slab=False)
    nxt = synth.WeightSet(wl, DEV, slab=False); roll = synth.WeightSet(wl, DEV, slab=False)
    synth.fill_base(snap, 11); cur.copy_from(snap); roll.copy_from(snap)
    plan = ctx.plan(snap.numels, wl.bucket_elems)
    cap = wl.bucket_elems
    for step in range(1, 5):
        synth.make_update(nxt, cur, 11, step=step)
        cur.copy_from(nxt)
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        ctx.extract_multi(plan, snap.tensors, cur.tensors, I, V, counts, cap)
        ctx.apply_multi(plan, roll.tensors, I, V, counts, cap)
        assert ctx.status() == 0
        assert snap.equal(cur) and roll.equal(cur)
    plan.close()


def test_bounded_look_back_exits_when_starved(srs):
    """A spin limit of 1 may make tiles give up: the kernel must still finish, and either the
    result is exact or the time-out flag says it is not."""
    c = srs.Context(0)
    try:
        c.set_option(srs.OPT_SPIN_LIMIT, 1)
        c.set_option(srs.OPT_TILE_ELEMS, 4096)
        n, be = 2_000_000, 1_000_000
        old_h, new_h = make_pair(n, 0.01, seed=9)
        want = oracle.extract(old_h.copy(), new_h, be, cap=20000)[:3]
        d_old, d_new = from_u16(old_h, DEV), from_u16(new_h, DEV)
        I, V, counts = srs.alloc_payload(2, 20000, DEV)
        c.extract(d_old, d_new, be, I, V, counts, 20000)
        flags = c.status()
        assert flags in (0, srs.FLAG_TIMEOUT)
        if flags == 0:
            assert_payload_equal(payload_to_host(I, V, counts), want, "spin limit 1")
        assert np.array_equal(u16(d_old), new_h)        # the refresh does not depend on the chain
    finally:
        c.close()


def test_two_contexts_on_two_streams_run_concurrently(srs):
    """Two extracts in flight at once compete for workgroup slots.  A tile only ever waits for tiles that are
    already running (ticket order inside a bucket is start order), so neither launch can starve the other;
    the bounded wait would raise SRS_FLAG_TIMEOUT instead of hanging if that reasoning were wrong."""
    n, be, cap = 24_000_011, 3_000_007, 60_000
    cases = []
    for s in range(2):
        old_h, new_h = make_pair(n, 0.01, seed=100 + s)
        cases.append((old_h, new_h, oracle.extract(old_h.copy(), new_h, be, cap=cap)[:3]))
    ctxs = [srs.Context(0), srs.Context(0)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    nb = (n + be - 1) // be
    try:
        for c in ctxs:
            c.set_option(srs.OPT_SPIN_LIMIT, 1 << 20)
            c.set_option(srs.OPT_TILE_ELEMS, 4096)          # many small tiles: more chain traffic, more waiting
        d_new = [from_u16(c[1], DEV) for c in cases]
        for rep in range(10):
            d_old = [from_u16(c[0], DEV) for c in cases]
            bufs = [srs.alloc_payload(nb, cap, DEV) for _ in cases]
            torch.cuda.synchronize()
            for k in range(2):
                with torch.cuda.stream(streams[k]):
                    ctxs[k].extract(d_old[k], d_new[k], be, *bufs[k], cap)
            torch.cuda.synchronize()
            for k in range(2):
                assert ctxs[k].status(streams[k]) == 0, f"rep {rep} stream {k}"
                assert_payload_equal(payload_to_host(*bufs[k]), cases[k][2], f"rep {rep} stream {k}")
                assert np.array_equal(u16(d_old[k]), cases[k][1])
    finally:
        for c in ctxs:
            c.close()


# ---------------------------------------------------------------------------------------------------------------
# More than 65,536 buckets: the per-bucket ticket counters are then packed 4 bytes apart instead of 256, and the
# extract, apply, encode and encoded-apply grids all exceed 65,536 workgroups with one-element tiles.
# ---------------------------------------------------------------------------------------------------------------
def _encoded_host(D, mg, an):
    return D.cpu().numpy().view(np.uint16), mg.cpu().numpy().view(np.uint32), an.cpu().numpy()


def _check_encoded(got, want):
    gD, gm, ga = got
    wD, wm, wa = want
    assert np.array_equal(gm, wm), "max_gap"
    assert np.array_equal(gD, wD), "differences (including untouched slots)"
    assert np.array_equal(ga.reshape(-1)[:wa.size].reshape(wa.shape), wa), "anchors"


@pytest.mark.parametrize("n,be,density", [(70_001, 1, 0.3), (140_003, 2, 0.4)])
def test_single_tensor_more_than_65536_buckets(srs, ctx, n, be, density):
    print(f"case many buckets single n={n} be={be}", flush=True)
    nb = (n + be - 1) // be
    assert nb > 65536
    old_h, new_h = make_pair(n, density, seed=n + be)
    wI, wV, wc, _ = oracle.extract(old_h.copy(), new_h, be)
    got, snap, roll, flags = run_single(srs, ctx, old_h, new_h, be)
    assert flags == 0
    assert_payload_equal(got, (wI, wV, wc), "many buckets, single")
    assert np.array_equal(snap, new_h) and np.array_equal(roll, new_h)
    # index coding of the same payload and the encoded apply
    want = oracle.encode_indices(wI, wc, base_stride=be)
    d_old, d_new, d_roll = from_u16(old_h, DEV), from_u16(new_h, DEV), from_u16(old_h, DEV)
    I, V, counts = srs.alloc_payload(nb, be, DEV)
    D, mg, an = srs.alloc_encoded(nb, be, DEV)
    ctx.extract(d_old, d_new, be, I, V, counts, be)
    ctx.encode_indices(I, counts, nb, be, be, D, mg, an)
    assert ctx.status() == 0
    _check_encoded(_encoded_host(D, mg, an), want)
    I_wide = I.clone()
    I_wide[mg.to(torch.int64) < 32768] = -4242          # the receiver has I only for wide buckets (none here)
    ctx.apply_encoded(d_roll, be, D, I_wide, V, counts, mg, an, be)
    assert ctx.status() == 0
    assert np.array_equal(u16(d_roll), new_h)


def test_tensor_list_more_than_65536_buckets(srs, ctx):
    numels = [50_001, 3, 0, 90_001]                        # odd sizes: tensors straddle the two-element buckets
    be = 2
    total = sum(numels)
    nb = (total + be - 1) // be
    assert nb > 65536
    print(f"case many buckets list numels={numels} be={be}", flush=True)
    pairs = [make_pair(max(k, 1), 0.35, seed=900 + i) for i, k in enumerate(numels)]
    olds = [p[0][:k].copy() for p, k in zip(pairs, numels)]
    news = [p[1][:k].copy() for p, k in zip(pairs, numels)]
    wI, wV, wc, _ = oracle.extract_multi([o.copy() for o in olds], news, numels, be)
    want = oracle.encode_indices(wI, wc)
    d_old = [from_u16(o, DEV) for o in olds]
    d_new = [from_u16(x, DEV) for x in news]
    d_roll = [from_u16(o, DEV) for o in olds]
    d_roll2 = [from_u16(o, DEV) for o in olds]
    plan = ctx.plan(numels, be)
    assert plan.nbuckets == nb
    I, V, counts = srs.alloc_payload(nb, be, DEV)
    D, mg, an = srs.alloc_encoded(nb, be, DEV)
    ctx.extract_multi(plan, d_old, d_new, I, V, counts, be)
    ctx.apply_multi(plan, d_roll, I, V, counts, be)
    ctx.encode_indices(I, counts, nb, be, 0, D, mg, an)
    assert ctx.status() == 0
    assert_payload_equal(payload_to_host(I, V, counts), (wI, wV, wc), "many buckets, list")
    _check_encoded(_encoded_host(D, mg, an), want)
    I_wide = I.clone()
    I_wide[mg.to(torch.int64) < 32768] = -4242
    ctx.apply_multi_encoded(plan, d_roll2, D, I_wide, V, counts, mg, an, be)
    assert ctx.status() == 0
    plan.close()
    for k in range(len(numels)):
        if numels[k]:
            assert np.array_equal(u16(d_old[k]), news[k]), f"snapshot of tensor {k}"
            assert np.array_equal(u16(d_roll[k]), news[k]), f"reconstruction of tensor {k}"
            assert np.array_equal(u16(d_roll2[k]), news[k]), f"encoded reconstruction of tensor {k}"


def test_one_byte_elements_more_than_65536_buckets(srs, ctx):
    n, be = 70_001, 1
    nb = n
    print(f"case many buckets u8 n={n} be={be}", flush=True)
    rng = np.random.default_rng(4711)
    old_h = rng.integers(0, 256, size=n, dtype=np.uint8)
    new_h = old_h.copy()
    pos = np.flatnonzero(rng.random(n) < 0.3)
    new_h[pos] = ((old_h[pos].astype(np.uint32) + rng.integers(1, 256, size=pos.size, dtype=np.uint32)) & 0xFF).astype(np.uint8)
    wI, wV, wc, _ = oracle.extract_u8(old_h.copy(), new_h, be)
    d_old, d_new, d_roll = (torch.from_numpy(x.copy()).to(DEV) for x in (old_h, new_h, old_h))
    I, V, counts = srs.alloc_payload_u8(nb, be, DEV)
    ctx.extract_u8(d_old, d_new, be, I, V, counts, be)
    ctx.apply_u8(d_roll, be, I, V, counts, be)
    assert ctx.status() == 0
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), wc)
    assert np.array_equal(I.cpu().numpy(), wI) and np.array_equal(V.cpu().numpy(), wV)
    assert np.array_equal(d_old.cpu().numpy(), new_h) and np.array_equal(d_roll.cpu().numpy(), new_h)
