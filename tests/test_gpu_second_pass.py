"""GPU parity of the second-pass snapshot refresh (SRS_OPT_SNAPSHOT = 2) against the CPU oracle.

Under this option the scan leaves the snapshot alone and the same call then scatters the payload into it (Alg. 1's
W_prev <- W after the diff instead of inside it); a bucket whose payload overflowed cap is copied whole.  What the
caller sees must be what the default gives: the oracle's payload, counts and flags, element by element, and a snapshot
bit-identical to the new weights -- also for overflowing buckets, unaligned tensors, ragged tiles, one-byte elements,
very many buckets, and through the no-allocation entry point.
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


def second_pass_ctx(srs, tile=None, interleave=None):
    c = srs.Context(0)
    c.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_SECOND_PASS)
    if tile:
        c.set_option(srs.OPT_TILE_ELEMS, tile)
    if interleave:
        c.set_option(srs.OPT_INTERLEAVE, interleave)
    return c


def make_pair(n, density, seed, bits=16):
    rng = np.random.default_rng(seed)
    dt = np.uint16 if bits == 16 else np.uint8
    old = rng.integers(0, 1 << bits, size=n, dtype=dt)
    new = old.copy()
    pos = np.flatnonzero(rng.random(n) < density)
    new[pos] ^= rng.integers(1, 1 << bits, size=pos.size, dtype=dt)
    return old, new


SINGLE = [(1, 1, 1.0), (9, 4, 0.5), (65, 64, 0.3), (2049, 2048, 0.1), (16385, 16384, 0.05), (100003, 4096, 0.01),
          (100003, 100003, 0.0), (100003, 20000, 1.0), ((1 << 20) + 5, (1 << 18) + 3, 0.01), (3000017, 1000, 0.02),
          (1 << 21, 1 << 19, 0.0007)]


@pytest.mark.parametrize("n,be,density", SINGLE)
@pytest.mark.parametrize("offset", [0, 3])
def test_single_tensor(srs, n, be, density, offset):
    print(f"case n={n} be={be} density={density} offset={offset}", flush=True)
    old_h, new_h = make_pair(n, density, seed=n + 7 * be + offset)
    want = oracle.extract(old_h.copy(), new_h, be)[:3]
    nb = (n + be - 1) // be
    d_old = from_u16(np.concatenate([np.zeros(offset, np.uint16), old_h]), DEV)[offset:]
    d_new = from_u16(np.concatenate([np.zeros(offset, np.uint16), new_h]), DEV)[offset:]
    c = second_pass_ctx(srs, tile=[4096, 32768][offset % 2])
    try:
        I, V, counts = srs.alloc_payload(nb, be, DEV)
        c.extract(d_old, d_new, be, I, V, counts, be)
        assert c.status() == 0
    finally:
        c.close()
    assert_payload_equal(payload_to_host(I, V, counts), want, "second pass, single")
    assert np.array_equal(u16(d_old), new_h), "snapshot not refreshed"
    assert np.array_equal(u16(d_new), new_h), "new weights were written"


@pytest.mark.parametrize("offset", [0, 1])
def test_single_tensor_with_overflowing_buckets(srs, offset):
    """Buckets 0 and 2 change in 3 % of their elements and overflow cap, 1 and 3 in 0.1 % and fit; the last is ragged."""
    be, cap = 50000, 300
    n = 4 * be + 12345
    rng = np.random.default_rng(5 + offset)
    old_h = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    new_h = old_h.copy()
    dens = np.repeat([0.03, 0.001, 0.03, 0.001, 0.05], be)[:n]
    pos = np.flatnonzero(rng.random(n) < dens)
    new_h[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
    wI, wV, wc, novf = oracle.extract(old_h.copy(), new_h, be, cap=cap)
    assert novf == 3 and wc[1] <= cap and wc[3] <= cap
    d_old = from_u16(np.concatenate([np.zeros(offset, np.uint16), old_h]), DEV)[offset:]
    d_new = from_u16(np.concatenate([np.zeros(offset, np.uint16), new_h]), DEV)[offset:]
    c = second_pass_ctx(srs)
    try:
        I, V, counts = srs.alloc_payload(5, cap, DEV)
        c.extract(d_old, d_new, be, I, V, counts, cap)
        assert c.status() == srs.FLAG_OVERFLOW
    finally:
        c.close()
    assert_payload_equal(payload_to_host(I, V, counts), (wI, wV, wc), "second pass, overflow")
    assert np.array_equal(u16(d_old), new_h), "snapshot of an overflowing bucket not brought up to date"


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
@pytest.mark.parametrize("slab,misalign", [(True, 0), (False, 1)])
def test_tensor_lists_tiny_model_shapes(srs, cfg, slab, misalign):
    print(f"case cfg={cfg} slab={slab} misalign={misalign}", flush=True)
    wl = synth.workload(cfg, tiny=True)
    a = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign)
    b = synth.WeightSet(wl, DEV, slab=slab, misalign=misalign * 2)
    synth.fill_base(a, cfg)
    nchanged, _ = synth.make_update(b, a, cfg)
    olds, news = a.to_numpy_u16(), b.to_numpy_u16()
    want = oracle.extract_multi(olds, news, a.numels, wl.bucket_elems)[:3]
    c = second_pass_ctx(srs, tile=[4096, 16384][cfg % 2], interleave=[3, 256][cfg % 2])
    try:
        plan = c.plan(a.numels, wl.bucket_elems)
        I, V, counts = srs.alloc_payload(plan.nbuckets, wl.bucket_elems, DEV)
        c.extract_multi(plan, a.tensors, b.tensors, I, V, counts, wl.bucket_elems)
        assert c.status() == 0
        plan.close()
    finally:
        c.close()
    got = payload_to_host(I, V, counts)
    assert_payload_equal(got, want, f"second pass, cfg {cfg}")
    assert int(got[2].sum()) == nchanged
    assert a.equal(b), "snapshot not refreshed"
    assert all(np.array_equal(x, y) for x, y in zip(b.to_numpy_u16(), news)), "new weights were written"


def _list_case(numel, be, cap, dens_of_bucket, seed, bits=16):
    """Host lists whose change density depends on the bucket an element falls into."""
    rng = np.random.default_rng(seed)
    dt = np.uint16 if bits == 16 else np.uint8
    total = sum(numel)
    flat_old = rng.integers(0, 1 << bits, size=total, dtype=dt)
    flat_new = flat_old.copy()
    dens = np.asarray(dens_of_bucket, dtype=np.float64)[np.arange(total) // be]
    pos = np.flatnonzero(rng.random(total) < dens)
    flat_new[pos] ^= rng.integers(1, 1 << bits, size=pos.size, dtype=dt)
    cuts = np.cumsum([0] + list(numel))
    olds = [flat_old[cuts[k]:cuts[k + 1]].copy() for k in range(len(numel))]
    news = [flat_new[cuts[k]:cuts[k + 1]].copy() for k in range(len(numel))]
    return olds, news


def test_tensor_list_with_overflowing_buckets_and_many_segments(srs):
    """1,301 tensors, most of them tiny and at odd addresses: buckets with more segments than the scatter's LDS table,
    some of them overflowing cap."""
    numel = [37] * 1000 + [50000] + [1] * 300 + [123457]
    be, cap = 20000, 400
    nb = (sum(numel) + be - 1) // be
    dens = [0.05 if b % 3 == 0 else 0.004 for b in range(nb)]
    olds, news = _list_case(numel, be, cap, dens, seed=31)
    wI, wV, wc, novf = oracle.extract_multi([o.copy() for o in olds], news, numel, be, cap=cap)
    assert 0 < novf < nb
    d_old = [from_u16(o, DEV) for o in olds]
    d_new = [from_u16(w, DEV) for w in news]
    c = second_pass_ctx(srs)
    try:
        plan = c.plan(numel, be)
        assert plan.nsegments > 1300
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        c.extract_multi(plan, d_old, d_new, I, V, counts, cap)
        assert c.status() == srs.FLAG_OVERFLOW
        plan.close()
    finally:
        c.close()
    assert_payload_equal(payload_to_host(I, V, counts), (wI, wV, wc), "second pass, list overflow")
    for k, (o, w) in enumerate(zip(d_old, news)):
        assert np.array_equal(u16(o), w), f"snapshot of tensor {k} not brought up to date"


def test_one_byte_elements(srs):
    numel = [40000, 7, 0, 65536, 9, 100001]
    be, cap = 16384, 500
    nb = (sum(numel) + be - 1) // be
    dens = [0.1 if b % 4 == 1 else 0.002 for b in range(nb)]
    olds, news = _list_case(numel, be, cap, dens, seed=8, bits=8)
    wI, wV, wc, novf = oracle.extract_multi_u8([o.copy() for o in olds], news, numel, be, cap=cap)
    assert 0 < novf < nb
    d_old = [torch.from_numpy(o.copy()).to(DEV) for o in olds]
    d_new = [torch.from_numpy(w.copy()).to(DEV) for w in news]
    c = second_pass_ctx(srs, tile=8192)
    try:
        plan = c.plan(numel, be)
        I, V, counts = srs.alloc_payload_u8(plan.nbuckets, cap, DEV)
        c.extract_multi_u8(plan, d_old, d_new, I, V, counts, cap)
        assert c.status() == srs.FLAG_OVERFLOW
        plan.close()
        got = (I.cpu().numpy(), V.cpu().numpy(), counts.cpu().numpy().view(np.uint32))
        assert_payload_equal(got, (wI, wV, wc), "second pass, one-byte list")
        for o, w in zip(d_old, news):
            assert np.array_equal(o.cpu().numpy(), w)
        # single tensor, one byte, nothing overflows
        o1, w1 = make_pair(300007, 0.003, seed=9, bits=8)
        want = oracle.extract_u8(o1.copy(), w1, 70000)[:3]
        d_o, d_w = torch.from_numpy(o1.copy()).to(DEV), torch.from_numpy(w1.copy()).to(DEV)
        I, V, counts = srs.alloc_payload_u8(5, 70000, DEV)
        c.extract_u8(d_o, d_w, 70000, I, V, counts, 70000)
        assert c.status() == 0
        assert_payload_equal((I.cpu().numpy(), V.cpu().numpy(), counts.cpu().numpy().view(np.uint32)), want, "u8 single")
        assert np.array_equal(d_o.cpu().numpy(), w1)
    finally:
        c.close()


def test_more_than_65536_buckets_and_the_no_allocation_entry_point(srs):
    n, be = 70001, 1
    old_h, new_h = make_pair(n, 0.4, seed=3)
    want = oracle.extract(old_h.copy(), new_h, be)[:3]
    c = second_pass_ctx(srs)
    try:
        for entry in ("extract", "extract_noalloc"):
            d_old, d_new = from_u16(old_h, DEV), from_u16(new_h, DEV)
            I, V, counts = srs.alloc_payload(n, 1, DEV)
            getattr(c, entry)(d_old, d_new, be, I, V, counts, 1)
            assert c.status() == 0
            assert_payload_equal(payload_to_host(I, V, counts), want, entry)
            assert np.array_equal(u16(d_old), new_h), entry
    finally:
        c.close()


def test_chain_of_synchronisations_matches_the_default_mode(srs):
    """Five updates in a row through both modes: same payloads, same snapshots after every step."""
    n, be = 700001, 65536
    nb = (n + be - 1) // be
    rng = np.random.default_rng(77)
    w = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    c0, c2 = srs.Context(0), second_pass_ctx(srs)
    try:
        s0, s2 = from_u16(w, DEV), from_u16(w, DEV)
        for step in range(5):
            pos = np.flatnonzero(rng.random(n) < [0.0005, 0.01, 0.0, 0.2, 0.003][step])
            w = w.copy(); w[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
            d_new = from_u16(w, DEV)
            out = []
            for c, s in ((c0, s0), (c2, s2)):
                I, V, counts = srs.alloc_payload(nb, be, DEV)
                c.extract(s, d_new, be, I, V, counts, be)
                assert c.status() == 0
                out.append(payload_to_host(I, V, counts))
                assert np.array_equal(u16(s), w), f"step {step}"
            assert_payload_equal(out[1], out[0], f"step {step}")
            assert int(out[0][2].sum()) == pos.size
    finally:
        c0.close(); c2.close()


def test_random_lists(srs):
    """Random tensor lists, bucket sizes, tiles, densities and capacities (so that some buckets overflow)."""
    rng = np.random.default_rng(2605)
    ctxs = {}
    try:
        for case in range(60):
            nt = int(rng.integers(1, 7))
            numel = []
            for _ in range(nt):
                kd = int(rng.integers(0, 4))
                numel.append(int(rng.integers(0, 40)) if kd == 0 else int(rng.integers(1, 5000)) if kd == 1
                             else int(rng.integers(1, 9)) * 4096 if kd == 2 else int(rng.integers(1, 150000)))
            total = sum(numel)
            if total == 0:
                continue
            be = int(rng.choice([7, 64, 1000, 4096, 16384, 50001, total, int(rng.integers(1, total + 1))]))
            if total // be > 2000:
                be = max(total // 2000, 1)
            nb = (total + be - 1) // be
            dens = float(rng.choice([0.0, 0.001, 0.01, 0.05, 0.3, 1.0]))
            cap = int(rng.choice([be, max(1, int(be * dens * 0.9)), max(1, be // 3)]))
            bits = 8 if case % 3 == 2 else 16
            tile = int(rng.choice([8192, 16384, 32768] if bits == 8 else [4096, 8192, 16384, 32768]))
            il = int(rng.choice([1, 3, 64, 1024]))
            tag = f"case {case}: numel={numel} be={be} cap={cap} dens={dens} bits={bits} tile={tile} il={il}"
            print(tag, flush=True)
            if (tile, il) not in ctxs:
                ctxs[(tile, il)] = second_pass_ctx(srs, tile=tile, interleave=il)
            c = ctxs[(tile, il)]
            olds, news = _list_case(numel, be, cap, [dens] * nb, seed=case, bits=bits)
            plan = c.plan(numel, be)
            if bits == 8:
                wI, wV, wc, novf = oracle.extract_multi_u8([o.copy() for o in olds], news, numel, be, cap=cap)
                d_old = [torch.from_numpy(o.copy()).to(DEV) for o in olds]
                d_new = [torch.from_numpy(x.copy()).to(DEV) for x in news]
                I, V, counts = srs.alloc_payload_u8(nb, cap, DEV)
                c.extract_multi_u8(plan, d_old, d_new, I, V, counts, cap)
                got = (I.cpu().numpy(), V.cpu().numpy(), counts.cpu().numpy().view(np.uint32))
                snaps = [d.cpu().numpy() for d in d_old]
            else:
                wI, wV, wc, novf = oracle.extract_multi([o.copy() for o in olds], news, numel, be, cap=cap)
                d_old = [from_u16(o, DEV) for o in olds]
                d_new = [from_u16(x, DEV) for x in news]
                I, V, counts = srs.alloc_payload(nb, cap, DEV)
                c.extract_multi(plan, d_old, d_new, I, V, counts, cap)
                got = payload_to_host(I, V, counts)
                snaps = [u16(d) for d in d_old]
            assert c.status() == (srs.FLAG_OVERFLOW if novf else 0), tag
            plan.close()
            assert_payload_equal(got, (wI, wV, wc), tag)
            for s, x in zip(snaps, news):
                assert np.array_equal(s, x), tag + ": snapshot"
    finally:
        for c in ctxs.values():
            c.close()
