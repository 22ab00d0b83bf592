"""Seeded random differential test: many small tensor lists with random sizes, bucket sizes, capacities, densities,
alignments and library options, GPU against oracle, bit for bit.  Complements the hand-picked edge cases."""
import numpy as np
import pytest
import torch

import oracle
from util import assert_payload_equal, from_u16, payload_to_host, u16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def random_case(rng):
    nt = int(rng.integers(1, 9))
    kinds = rng.integers(0, 4, size=nt)
    numel = []
    for kd in kinds:
        if kd == 0:
            numel.append(int(rng.integers(0, 40)))
        elif kd == 1:
            numel.append(int(rng.integers(1, 5000)))
        elif kd == 2:
            numel.append(int(rng.integers(1, 9)) * 4096)
        else:
            numel.append(int(rng.integers(1, 120000)))
    total = sum(numel)
    be = int(rng.choice([1, 7, 64, 1000, 4096, 16384, 50001, max(total, 1), max(total, 1) + 5, int(rng.integers(1, max(total, 2)))]))
    if total // max(be, 1) > 3000:
        be = max(total // 3000, 1)                       # keep the bucket count bounded
    density = float(rng.choice([0.0, 0.001, 0.01, 0.05, 0.3, 1.0]))
    cap = int(rng.choice([be, max(1, int(be * density * 1.5) + 3), 1 + be // 7]))
    opts = (int(rng.choice([4096, 8192, 16384, 32768])), int(rng.choice([1, 2, 5, 64, 1024])), int(rng.choice([0, 8])))
    pad = [int(rng.integers(0, 8)) if rng.random() < 0.5 else 0 for _ in numel]
    return numel, be, cap, density, opts, pad


def test_random_lists_match_oracle():
    from paper_2605_07330_amd import srs
    rng = np.random.default_rng(20260527)
    ctxs = {}
    try:
        for case in range(160):
            numel, be, cap, density, opts, pad = random_case(rng)
            tag = f"case {case}: numel={numel} be={be} cap={cap} density={density} tile/interleave/refresh={opts} pad={pad}"
            print(tag, flush=True)
            olds, news = [], []
            for m in numel:
                o = rng.integers(0, 1 << 16, size=m, dtype=np.uint16)
                w = o.copy()
                pos = np.flatnonzero(rng.random(m) < density)
                w[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
                olds.append(o); news.append(w)
            wI, wV, wc, ovf = oracle.extract_multi([o.copy() for o in olds], news, numel, be, cap=cap)
            exp_roll = [o.copy() for o in olds]
            oracle.apply_multi(exp_roll, numel, be, wI, wV, wc)
            if opts not in ctxs:
                c = srs.Context(0)
                c.set_option(srs.OPT_TILE_ELEMS, opts[0]); c.set_option(srs.OPT_INTERLEAVE, opts[1])
                c.set_option(srs.OPT_REFRESH_GROUP, opts[2])
                ctxs[opts] = c
            c = ctxs[opts]

            def dev(a, p):
                return from_u16(np.concatenate([np.zeros(p, np.uint16), a]), DEV)[p:]
            d_old = [dev(o, p) for o, p in zip(olds, pad)]
            d_new = [dev(w, (p * 3) % 8) for w, p in zip(news, pad)]
            d_roll = [dev(o, (p * 5) % 8) for o, p in zip(olds, pad)]
            plan = c.plan(numel, be)
            nb = plan.nbuckets
            I, V, counts = srs.alloc_payload(max(nb, 1), cap, DEV)
            c.extract_multi(plan, d_old, d_new, I, V, counts, cap)
            c.apply_multi(plan, d_roll, I, V, counts, cap)
            flags = c.status()
            plan.close()
            assert flags == (srs.FLAG_OVERFLOW if ovf else 0), tag
            got = payload_to_host(I, V, counts)
            assert_payload_equal((got[0][:nb], got[1][:nb], got[2][:nb]), (wI, wV, wc), tag)
            for o, w, r, er in zip(d_old, news, d_roll, exp_roll):
                assert np.array_equal(u16(o), w), tag + " (snapshot)"
                assert np.array_equal(u16(r), er), tag + " (rollout)"
    finally:
        for c in ctxs.values():
            c.close()


def test_random_single_tensors_match_oracle():
    from paper_2605_07330_amd import srs
    rng = np.random.default_rng(77)
    c = srs.Context(0)
    try:
        for case in range(80):
            n = int(rng.choice([1, 2, 9, 100, 4095, 4096, 4097, 20000, 65536, 131071, int(rng.integers(1, 300000))]))
            be = int(rng.choice([1, 3, 8, 1000, 4096, 16384, n, n + 1, int(rng.integers(1, n + 1))]))
            if n // be > 3000:
                be = max(n // 3000, 1)
            density = float(rng.choice([0.0, 0.01, 0.2, 1.0]))
            c.set_option(srs.OPT_TILE_ELEMS, int(rng.choice([4096, 8192, 16384, 32768])))
            c.set_option(srs.OPT_INTERLEAVE, int(rng.choice([1, 3, 64, 1024])))
            c.set_option(srs.OPT_REFRESH_GROUP, int(rng.choice([0, 8])))
            off = int(rng.integers(0, 8)) if rng.random() < 0.5 else 0
            tag = f"case {case}: n={n} be={be} density={density} offset={off}"
            print(tag, flush=True)
            o = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
            w = o.copy()
            pos = np.flatnonzero(rng.random(n) < density)
            w[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
            want = oracle.extract(o.copy(), w, be)[:3]
            d_old = from_u16(np.concatenate([np.zeros(off, np.uint16), o]), DEV)[off:]
            d_new = from_u16(w, DEV)
            d_roll = from_u16(o, DEV)
            nb = (n + be - 1) // be
            I, V, counts = srs.alloc_payload(nb, be, DEV)
            c.extract(d_old, d_new, be, I, V, counts, be)
            c.apply(d_roll, be, I, V, counts, be)
            assert c.status() == 0, tag
            assert_payload_equal(payload_to_host(I, V, counts), want, tag)
            assert np.array_equal(u16(d_old), w) and np.array_equal(u16(d_roll), w), tag
    finally:
        c.close()


# ---------------------------------------------------------------------------------------------------------------
# The same kind of random lists through the other calls: one-byte elements, the fused cast, the cumulative set,
# the rotating-snapshot option, index coding with the encoded apply, the no-allocation extract, value coding.
# ---------------------------------------------------------------------------------------------------------------
def _optional_case_list(rng):
    nt = int(rng.integers(1, 7))
    numel = []
    for _ in range(nt):
        kd = int(rng.integers(0, 4))
        numel.append(int(rng.integers(0, 40)) if kd == 0 else int(rng.integers(1, 5000)) if kd == 1
                     else int(rng.integers(1, 9)) * 4096 if kd == 2 else int(rng.integers(1, 150000)))
    total = sum(numel)
    be = int(rng.choice([7, 64, 1000, 4096, 16384, 50001, max(total, 1), int(rng.integers(1, max(total, 2)))]))
    if total // max(be, 1) > 2000: be = max(total // 2000, 1)
    dens = float(rng.choice([0.0, 0.001, 0.01, 0.05, 0.3, 1.0]))
    return numel, be, dens

def _opt_payload(I, V, c, u8=False):
    return I.cpu().numpy(), (V.cpu().numpy() if u8 else V.cpu().numpy().view(np.uint16)), c.cpu().numpy().view(np.uint32)

def _opt_same(got, want, tag):
    for g, w, n in zip(got, want, ("I", "V", "counts")):
        assert np.array_equal(g, w), f"{tag}: {n} differ"


def test_random_lists_through_the_optional_calls():
    from paper_2605_07330_amd import srs
    rng = np.random.default_rng(20261128)
    ncases = 140
    try:
        ctxs = {}
        def ctx_for(tile, il, rg, rot=0):
            k = (tile, il, rg, rot)
            if k not in ctxs:
                c = srs.Context(0); c.set_option(srs.OPT_TILE_ELEMS, tile); c.set_option(srs.OPT_INTERLEAVE, il)
                c.set_option(srs.OPT_REFRESH_GROUP, rg); c.set_option(srs.OPT_SNAPSHOT, rot); ctxs[k] = c
            return ctxs[k]

        for case in range(ncases):
            numel, be, dens = _optional_case_list(rng)
            total = sum(numel); nb = (total + be - 1) // be
            tile = int(rng.choice([4096, 8192, 16384, 32768])); il = int(rng.choice([1, 3, 64, 1024])); rg = int(rng.choice([0, 8]))
            kind = ["u8", "cast", "cum", "rot", "enc", "noalloc", "vc"][case % 7]
            tag = f"case {case} {kind}: numel={numel} be={be} dens={dens} tile={tile} il={il} rg={rg}"
            print(tag, flush=True)
            if total == 0: continue
            cap = be
            if kind == "u8":
                if tile < 8192: tile = 8192
                c = ctx_for(tile, il, rg)
                olds = [rng.integers(0, 256, size=m, dtype=np.uint8) for m in numel]
                news = [o.copy() for o in olds]
                for w in news:
                    pos = np.flatnonzero(rng.random(w.size) < dens); w[pos] ^= rng.integers(1, 256, size=pos.size, dtype=np.uint8)
                want = oracle.extract_multi_u8([o.copy() for o in olds], news, numel, be)[:3]
                d_old = [torch.from_numpy(o.copy()).to(DEV) for o in olds]; d_new = [torch.from_numpy(w.copy()).to(DEV) for w in news]
                d_roll = [torch.from_numpy(o.copy()).to(DEV) for o in olds]
                plan = c.plan(numel, be); I, V, cnt = srs.alloc_payload_u8(nb, cap, DEV)
                c.extract_multi_u8(plan, d_old, d_new, I, V, cnt, cap); c.apply_multi_u8(plan, d_roll, I, V, cnt, cap)
                assert c.status() == 0, tag; plan.close()
                _opt_same(_opt_payload(I, V, cnt, True), want, tag)
                for o, r, w in zip(d_old, d_roll, news):
                    assert np.array_equal(o.cpu().numpy(), w) and np.array_equal(r.cpu().numpy(), w), tag
                continue
            olds = [rng.integers(0, 1 << 16, size=m, dtype=np.uint16) for m in numel]
            news = [o.copy() for o in olds]
            for w in news:
                pos = np.flatnonzero(rng.random(w.size) < dens); w[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
            if kind == "cast":
                c = ctx_for(tile, il, rg)
                # masters: arbitrary float32 patterns for a fraction, else a value that rounds back to the old weight
                masters = []
                for o in olds:
                    m = (o.astype(np.uint32) << 16)
                    pos = np.flatnonzero(rng.random(o.size) < dens)
                    m[pos] = rng.integers(0, 1 << 32, size=pos.size, dtype=np.uint64).astype(np.uint32)
                    masters.append(m.view(np.float32))
                w_or = [o.copy() for o in olds]
                want = oracle.extract_cast_multi(w_or, masters, numel, be)[:3]
                d_w = [from_u16(o, DEV) for o in olds]; d_m = [torch.from_numpy(m.view(np.int32).copy()).to(DEV).view(torch.float32) for m in masters]
                plan = c.plan(numel, be); I, V, cnt = srs.alloc_payload(nb, cap, DEV)
                c.extract_cast_multi(plan, d_w, d_m, I, V, cnt, cap)
                assert c.status() == 0, tag; plan.close()
                _opt_same(_opt_payload(I, V, cnt), want, tag)
                for d, w in zip(d_w, w_or): assert np.array_equal(u16(d), w), tag + " weights"
            elif kind == "cum":
                c = ctx_for(tile, il, rg)
                mids = [o.copy() for o in olds]
                for w in mids:
                    pos = np.flatnonzero(rng.random(w.size) < dens / 2 + 0.001); w[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
                bm = np.zeros(oracle.bitmap_words(total), np.uint32)
                oracle.mark_multi(olds, mids, numel, bm); oracle.mark_multi(mids, news, numel, bm)
                want = oracle.extract_marked_multi(news, numel, be, bm)[:3]
                d0 = [from_u16(o, DEV) for o in olds]; d1 = [from_u16(o, DEV) for o in mids]; d2 = [from_u16(o, DEV) for o in news]
                plan = c.plan(numel, be); I, V, cnt = srs.alloc_payload(nb, cap, DEV)
                dbm = torch.zeros(srs.bitmap_words(total), dtype=torch.int32, device=DEV)
                c.mark_multi(plan, d0, d1, dbm); c.mark_multi(plan, d1, d2, dbm)
                c.extract_marked_multi(plan, d2, dbm, I, V, cnt, cap)
                assert c.status() == 0, tag; plan.close()
                assert np.array_equal(dbm.cpu().numpy().view(np.uint32), bm), tag + " bitmap"
                _opt_same(_opt_payload(I, V, cnt), want, tag)
            elif kind == "rot":
                c = ctx_for(tile, il, rg, 1)
                want = oracle.extract_multi([o.copy() for o in olds], news, numel, be)[:3]
                d_old = [from_u16(o, DEV) for o in olds]; d_new = [from_u16(w, DEV) for w in news]
                plan = c.plan(numel, be); I, V, cnt = srs.alloc_payload(nb, cap, DEV)
                c.extract_multi(plan, d_old, d_new, I, V, cnt, cap)
                assert c.status() == 0, tag; plan.close()
                _opt_same(_opt_payload(I, V, cnt), want, tag)
                for d, o in zip(d_old, olds): assert np.array_equal(u16(d), o), tag + " snapshot touched"
            elif kind == "enc":
                c = ctx_for(tile, il, rg)
                wI, wV, wc, _ = oracle.extract_multi([o.copy() for o in olds], news, numel, be)
                wenc = oracle.encode_indices(wI, wc)
                d_old = [from_u16(o, DEV) for o in olds]; d_new = [from_u16(w, DEV) for w in news]; d_roll = [from_u16(o, DEV) for o in olds]
                plan = c.plan(numel, be); I, V, cnt = srs.alloc_payload(nb, cap, DEV); D, mg, an = srs.alloc_encoded(nb, cap, DEV)
                c.extract_multi(plan, d_old, d_new, I, V, cnt, cap); c.encode_indices(I, cnt, nb, cap, 0, D, mg, an)
                Iw = I.clone(); Iw[mg.to(torch.int64) < 32768] = -99
                c.apply_multi_encoded(plan, d_roll, D, Iw, V, cnt, mg, an, cap)
                assert c.status() == 0, tag; plan.close()
                assert np.array_equal(D.cpu().numpy().view(np.uint16), wenc[0]) and np.array_equal(mg.cpu().numpy().view(np.uint32), wenc[1]), tag
                for r, w in zip(d_roll, news): assert np.array_equal(u16(r), w), tag + " rollout"
            elif kind == "noalloc":
                c = ctx_for(tile, il, rg)
                o = np.concatenate(olds); w = np.concatenate(news)
                want = oracle.extract(o.copy(), w, be)[:3]
                d_o = from_u16(o, DEV); d_w = from_u16(w, DEV)
                I, V, cnt = srs.alloc_payload(nb, cap, DEV)
                c.extract_noalloc(d_o, d_w, be, I, V, cnt, cap)
                assert c.status() == 0, tag
                _opt_same(_opt_payload(I, V, cnt), want, tag); assert np.array_equal(u16(d_o), w), tag
            elif kind == "vc":
                c = ctx_for(tile, il, rg)
                wI, wV, wc, _ = oracle.extract_multi([o.copy() for o in olds], news, numel, be)
                wenc = oracle.encode_values(wV, wc)
                d_old = [from_u16(o, DEV) for o in olds]; d_new = [from_u16(w, DEV) for w in news]
                plan = c.plan(numel, be); I, V, cnt = srs.alloc_payload(nb, cap, DEV)
                c.extract_multi(plan, d_old, d_new, I, V, cnt, cap)
                enc = srs.alloc_value_stream(nb, cap, DEV); V2 = torch.full_like(V, -1)
                c.encode_values(V, cnt, nb, cap, enc); c.decode_values(enc, cnt, nb, cap, V2)
                assert c.status() == 0, tag; plan.close()
                assert np.array_equal(enc["lens"].cpu().numpy().reshape(nb, 256), wenc["lens"]), tag + " lens"
                g2 = V2.cpu().numpy().view(np.uint16)
                for b in range(nb):
                    k = int(wc[b]); assert np.array_equal(g2[b, :k], wV[b, :k]), tag + f" decoded bucket {b}"
    finally:
        for c in ctxs.values():
            c.close()
