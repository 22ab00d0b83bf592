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
