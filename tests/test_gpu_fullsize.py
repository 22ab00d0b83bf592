"""Full-size parity on the benchmark workloads (Qwen3-8B / 30B-A3B / 30B-A3B skewed / 32B shaped),
in the launch configuration bench.py times.

The oracle cannot redo 30 G elements inside a test, so each workload is checked in two ways:
  * sampled buckets (first, last, around tensor boundaries, and a seeded random draw) are copied to
    the host BEFORE the GPU run, extracted and applied by the oracle, and compared element by
    element with the GPU payload and with the GPU's reconstructed weights for those buckets;
  * properties that hold at any size are checked over the whole set on the device: the sum of the
    counts equals the generator's number of changed elements, indices ascend strictly and stay
    inside their bucket, the snapshot and the rollout copy both equal the new weights bit for bit
    (the tensor-by-tensor comparison of the paper's Sec. 4.2 protocol), no device flag is raised.
"""
import gc
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HOST_THREADS = max(1, min(16, os.cpu_count() or 1))       # a one-GPU machine's share of host cores


def bucket_segments(numels, be, b):
    """(tensor, offset, length) runs of bucket b of the packed list -- plain bookkeeping."""
    lo, hi, g, out = b * be, (b + 1) * be, 0, []
    for k, m in enumerate(numels):
        s, e = max(g, lo), min(g + m, hi)
        if s < e:
            out.append((k, s - g, e - s))
        g += m
    return out


def sample_buckets(wl, count, seed):
    nb, be = wl.num_buckets, wl.bucket_elems
    picks = {0, 1, nb - 2, nb - 1}
    g = 0
    for t in wl.tensors[:3] + wl.tensors[-2:]:        # buckets that hold the ends of the largest tensors
        g0 = g
        g += t.numel
        picks.update({g0 // be, (g - 1) // be})
    # a bucket in the middle of the list, where many small tensors share one bucket (expert weights)
    picks.add(nb // 2)
    rng = np.random.default_rng(seed)
    picks.update(int(x) for x in rng.integers(0, nb, size=max(0, count - len(picks))))
    return sorted(p for p in picks if 0 <= p < nb)


def host_slices(ws, segs):
    out = []
    for k, off, ln in segs:
        t = ws.tensors[k][off:off + ln]
        out.append(t.view(torch.int16).cpu().numpy().view(np.uint16).copy())
    return out


def check_workload(srs, wl, S, W1, R, nchanged, seed, nsample, second_pass=False):
    numels = S.numels
    be = wl.bucket_elems
    ctx = srs.Context(0)
    try:
        if second_pass:                                  # the configuration bench.py times this mode in
            ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_SECOND_PASS)
            ctx.set_option(srs.OPT_INTERLEAVE, 256)
        plan = ctx.plan(numels, be)
        assert plan.nbuckets == wl.num_buckets and plan.total == wl.numel
        cap = (synth.payload_capacity(wl) + 7) // 8 * 8
        I = torch.full((plan.nbuckets, cap), -1, dtype=torch.int32, device=DEV)
        V = torch.full((plan.nbuckets, cap), -1, dtype=torch.int16, device=DEV)
        counts = torch.zeros(plan.nbuckets, dtype=torch.int32, device=DEV)

        picks = sample_buckets(wl, nsample, seed)
        before = {}
        for b in picks:                                  # host copies taken before the GPU touches anything
            segs = bucket_segments(numels, be, b)
            before[b] = (segs, host_slices(S, segs), host_slices(W1, segs))
        print(f"  {wl.name}: {len(picks)} sampled buckets copied; running extract + apply", flush=True)

        ctx.extract_multi(plan, S.tensors, W1.tensors, I, V, counts, cap)
        ctx.apply_multi(plan, R.tensors, I, V, counts, cap)
        flags = ctx.status()
        assert flags == 0, f"device flags {flags}"

        # ---- whole-set properties
        c64 = counts.to(torch.int64)
        assert int(c64.sum().item()) == nchanged
        assert int(c64.max().item()) <= cap
        col = torch.arange(cap, device=DEV).unsqueeze(0)
        live = col < c64.unsqueeze(1)
        blen = torch.full((plan.nbuckets,), be, dtype=torch.int64, device=DEV)
        blen[-1] = wl.numel - (plan.nbuckets - 1) * be
        for lo in range(0, plan.nbuckets, 64):           # in slabs, to bound temporaries
            hi = min(plan.nbuckets, lo + 64)
            Ii, lv = I[lo:hi].to(torch.int64), live[lo:hi]
            assert bool(((Ii >= 0) & (Ii < blen[lo:hi].unsqueeze(1)) | ~lv).all().item()), "index outside its bucket"
            asc = (Ii[:, 1:] > Ii[:, :-1]) | ~lv[:, 1:]
            assert bool(asc.all().item()), "indices not strictly ascending"
            assert bool(((I[lo:hi] == -1) | lv).all().item()), "slot beyond counts was written"
            del Ii, lv, asc
        assert S.equal(W1), "snapshot differs from the new weights"
        assert R.equal(W1), "reconstructed weights differ from the trainer's"

        # ---- sampled buckets against the oracle (the unmodified single-threaded oracle, one bucket per host
        # thread at a time: ctypes releases the interpreter lock during the call)
        gc_host = counts.cpu().numpy().view(np.uint32)
        got = {b: (I[b].cpu().numpy(), V[b].cpu().numpy().view(np.uint16), host_slices(R, before[b][0])) for b in picks}

        def check_bucket(b):
            segs, olds, news = before[b]
            lens = [ln for _, _, ln in segs]
            oI, oV, oc, ovf = oracle.extract_multi([o.copy() for o in olds], news, lens, be, cap=cap)
            if ovf != 0 or oc.shape != (1,):
                return f"bucket {b}: oracle overflow"
            c = int(oc[0])
            if gc_host[b] != c:
                return f"bucket {b}: count {gc_host[b]} != oracle {c}"
            gI, gV, got_roll = got[b]
            if not (np.array_equal(gI[:c], oI[0, :c]) and np.array_equal(gV[:c], oV[0, :c])):
                return f"bucket {b}: payload differs"
            roll = [o.copy() for o in olds]
            if oracle.apply_multi(roll, lens, be, oI, oV, oc) != oracle.OK:
                return f"bucket {b}: oracle apply failed"
            for x, y, w in zip(roll, got_roll, news):
                if not (np.array_equal(x, y) and np.array_equal(x, w)):
                    return f"bucket {b}: reconstruction differs"
            return None

        with ThreadPoolExecutor(max_workers=HOST_THREADS) as pool:
            errors = [e for e in pool.map(check_bucket, picks) if e]
        assert not errors, errors[:4]
        print(f"  {wl.name}: ok ({nchanged} changed, {len(picks)} buckets matched the oracle)", flush=True)
        plan.close()
    finally:
        ctx.close()


def free_all():
    gc.collect()
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def srs():
    from paper_2605_07330_amd import srs as m
    return m


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_full_size_workload(srs, cfg):
    print(f"case full-size cfg={cfg}", flush=True)
    wl = synth.workload(cfg)
    S = synth.WeightSet(wl, DEV); W1 = synth.WeightSet(wl, DEV); R = synth.WeightSet(wl, DEV)
    try:
        synth.fill_base(S, cfg)
        nchanged, _ = synth.make_update(W1, S, cfg)
        R.copy_from(S)
        if cfg == 3:                                      # the skewed set must really have empty buckets
            assert nchanged < 0.006 * wl.numel
        check_workload(srs, wl, S, W1, R, nchanged, seed=cfg, nsample=96)
    finally:
        del S, W1, R
        free_all()


def test_every_bucket_of_the_8b_shaped_set(srs):
    """All 245 buckets of the Qwen3-8B-shaped set against the oracle, element by element: indices, values, counts,
    untouched slots, refreshed snapshot and reconstructed weights.  The oracle runs unmodified on contiguous runs
    of buckets, one run per host thread."""
    print("case every bucket, cfg=1", flush=True)
    wl = synth.workload(1)
    S = synth.WeightSet(wl, DEV); W1 = synth.WeightSet(wl, DEV); R = synth.WeightSet(wl, DEV)
    ctx = srs.Context(0)
    try:
        synth.fill_base(S, 11)
        nchanged, _ = synth.make_update(W1, S, 11)
        R.copy_from(S)
        numels, be, nb = S.numels, wl.bucket_elems, wl.num_buckets
        olds, news = S.to_numpy_u16(), W1.to_numpy_u16()            # host copies before the GPU touches anything
        rolls = [o.copy() for o in olds]
        cap = (synth.payload_capacity(wl) + 7) // 8 * 8
        plan = ctx.plan(numels, be)
        I = torch.full((nb, cap), -1, dtype=torch.int32, device=DEV)
        V = torch.full((nb, cap), -1, dtype=torch.int16, device=DEV)
        counts = torch.zeros(nb, dtype=torch.int32, device=DEV)
        ctx.extract_multi(plan, S.tensors, W1.tensors, I, V, counts, cap)
        ctx.apply_multi(plan, R.tensors, I, V, counts, cap)
        assert ctx.status() == 0
        gI, gV = I.cpu().numpy(), V.cpu().numpy().view(np.uint16)
        gcnt = counts.cpu().numpy().view(np.uint32)
        print("  GPU done; oracle over all buckets", flush=True)
        per = (nb + HOST_THREADS - 1) // HOST_THREADS
        ranges = [(lo, min(nb, lo + per)) for lo in range(0, nb, per)]

        def run(r):
            lo, hi = r
            # bucket ranges are disjoint in the packed space, so concurrent refreshes of `olds` never touch the
            # same element; tensors that straddle a range boundary are shared between two threads but not their bytes
            oI, oV, oc, ovf = oracle.extract_multi(olds, news, numels, be, cap=cap, b_lo=lo, b_hi=hi)
            if ovf:
                return f"buckets {lo}..{hi}: oracle overflow"
            if not np.array_equal(gcnt[lo:hi], oc):
                return f"buckets {lo}..{hi}: counts differ"
            if not (np.array_equal(gI[lo:hi], oI) and np.array_equal(gV[lo:hi], oV)):
                return f"buckets {lo}..{hi}: payload (or an untouched slot) differs"
            if oracle.apply_multi(rolls, numels, be, oI, oV, oc, b_lo=lo, b_hi=hi) != oracle.OK:
                return f"buckets {lo}..{hi}: oracle apply failed"
            return None

        with ThreadPoolExecutor(max_workers=HOST_THREADS) as pool:
            errors = [e for e in pool.map(run, ranges) if e]
        assert not errors, errors
        assert int(gcnt.astype(np.int64).sum()) == nchanged
        for k, (snap, roll) in enumerate(zip(S.to_numpy_u16(), R.to_numpy_u16())):
            assert np.array_equal(olds[k], news[k]), f"oracle snapshot of tensor {k}"
            assert np.array_equal(snap, news[k]), f"GPU snapshot of tensor {k}"
            assert np.array_equal(roll, news[k]) and np.array_equal(rolls[k], news[k]), f"reconstruction of tensor {k}"
        plan.close()
    finally:
        ctx.close()
        del S, W1, R
        free_all()


def test_full_size_qwen3_32b_density_sweep(srs):
    base = synth.workload(4)
    S = synth.WeightSet(base, DEV); W1 = synth.WeightSet(base, DEV); R = synth.WeightSet(base, DEV)
    try:
        synth.fill_base(S, 4)
        R.copy_from(S)
        # the last round repeats the sparsest density with the snapshot refreshed by a second pass
        for step, p in enumerate([0.001, 0.01, 0.1, 0.001], start=1):
            print(f"case full-size cfg=4 density={p} step={step}", flush=True)
            wl = synth.workload(4, density=p)
            S.wl = W1.wl = R.wl = wl
            # after the previous round S == W1 == R bitwise, so W1 can be rebuilt from S in place
            nchanged, _ = synth.make_update(W1, S, 4, step=step)
            sigma = (wl.numel * p * (1 - p)) ** 0.5
            assert abs(nchanged - wl.numel * p) < 6 * sigma
            check_workload(srs, wl, S, W1, R, nchanged, seed=40 + step, nsample=36 if step < 4 else 12, second_pass=step == 4)
            # payload size against the cost model of Eq. (1)/(2): ratio 1/(3 rho)
            assert abs((2 * wl.numel) / (6 * nchanged) - 1 / (3 * p)) < 0.01 / (3 * p)
    finally:
        del S, W1, R
        free_all()


def test_largest_single_tensor(srs):
    """n = 2^31 - 1 elements, the largest tensor int32 indexing admits (Sec. 3.2): one bucket of the whole
    tensor (indices up to 2^31 - 2), then 37 ragged buckets.  The oracle runs on the full tensor."""
    n = (1 << 31) - 1
    g = torch.Generator(device=DEV); g.manual_seed(77)
    old = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    synth.fill_base_(old, 77)
    new = torch.empty_like(old)
    nchanged, _ = synth.iid_update_(new, old, 0.002, 77)
    # make sure the very first and the very last element change
    for pos in (0, n - 1):
        new.view(torch.int16)[pos] = old.view(torch.int16)[pos] ^ 1
    old_h = old.view(torch.int16).cpu().numpy().view(np.uint16)
    new_h = new.view(torch.int16).cpu().numpy().view(np.uint16)
    ctx = srs.Context(0)
    try:
        for be, cap in ((n, 5_000_000), (58_000_001, 200_000)):
            print(f"case largest tensor be={be}", flush=True)
            snap = old.clone(); roll = old.clone()
            nb = (n + be - 1) // be
            I, V, counts = srs.alloc_payload(nb, cap, DEV)
            ctx.extract(snap, new, be, I, V, counts, cap)
            ctx.apply(roll, be, I, V, counts, cap)
            assert ctx.status() == 0
            wI, wV, wc, ovf = oracle.extract(old_h.copy(), new_h, be, cap=cap)
            assert ovf == 0
            gc_ = counts.cpu().numpy().view(np.uint32)
            assert np.array_equal(gc_, wc)
            gI, gV = I.cpu().numpy(), V.cpu().numpy().view(np.uint16)
            for b in range(nb):
                c = int(wc[b])
                assert np.array_equal(gI[b, :c], wI[b, :c]) and np.array_equal(gV[b, :c], wV[b, :c]), f"bucket {b}"
            assert int(gI[nb - 1, int(wc[nb - 1]) - 1]) == n - 1 and int(gI[0, 0]) == 0
            assert torch.equal(snap.view(torch.int16), new.view(torch.int16))
            assert torch.equal(roll.view(torch.int16), new.view(torch.int16))
            del snap, roll, I, V, counts
        # one element more is rejected before anything is launched
        with pytest.raises(srs.SrsError):
            srs._check(srs._lib.srs_extract(ctx._h, old.data_ptr(), new.data_ptr(), n + 1, n + 1, 8, 8, 8, 16, None), "srs_extract")
    finally:
        ctx.close()
        del old, new
        free_all()


@pytest.mark.parametrize("second_pass", [False, True])
def test_full_size_fp8_workload(srs, second_pass):
    """The 30B-A3B-shaped list as one-byte patterns at the FP8 density of Sec. 2.1 (0.0655 %), 64 MiB buckets,
    library defaults, and again with the snapshot refreshed by a second pass (256 buckets interleaved).  The slab is the packed space, so bucket b of the list is the flat slice [b*be, (b+1)*be)
    and the single-tensor oracle on that slice gives the bucket's payload."""
    import dataclasses
    print(f"case full-size fp8 cfg=2 second_pass={second_pass}", flush=True)
    wl = dataclasses.replace(synth.workload(2), bucket_elems=2 * synth.workload(2).bucket_elems, density=synth.FP8_DENSITY)
    N, be = wl.numel, wl.bucket_elems
    S = synth.ByteSet(wl, DEV); W1 = synth.ByteSet(wl, DEV); R = synth.ByteSet(wl, DEV)
    ctx = srs.Context(0)
    try:
        if second_pass:
            ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_SECOND_PASS)
            ctx.set_option(srs.OPT_INTERLEAVE, 256)
        synth.fill_base_fp8_(S.flat, 5)
        nchanged, _ = synth.iid_update_fp8_(W1.flat, S.flat, wl.density, 5)
        R.copy_from(S)
        sigma = (N * wl.density * (1 - wl.density)) ** 0.5
        assert abs(nchanged - N * wl.density) < 6 * sigma
        plan = ctx.plan(S.numels, be)
        nb = plan.nbuckets
        assert nb == wl.num_buckets == (N + be - 1) // be
        cap = (synth.payload_capacity(wl) + 15) // 16 * 16
        I, V, counts = srs.alloc_payload_u8(nb, cap, DEV)
        picks = sorted({0, 1, nb // 2, nb - 2, nb - 1} | {int(x) for x in np.random.default_rng(5).integers(0, nb, 8)})
        before = {b: (S.flat[b * be:(b + 1) * be].cpu().numpy(), W1.flat[b * be:(b + 1) * be].cpu().numpy()) for b in picks}
        ctx.extract_multi_u8(plan, S.tensors, W1.tensors, I, V, counts, cap)
        ctx.apply_multi_u8(plan, R.tensors, I, V, counts, cap)
        assert ctx.status() == 0
        c64 = counts.to(torch.int64)
        assert int(c64.sum().item()) == nchanged and int(c64.max().item()) <= cap
        live = torch.arange(cap, device=DEV).unsqueeze(0) < c64.unsqueeze(1)
        I64 = I.to(torch.int64)
        blen = torch.full((nb,), be, dtype=torch.int64, device=DEV); blen[-1] = N - (nb - 1) * be
        assert bool((((I64 >= 0) & (I64 < blen.unsqueeze(1))) | ~live).all().item()), "index outside its bucket"
        assert bool(((I64[:, 1:] > I64[:, :-1]) | ~live[:, 1:]).all().item()), "indices not strictly ascending"
        assert bool(((I == -1) | live).all().item()), "slot beyond counts was written"
        assert S.equal(W1) and R.equal(W1)
        ch = counts.cpu().numpy().view(np.uint32)
        for b in picks:
            old_h, new_h = before[b]
            oI, oV, oc, ovf = oracle.extract_u8(old_h.copy(), new_h, be, cap=cap)
            c = int(oc[0])
            assert ovf == 0 and ch[b] == c, f"bucket {b}: count"
            assert np.array_equal(I[b, :c].cpu().numpy(), oI[0, :c]) and np.array_equal(V[b, :c].cpu().numpy(), oV[0, :c]), f"bucket {b}"
        plan.close()
    finally:
        ctx.close()
        del S, W1, R
        free_all()
