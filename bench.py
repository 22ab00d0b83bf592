#!/usr/bin/env python3
"""Benchmark of the sparse-weight-sync hot path on one MI355X.

One "step" = one pass of the whole hot path over one synthetic update of the workload:
    srs_extract_multi(snapshot, new)  ->  (I, V, counts)      (Trainer side, Alg. 1 + Alg. 2)
    srs_apply_multi(rollout weights, I, V, counts)             (Rollout side, Alg. 3)
with every input resident in HBM before the timed region.  Default workload: the
Qwen3-30B-A3B-shaped set (30.5 G BF16 elements, 910 buckets of 64 MiB) at 1 % changed elements.

Two full weight versions W0 and W1 (W1 = W0 with an iid 1 % update) stay resident; step i
extracts against W1 when i is even and against W0 when i is odd, so every step sees exactly the
same 1 % change mask while the snapshot and the rollout copy keep being refreshed for real.

Prints ONE JSON line (see the keys at the bottom).  `value` = dense bytes scanned (old + new,
4 B per element) per second of extract + apply wall time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic per launch comes from a tracked rocprofv3 summary (FETCH_SIZE / WRITE_SIZE runs of this very command,
# scaled by what the same counters read for a device copy of known size).  The summary names the command and the
# commit it was taken at and carries a hash of the kernel sources; when the sources have changed since, the
# figures are withheld (null) rather than reported as if measured.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "traffic_extract_apply_qwen3-30b-a3b.txt")
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2605_07330_amd", "csrc", f)
                  for f in ("srs_kernels.hpp", "srs.hip", "device_guard.hpp")]


def kernel_source_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def measured_traffic(workload: str):
    """{"extract": (read, written), "apply": (read, written)} in bytes per launch, or None when there is no
    summary for this workload or the kernel sources are not the ones it was measured with."""
    try:
        kv = {}
        with open(TRAFFIC_SUMMARY) as fh:
            for line in fh:
                if "=" in line and not line.lstrip().startswith("#"):
                    k, v = line.split("=", 1)
                    kv[k.strip()] = v.strip()
        if kv.get("workload") != workload or kv.get("sources_sha256") != kernel_source_hash():
            return None
        return {"extract": (float(kv["extract_read_bytes"]), float(kv["extract_written_bytes"])),
                "apply": (float(kv["apply_read_bytes"]), float(kv["apply_written_bytes"]))}
    except (OSError, KeyError, ValueError):
        return None


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def overlapping_tensors(numels, be, b_lo, b_hi):
    lo, hi, out, g = b_lo * be, b_hi * be, [], 0
    for k, m in enumerate(numels):
        if g + m > lo and g < hi and m:
            out.append(k)
        g += m
    return out


def cpu_baseline_and_check(torch, np, oracle, wl, old_ws, new_ws, payload, buckets_per_group, ngroups):
    """Times the oracle (as it stands, one thread) on a sample of the workload's buckets and checks
    the GPU payload of those buckets against it.  old_ws/new_ws are the weight sets the last GPU
    extract compared (old_ws untouched by it)."""
    I, V, counts = payload
    be, numels = wl.bucket_elems, [t.numel for t in wl.tensors]
    nb = wl.num_buckets
    stride = max(1, (nb - buckets_per_group) // max(1, ngroups - 1)) if ngroups > 1 else 1
    starts = sorted({min(max(0, nb - buckets_per_group), g * stride) for g in range(ngroups)})
    t_extract = t_apply = 0.0
    elems = 0
    cap = I.shape[1]
    for b_lo in starts:
        b_hi = min(nb, b_lo + buckets_per_group)
        ks = overlapping_tensors(numels, be, b_lo, b_hi)
        olds = [None] * len(numels); news = [None] * len(numels); rolls = [None] * len(numels)
        for k in ks:
            olds[k] = old_ws.tensors[k].view(torch.int16).cpu().numpy().view(np.uint16)
            news[k] = new_ws.tensors[k].view(torch.int16).cpu().numpy().view(np.uint16)
            rolls[k] = olds[k].copy()
        t0 = time.perf_counter()
        oI, oV, oc, _ = oracle.extract_multi(olds, news, numels, be, cap=cap, b_lo=b_lo, b_hi=b_hi)
        t1 = time.perf_counter()
        oracle.apply_multi(rolls, numels, be, oI, oV, oc, b_lo=b_lo, b_hi=b_hi)
        t2 = time.perf_counter()
        t_extract += t1 - t0; t_apply += t2 - t1
        elems += min(wl.numel, b_hi * be) - b_lo * be
        gI = I[b_lo:b_hi].cpu().numpy(); gV = V[b_lo:b_hi].cpu().numpy().view(np.uint16)
        gc = counts[b_lo:b_hi].cpu().numpy().view(np.uint32)
        if not np.array_equal(gc, oc):
            raise SystemExit(f"bench self-check failed: counts differ in buckets {b_lo}..{b_hi}")
        for j in range(b_hi - b_lo):
            c = int(oc[j])
            if not (np.array_equal(gI[j, :c], oI[j, :c]) and np.array_equal(gV[j, :c], oV[j, :c])):
                raise SystemExit(f"bench self-check failed: payload differs in bucket {b_lo + j}")
        done = starts.index(b_lo) + 1
        if done % 6 == 0 or done == len(starts):         # a progress line every couple of seconds
            log(f"oracle: {done} of {len(starts)} groups of {buckets_per_group} buckets done (last [{b_lo},{b_hi})): "
                f"extract {t_extract:.2f}s apply {t_apply:.2f}s so far, GPU payload matches")
    return t_extract, t_apply, elems, len(starts) * buckets_per_group


def cpu_all_cores(torch, np, oracle, wl, old_ws, new_ws, cores, buckets_per_thread):
    """The same unmodified oracle on `cores` host threads at once, each on its own disjoint bucket range
    (ctypes releases the interpreter lock during the call).  Host copies are made first; only the concurrent
    oracle calls are timed (wall clock of the whole pool)."""
    from concurrent.futures import ThreadPoolExecutor
    be, numels = wl.bucket_elems, [t.numel for t in wl.tensors]
    nb = wl.num_buckets
    cores = max(1, min(cores, nb // buckets_per_thread))
    stride = nb // cores
    cap = int(1.5 * wl.density * be) + 8192
    jobs = []
    for c in range(cores):
        b_lo = c * stride
        b_hi = min(nb, b_lo + buckets_per_thread)
        ks = overlapping_tensors(numels, be, b_lo, b_hi)
        olds = [None] * len(numels); news = [None] * len(numels); rolls = [None] * len(numels)
        for k in ks:
            olds[k] = old_ws.tensors[k].view(torch.int16).cpu().numpy().view(np.uint16)
            news[k] = new_ws.tensors[k].view(torch.int16).cpu().numpy().view(np.uint16)
            rolls[k] = olds[k].copy()
        jobs.append((b_lo, b_hi, olds, news, rolls))

    def work(job):
        b_lo, b_hi, olds, news, rolls = job
        oI, oV, oc, _ = oracle.extract_multi(olds, news, numels, be, cap=cap, b_lo=b_lo, b_hi=b_hi)
        oracle.apply_multi(rolls, numels, be, oI, oV, oc, b_lo=b_lo, b_hi=b_hi)
        return int(oc.sum())

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        changed = sum(pool.map(work, jobs))
    wall = time.perf_counter() - t0
    elems = sum(min(wl.numel, b_hi * be) - b_lo * be for b_lo, b_hi, *_ in jobs)
    return wall, elems, cores, changed


SECOND_PASS_BELOW = 0.002    # other_configs also time SRS_OPT_SNAPSHOT = 2 where at most this fraction changes


def measure_other_config(args, torch, srs, synth, cfg, densities, steps, dev):
    """Extract + apply on another workload of the same family, three resident weight sets (snapshot, new weights,
    rollout copy): the new weights are rebuilt, untimed, from the refreshed snapshot before every step.  Library
    defaults; every step is checked (flags, total count against the generator's, snapshot and rollout copy
    bit-identical to the new weights).  Returns {label: figures}."""
    out = {}
    wl0 = synth.workload(cfg)
    S = synth.WeightSet(wl0, dev); W1 = synth.WeightSet(wl0, dev); R = synth.WeightSet(wl0, dev)
    synth.fill_base(S, args.seed)
    R.copy_from(S)
    ctx = srs.Context(0)
    plan = ctx.plan(S.numels, wl0.bucket_elems)
    N = wl0.numel
    update_no = 0
    for dens in densities:
        wl = synth.workload(cfg, density=dens)
        S.wl = W1.wl = R.wl = wl              # the sets keep their storage; only the update recipe (density) changes
        cap = (synth.payload_capacity(wl) + 7) // 8 * 8
        I = torch.empty((plan.nbuckets, cap), dtype=torch.int32, device=dev)
        V = torch.empty((plan.nbuckets, cap), dtype=torch.int16, device=dev)
        counts = torch.zeros(plan.nbuckets, dtype=torch.int32, device=dev)
        pairs = ctx.bind_pairs(plan, S.tensors, W1.tensors)
        rolls = ctx.bind_weights(plan, R.tensors)
        ext, app, rho = [], [], 0.0
        for i in range(1 + steps):                       # the first step is the warm-up
            update_no += 1
            nchanged, _ = synth.make_update(W1, S, args.seed, step=update_no)
            rho = nchanged / N
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record()
            ctx.extract_multi(plan, None, None, I, V, counts, cap, pairs=pairs)
            e[1].record()
            ctx.apply_multi(plan, None, I, V, counts, cap, tensors=rolls)
            e[2].record()
            torch.cuda.synchronize()
            flags = ctx.status()
            total = int(counts.to(torch.int64).sum().item())
            ok = flags == 0 and total == nchanged and torch.equal(S.flat.view(torch.int16), W1.flat.view(torch.int16)) \
                and torch.equal(R.flat.view(torch.int16), W1.flat.view(torch.int16))
            if not ok and not args.no_check:
                raise SystemExit(f"bench self-check failed ({wl.name}, density {dens}): flags={flags} counts={total} "
                                 f"expected={nchanged}")
            if i > 0:
                ext.append(e[0].elapsed_time(e[1])); app.append(e[1].elapsed_time(e[2]))
        e_ms, a_ms = sum(ext) / len(ext), sum(app) / len(app)
        b_e, b_a = (4.0 + 8.0 * rho) * N, 8.0 * rho * N
        label = wl.name if len(densities) == 1 else f"{wl.name}@{dens:g}"
        sp_ms = None
        if dens is not None and dens <= SECOND_PASS_BELOW:       # same steps with SRS_OPT_SNAPSHOT = 2
            ctx2 = srs.Context(0)
            ctx2.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_SECOND_PASS)
            ctx2.set_option(srs.OPT_INTERLEAVE, 256)
            plan2 = ctx2.plan(S.numels, wl0.bucket_elems)
            pairs2 = ctx2.bind_pairs(plan2, S.tensors, W1.tensors)
            sp = []
            for i in range(1 + steps):
                update_no += 1
                nchanged, _ = synth.make_update(W1, S, args.seed, step=update_no)
                e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                e[0].record()
                ctx2.extract_multi(plan2, None, None, I, V, counts, cap, pairs=pairs2)
                e[1].record()
                torch.cuda.synchronize()
                ok = ctx2.status() == 0 and int(counts.to(torch.int64).sum().item()) == nchanged \
                    and torch.equal(S.flat.view(torch.int16), W1.flat.view(torch.int16))
                if not ok and not args.no_check:
                    raise SystemExit(f"bench self-check failed ({wl.name}, density {dens}, second-pass refresh)")
                if i > 0:
                    sp.append(e[0].elapsed_time(e[1]))
            sp_ms = sum(sp) / len(sp)
            R.copy_from(S)                               # the rollout copy follows for the next density
            plan2.close(); ctx2.close()
            log(f"{label}: extract with the snapshot refreshed in a second pass {sp_ms:.3f} ms against {e_ms:.3f} ms fused")
        out[label] = {"elements": N, "buckets": plan.nbuckets, "changed_fraction": round(rho, 6),
                      "extract_ms": round(e_ms, 4), "apply_ms": round(a_ms, 4), "sync_ms": round(e_ms + a_ms, 4),
                      "frac": round(b_e / (e_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                      "frac_combined": round((b_e + b_a) / ((e_ms + a_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                      "dense_gbs_scanned": round(4.0 * N / ((e_ms + a_ms) * 1e-3) / 1e9, 1), "steps": steps}
        if sp_ms is not None:
            out[label]["extract_second_pass_ms"] = round(sp_ms, 4)
        log(f"{label}: rho {rho:.5f}, extract {e_ms:.3f} ms = {100 * out[label]['frac']:.1f}% of peak on (4 + 8 rho) N, "
            f"apply {a_ms:.3f} ms, combined {100 * out[label]['frac_combined']:.1f}%")
        del I, V, counts
    plan.close(); ctx.close()
    del S, W1, R
    torch.cuda.empty_cache()
    return out


def bench_cast(args, torch, srs, synth, wl, dev) -> int:
    """Fused cast + diff: W (BF16 model parameters) <- round(master FP32), payload out, then apply to the
    rollout copy.  Before every step the master weights are rebuilt (untimed) from a fresh sparse update of W."""
    N = wl.numel
    W = synth.WeightSet(wl, dev); R = synth.WeightSet(wl, dev)
    master = torch.empty(N, dtype=torch.float32, device=dev)
    masters, off = [], 0
    for t in wl.tensors:
        masters.append(master[off:off + t.numel]); off += t.numel
    synth.fill_base(W, args.seed)
    R.copy_from(W)
    ctx = srs.Context(0)
    if args.tile:
        ctx.set_option(srs.OPT_TILE_ELEMS, args.tile)
    if args.interleave:
        ctx.set_option(srs.OPT_INTERLEAVE, args.interleave)
    if args.refresh_group >= 0:
        ctx.set_option(srs.OPT_REFRESH_GROUP, args.refresh_group)
    plan = ctx.plan(W.numels, wl.bucket_elems)
    cap = (synth.payload_capacity(wl) + 7) // 8 * 8
    I = torch.empty((plan.nbuckets, cap), dtype=torch.int32, device=dev)
    V = torch.empty((plan.nbuckets, cap), dtype=torch.int16, device=dev)
    counts = torch.zeros(plan.nbuckets, dtype=torch.int32, device=dev)
    pairs = ctx.bind_cast_pairs(plan, W.tensors, masters)
    rolls = ctx.bind_weights(plan, R.tensors)
    chunk = 1 << 26
    ext, app, rho = [], [], 0.0
    for i in range(args.warmup + args.steps):
        changed = 0
        for c, lo in enumerate(range(0, N, chunk)):        # master <- weights that round to an updated W, chunk by chunk
            hi = min(N, lo + chunk)
            new = torch.empty(hi - lo, dtype=torch.bfloat16, device=dev)
            n_c, _ = synth.iid_update_(new, W.flat[lo:hi], wl.density, args.seed, salt=(i + 1) * 100003 + c)
            changed += n_c
            synth.master_from_(master[lo:hi], new, args.seed, salt=(i + 1) * 100003 + c)
        rho = changed / N
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        ctx.extract_cast_multi(plan, None, None, I, V, counts, cap, pairs=pairs)
        e[1].record()
        ctx.apply_multi(plan, None, I, V, counts, cap, tensors=rolls)
        e[2].record()
        torch.cuda.synchronize()
        flags = ctx.status()
        total = int(counts.to(torch.int64).sum().item())
        if flags or total != changed or not torch.equal(R.flat.view(torch.int16), W.flat.view(torch.int16)):
            raise SystemExit(f"bench self-check failed (cast): flags={flags} counts={total} expected={changed}")
        if i >= args.warmup:
            ext.append(e[0].elapsed_time(e[1])); app.append(e[1].elapsed_time(e[2]))
    ext_avg, app_avg = sum(ext) / len(ext), sum(app) / len(app)
    bytes_extract = (6.0 + 8.0 * rho) * N          # read 4 (master) + 2 (parameters); write payload 6 rho + parameters 2 rho
    ach = bytes_extract / (ext_avg * 1e-3) / 1e9
    log(f"cast+diff extract {ext_avg:.3f} ms (min {min(ext):.3f}), apply {app_avg:.3f} ms; "
        f"{ach:.0f} GB/s = {100 * ach / HBM_PEAK_GBS:.1f}% of peak on (6 + 8 rho) N bytes")
    out = {"metric": "fused cast+diff extract + apply, dense GB/s scanned", "value": round(6.0 * N / ((ext_avg + app_avg) * 1e-3) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ext_avg + app_avg, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16", "data": "synthetic",
           "config": {"workload": wl.name + "+fp32-master", "elements": N, "changed_fraction": round(rho, 6)},
           "extract_ms": round(ext_avg, 4), "apply_ms": round(app_avg, 4),
           "roofline": {"bound": "hbm", "kernel": "extract_kernel<cast>", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None},
           "cpu_baseline": None}
    print(json.dumps(out), flush=True)
    plan.close(); ctx.close()
    return 0


def bench_fp8(args, torch, srs, synth, wl, dev) -> int:
    """The same tensor list at FP8 synchronisation precision (Sec. 2.1: 0.0655 % of the elements change):
    srs_extract_multi_u8 + srs_apply_multi_u8 on one-byte patterns, buckets of the same 64 MiB, first with the
    in-place snapshot refresh, then with the rotating snapshot.  CPU leg (unless --no-cpu-baseline): the oracle is
    timed on four buckets of the last step and the GPU payload of those buckets is compared with it."""
    import dataclasses

    import numpy as np
    oracle = None
    if not args.no_cpu_baseline:
        import oracle
    cpu = None
    wl = dataclasses.replace(wl, name=wl.name + "+fp8", bucket_elems=2 * wl.bucket_elems,
                             density=args.density or synth.FP8_DENSITY)
    N, be = wl.numel, wl.bucket_elems
    W0 = synth.ByteSet(wl, dev); W1 = synth.ByteSet(wl, dev); S = synth.ByteSet(wl, dev); R = synth.ByteSet(wl, dev)
    synth.fill_base_fp8_(W0.flat, args.seed)
    nchanged, _ = synth.iid_update_fp8_(W1.flat, W0.flat, wl.density, args.seed)
    S.copy_from(W0); R.copy_from(W0)
    rho = nchanged / N
    log(f"fp8: {N} one-byte elements ({N / 1e9:.2f} GB per copy), {wl.num_buckets} buckets of {be}, {nchanged} changed "
        f"(rho = {rho:.6f})")
    versions = [W1, W0]
    cap = (synth.payload_capacity(wl) + 15) // 16 * 16
    out_modes = {}
    for mode in ("refresh-in-place", "rotate", "refresh-second-pass"):
        ctx = srs.Context(0)
        if args.tile:
            ctx.set_option(srs.OPT_TILE_ELEMS, args.tile)
        if args.interleave:
            ctx.set_option(srs.OPT_INTERLEAVE, args.interleave)
        if args.refresh_group >= 0:
            ctx.set_option(srs.OPT_REFRESH_GROUP, args.refresh_group)
        if mode != "refresh-in-place":
            ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_ROTATE if mode == "rotate" else srs.SNAPSHOT_SECOND_PASS)
            if not args.interleave:
                ctx.set_option(srs.OPT_INTERLEAVE, 256)
        plans = [ctx.plan(S.numels, be) for _ in (0, 1)]
        nb = plans[0].nbuckets
        I = torch.empty((nb, cap), dtype=torch.int32, device=dev)
        V = torch.empty((nb, cap), dtype=torch.uint8, device=dev)
        counts = torch.zeros(nb, dtype=torch.int32, device=dev)
        if mode == "rotate":
            pairs = [ctx.bind_pairs(plans[d], versions[1 - d].tensors, versions[d].tensors, 1) for d in (0, 1)]
        else:
            pairs = [ctx.bind_pairs(plans[d], S.tensors, versions[d].tensors, 1) for d in (0, 1)]
        rolls = [ctx.bind_weights(plans[d], R.tensors, 1) for d in (0, 1)]
        steps = max(2, args.steps // 2 * 2)            # even: both modes end where they started
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps + 2)]
        for k in range(steps + 2):                     # the first two are warm-up
            d = k % 2
            ev[k][0].record()
            ctx.extract_multi_u8(plans[d], None, None, I, V, counts, cap, pairs=pairs[d])
            ev[k][1].record()
            ctx.apply_multi_u8(plans[d], None, I, V, counts, cap, tensors=rolls[d])
            ev[k][2].record()
        torch.cuda.synchronize()
        flags = ctx.status()
        last, prev = versions[1], versions[0]          # the last step (d = 1) went from versions[0] to versions[1]
        total = int(counts.to(torch.int64).sum().item())
        ok = flags == 0 and total == nchanged and torch.equal(R.flat, last.flat)
        ok = ok and (mode == "rotate" or torch.equal(S.flat, last.flat))
        if not ok and not args.no_check:
            raise SystemExit(f"bench self-check failed (fp8, {mode}): flags={flags} counts={total} expected={nchanged}")
        if not args.no_cpu_baseline:                   # the CPU leg: the oracle timed on four buckets, the GPU payload checked against it
            ch = counts.cpu().numpy().view(np.uint32)
            t_cpu, elems = 0.0, 0
            for b in sorted({0, nb // 3, nb // 2, nb - 1}):
                lo, hi = b * be, min(N, (b + 1) * be)
                h_old, h_new = prev.flat[lo:hi].cpu().numpy(), last.flat[lo:hi].cpu().numpy()
                t0 = time.perf_counter()
                oI, oV, oc, _ = oracle.extract_u8(h_old, h_new, be, cap=cap)
                t1 = time.perf_counter()
                c = int(oc[0])
                if ch[b] != c or not np.array_equal(I[b, :c].cpu().numpy(), oI[0, :c]) \
                        or not np.array_equal(V[b, :c].cpu().numpy(), oV[0, :c]):
                    raise SystemExit(f"bench self-check failed (fp8, {mode}): bucket {b} differs from the oracle")
                h_roll = prev.flat[lo:hi].cpu().numpy().copy()
                t2 = time.perf_counter()
                oracle.apply_u8(h_roll, be, oI, oV, oc)
                t3 = time.perf_counter()
                if not np.array_equal(h_roll, last.flat[lo:hi].cpu().numpy()):
                    raise SystemExit(f"bench self-check failed (fp8, {mode}): oracle apply of bucket {b}")
                t_cpu += (t1 - t0) + (t3 - t2); elems += hi - lo
            if mode == "refresh-in-place":
                cpu = {"value": round(2.0 * elems / t_cpu / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                       "sample": f"{elems} one-byte elements (4 of {nb} buckets); oracle extract + apply {t_cpu:.2f}s, compute only"}
        ext = sum(e[0].elapsed_time(e[1]) for e in ev[2:]) / steps
        app = sum(e[1].elapsed_time(e[2]) for e in ev[2:]) / steps
        per_changed = 5.0 if mode == "rotate" else 6.0         # I (4) + V (1) [+ snapshot (1)]
        ach = (2.0 + per_changed * rho) * N / (ext * 1e-3) / 1e9
        log(f"fp8 {mode}: extract {ext:.3f} ms = {ach:.0f} GB/s on (2 + {per_changed:.0f} rho) N bytes = "
            f"{100 * ach / HBM_PEAK_GBS:.1f}% of peak, apply {app:.3f} ms")
        out_modes[mode] = {"extract_ms": round(ext, 4), "apply_ms": round(app, 4), "achieved": round(ach, 1),
                           "frac": round(ach / HBM_PEAK_GBS, 4)}
        for pl in plans:
            pl.close()
        ctx.close()
    m = out_modes["refresh-in-place"]
    step_ms = m["extract_ms"] + m["apply_ms"]
    log(f"fp8: snapshot refreshed in a second pass (SRS_OPT_SNAPSHOT = 2): extract "
        f"{out_modes['refresh-second-pass']['extract_ms']:.3f} ms against {m['extract_ms']:.3f} ms fused")
    out = {"metric": "extract+apply dense GB/s scanned (one-byte elements)", "value": round(2.0 * N / (step_ms * 1e-3) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": 2, "ms_per_step": round(step_ms, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
           "config": {"workload": wl.name, "elements": N, "buckets": wl.num_buckets, "bucket_elems": be,
                      "changed_fraction": round(rho, 6), "payload_cap": cap},
           "extract_ms": m["extract_ms"], "apply_ms": m["apply_ms"],
           "roofline": {"bound": "hbm", "kernel": "extract_kernel<u8>", "achieved": m["achieved"], "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": m["frac"], "traffic": None},
           "rotating_snapshot": out_modes["rotate"], "second_pass_snapshot": out_modes["refresh-second-pass"],
           "cpu_baseline": cpu, "checked": not args.no_check}
    print(json.dumps(out), flush=True)
    return 0


def chunked_sum(torch, flat) -> int:
    """Sum of the 16-bit patterns of a weight slab, in pieces that keep the temporaries small."""
    v = flat.view(torch.int16)
    return sum(int(v[i:i + (1 << 28)].sum(dtype=torch.int64).item()) for i in range(0, v.numel(), 1 << 28))


def rotating_leg(args, torch, srs, wl, versions, R, payload, cap, i0, nchanged, rho, N):
    """Extract + apply with SRS_OPT_SNAPSHOT = 1: each version is diffed, read-only, against the other one."""
    I, V, counts = payload
    ctx = srs.Context(0)
    ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_ROTATE)
    ctx.set_option(srs.OPT_INTERLEAVE, 256)          # with no stores into the weights this mode measures best with
                                                     # more buckets in flight than the in-place one (18.7 against 19.0 ms)
    plans = [ctx.plan(R.numels, wl.bucket_elems) for _ in (0, 1)]
    pairs = [ctx.bind_pairs(plans[d], versions[1 - d].tensors, versions[d].tensors) for d in (0, 1)]
    rolls = [ctx.bind_weights(plans[d], R.tensors) for d in (0, 1)]
    steps = max(2, args.steps // 2 * 2)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps + 2)]
    for k in range(steps + 2):                       # the first two are warm-up
        d = (i0 + k) % 2
        ev[k][0].record()
        ctx.extract_multi(plans[d], None, None, I, V, counts, cap, pairs=pairs[d])
        ev[k][1].record()
        ctx.apply_multi(plans[d], None, I, V, counts, cap, tensors=rolls[d])
        ev[k][2].record()
    torch.cuda.synchronize()
    flags = ctx.status()
    last = versions[(i0 + steps + 1) % 2]
    total = int(counts.to(torch.int64).sum().item())
    if not args.no_check and (flags or total != nchanged or not torch.equal(R.flat.view(torch.int16), last.flat.view(torch.int16))):
        raise SystemExit(f"bench self-check failed (rotating snapshot): flags={flags} counts={total} expected={nchanged}")
    ext = sum(e[0].elapsed_time(e[1]) for e in ev[2:]) / steps
    app = sum(e[1].elapsed_time(e[2]) for e in ev[2:]) / steps
    ach = (4.0 + 6.0 * rho) * N / (ext * 1e-3) / 1e9
    log(f"rotating snapshot: extract {ext:.3f} ms = {ach:.0f} GB/s on (4 + 6 rho) N bytes = {100 * ach / HBM_PEAK_GBS:.1f}% "
        f"of peak, apply {app:.3f} ms")
    for pl in plans:
        pl.close()
    ctx.close()
    return {"extract_ms": round(ext, 4), "apply_ms": round(app, 4), "sync_ms": round(ext + app, 4),
            "achieved": round(ach, 1), "frac": round(ach / HBM_PEAK_GBS, 4), "steps": steps,
            "value": round(4.0 * N / ((ext + app) * 1e-3) / 1e9, 1),
            "note": "extract leaves the snapshot untouched; the two resident BF16 versions swap roles every step"}


def bench_cumulative(args, torch, srs, synth, wl, dev) -> int:
    """Alg. 1 as printed, one optimizer step per synchronisation: mark (diff of two resident versions OR-ed into
    the bitmap), extract from the bitmap with the current values, apply.  The two versions swap roles every cycle."""
    N = wl.numel
    A = synth.WeightSet(wl, dev); B = synth.WeightSet(wl, dev); R = synth.WeightSet(wl, dev)
    synth.fill_base(A, args.seed)
    nchanged, _ = synth.make_update(B, A, args.seed)
    R.copy_from(A)
    rho = nchanged / N
    ctx = srs.Context(0)
    # extract from the bitmap is a gather by many light workgroups: it measures best with all buckets interleaved
    # (7.0 ms against 7.5 ms at the library default of 64)
    if args.tile:
        ctx.set_option(srs.OPT_TILE_ELEMS, args.tile)
    ctx.set_option(srs.OPT_INTERLEAVE, args.interleave or 1024)
    plans = [ctx.plan(A.numels, wl.bucket_elems), ctx.plan(A.numels, wl.bucket_elems)]
    cap = (synth.payload_capacity(wl) + 7) // 8 * 8
    nb = plans[0].nbuckets
    I = torch.empty((nb, cap), dtype=torch.int32, device=dev)
    V = torch.empty((nb, cap), dtype=torch.int16, device=dev)
    counts = torch.zeros(nb, dtype=torch.int32, device=dev)
    bitmap = torch.zeros(srs.bitmap_words(N), dtype=torch.int32, device=dev)
    vers = [(A, B), (B, A)]
    pairs = [ctx.bind_pairs(plans[d], vers[d][0].tensors, vers[d][1].tensors) for d in (0, 1)]
    curs = [ctx.bind_weights(plans[d], vers[d][1].tensors) for d in (0, 1)]
    rolls = ctx.bind_weights(plans[0], R.tensors)
    tm, te, ta = [], [], []
    for i in range(args.warmup + args.steps):
        d = i % 2
        bitmap.zero_()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record()
        ctx.mark_multi(plans[d], None, None, bitmap, pairs=pairs[d])
        e[1].record()
        ctx.extract_marked_multi(plans[d], None, bitmap, I, V, counts, cap, tensors=curs[d])
        e[2].record()
        ctx.apply_multi(plans[0], None, I, V, counts, cap, tensors=rolls)
        e[3].record()
        torch.cuda.synchronize()
        flags = ctx.status()
        total = int(counts.to(torch.int64).sum().item())
        if flags or total != nchanged or not torch.equal(R.flat.view(torch.int16), vers[d][1].flat.view(torch.int16)):
            raise SystemExit(f"bench self-check failed (cumulative): flags={flags} counts={total} expected={nchanged}")
        if i >= args.warmup:
            tm.append(e[0].elapsed_time(e[1])); te.append(e[1].elapsed_time(e[2])); ta.append(e[2].elapsed_time(e[3]))
    am, ae, aa = (sum(x) / len(x) for x in (tm, te, ta))
    bytes_mark = (4.0 + 0.25) * N          # read both versions; read-modify-write of one bit per element
    log(f"cumulative: mark {am:.3f} ms ({bytes_mark / (am * 1e-3) / 1e9:.0f} GB/s on 4.25 N bytes), "
        f"extract_marked {ae:.3f} ms, apply {aa:.3f} ms")
    out = {"metric": "Alg. 1 cumulative set: mark + extract_marked + apply, dense GB/s scanned",
           "value": round(4.0 * N / ((am + ae + aa) * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(am + ae + aa, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "u16", "data": "synthetic",
           "config": {"workload": wl.name + "+cumulative-bitmap", "elements": N, "changed_fraction": round(rho, 6)},
           "mark_ms": round(am, 4), "extract_marked_ms": round(ae, 4), "apply_ms": round(aa, 4),
           "roofline": {"bound": "hbm", "kernel": "mark_kernel", "achieved": round(bytes_mark / (am * 1e-3) / 1e9, 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(bytes_mark / (am * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                        "traffic": None},
           "cpu_baseline": None}
    print(json.dumps(out), flush=True)
    for pl in plans:
        pl.close()
    ctx.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", type=int, default=2, help="workload id 0..4 (synth.workload); 2 = Qwen3-30B-A3B-shaped, the headline workload")
    ap.add_argument("--density", type=float, default=None)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--tile", type=int, default=0, help="extract tile elements (0 = library default)")
    ap.add_argument("--refresh-group", type=int, default=-1, help="snapshot refresh: 8 = whole 128-byte lines (default), 0 = element by element")
    ap.add_argument("--interleave", type=int, default=0, help="buckets interleaved over consecutive workgroups (0 = default)")
    ap.add_argument("--tiny", action="store_true", help="structure-preserving tiny workload (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-groups", type=int, default=36,
                    help="oracle sample: groups of 16 buckets spread over the set (36 groups = 63 %% of the default "
                         "workload, about 12 s of single-thread oracle work)")
    ap.add_argument("--cpu-cores", type=int, default=0,
                    help="threads of the all-cores oracle leg (0 = the host's cores, at most 16: a one-GPU box's share)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the other workloads (Qwen3-8B-shaped, skewed 30B-A3B, Qwen3-32B-shaped at three "
                         "densities) that the default run times after the headline")
    ap.add_argument("--print-source-hash", action="store_true",
                    help="print the hash of the kernel sources that a traffic summary under profiles/ must carry, and exit")
    ap.add_argument("--probe", action="store_true", help="also time the two-stream read probe")
    ap.add_argument("--no-check", action="store_true", help="skip the result checks (kernel experiments only)")
    ap.add_argument("--index-coding", action="store_true",
                    help="also run the 16-bit index coding of Sec. 3.3: extract, srs_encode_indices, then "
                         "srs_apply_multi_encoded instead of srs_apply_multi (not the headline path)")
    ap.add_argument("--value-coding", action="store_true",
                    help="also run the value entropy coding of Sec. 3.3: srs_encode_values after extract and "
                         "srs_decode_values before apply (not the headline path)")
    ap.add_argument("--cast", action="store_true",
                    help="time the fused cast + diff instead (srs_extract_cast_multi on FP32 master weights that are "
                         "rebuilt, untimed, before every step; implies 3 resident sets: master, model parameters, "
                         "rollout copy) -- not the headline path")
    ap.add_argument("--fp8", action="store_true",
                    help="time the one-byte calls instead (srs_extract_multi_u8 / srs_apply_multi_u8): the same tensor "
                         "list as E4M3 patterns, 0.0655 %% changed unless --density is given -- not the headline path")
    ap.add_argument("--cumulative", action="store_true",
                    help="time Alg. 1 as printed instead: srs_mark_multi (one optimizer step's diff OR-ed into the bitmap), "
                         "srs_extract_marked_multi, srs_apply_multi -- not the headline path")
    ap.add_argument("--rotate-snapshot", action="store_true",
                    help="SRS_OPT_SNAPSHOT = 1: extract leaves the snapshot alone and the two resident BF16 versions "
                         "swap roles every step (the new weights of one step are the snapshot of the next) -- "
                         "not the headline contract, which refreshes the snapshot in place")
    ap.add_argument("--second-pass", action="store_true",
                    help="SRS_OPT_SNAPSHOT = 2: the scan leaves the snapshot alone and the same call then scatters the "
                         "payload into it (same contract as the headline; pays when few elements change) -- not the "
                         "headline mode")
    ap.add_argument("--regen", action="store_true",
                    help="keep one new-weights version and rebuild it (untimed) before every step instead of "
                         "alternating two resident versions: 3 weight sets instead of 4, for workloads that do not "
                         "fit otherwise; step time is then the sum of the per-step event times")
    args = ap.parse_args()

    if args.print_source_hash:
        print(kernel_source_hash())
        return 0
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2605_07330_amd import srs, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)

    wl = synth.workload(args.config, density=args.density, tiny=args.tiny)
    N = wl.numel
    log(f"workload {wl.name}: {len(wl.tensors)} tensors, {N} elements ({2 * N / 1e9:.2f} GB), "
        f"{wl.num_buckets} buckets of {wl.bucket_elems} elements")

    if args.cast:
        return bench_cast(args, torch, srs, synth, wl, dev)
    if args.cumulative:
        return bench_cumulative(args, torch, srs, synth, wl, dev)
    if args.fp8:
        return bench_fp8(args, torch, srs, synth, wl, dev)

    if args.rotate_snapshot and args.second_pass:
        print("bench.py: --rotate-snapshot and --second-pass are two values of one option", file=sys.stderr)
        return 2
    if args.rotate_snapshot and args.regen:
        print("bench.py: --rotate-snapshot alternates two resident versions; it cannot be combined with --regen",
              file=sys.stderr)
        return 2
    t0 = time.perf_counter()
    if args.rotate_snapshot:
        W0 = synth.WeightSet(wl, dev); W1 = synth.WeightSet(wl, dev); R = synth.WeightSet(wl, dev)
        synth.fill_base(W0, args.seed)
        nchanged, _ = synth.make_update(W1, W0, args.seed)
        R.copy_from(W0)
        S = W0                                   # only for its shape list below; never bound as a snapshot
    elif args.regen:
        S = synth.WeightSet(wl, dev); W1 = synth.WeightSet(wl, dev); R = synth.WeightSet(wl, dev)
        synth.fill_base(S, args.seed)
        nchanged, _ = synth.make_update(W1, S, args.seed)
        R.copy_from(S)
        W0 = W1
    else:
        W0 = synth.WeightSet(wl, dev); W1 = synth.WeightSet(wl, dev)
        S = synth.WeightSet(wl, dev); R = synth.WeightSet(wl, dev)
        synth.fill_base(W0, args.seed)
        nchanged, _ = synth.make_update(W1, W0, args.seed)
        S.copy_from(W0); R.copy_from(W0)
    torch.cuda.synchronize()
    rho = nchanged / N
    log(f"generated in {time.perf_counter() - t0:.1f}s: {nchanged} changed elements (rho = {rho:.5f})")

    ctx = srs.Context(0)
    if args.tile:
        ctx.set_option(srs.OPT_TILE_ELEMS, args.tile)
    if args.refresh_group >= 0:
        ctx.set_option(srs.OPT_REFRESH_GROUP, args.refresh_group)
    ctx.set_option(srs.OPT_INTERLEAVE, args.interleave) if args.interleave else None
    if args.rotate_snapshot:
        ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_ROTATE)
        # with no stores into the weights this mode measures best with more buckets in flight than the in-place one
        if args.tile:
            ctx.set_option(srs.OPT_TILE_ELEMS, args.tile)
        ctx.set_option(srs.OPT_INTERLEAVE, args.interleave or 256)
    if args.second_pass:
        ctx.set_option(srs.OPT_SNAPSHOT, srs.SNAPSHOT_SECOND_PASS)
        ctx.set_option(srs.OPT_INTERLEAVE, args.interleave or 256)
    # one plan per direction: each keeps its own device copy of the pointer table, so alternating the
    # `new` version does not re-upload it every step
    plans = [ctx.plan(S.numels, wl.bucket_elems), ctx.plan(S.numels, wl.bucket_elems)]
    plan = plans[0]
    cap = synth.payload_capacity(wl)
    cap = (cap + 7) // 8 * 8
    I = torch.empty((plan.nbuckets, cap), dtype=torch.int32, device=dev)
    V = torch.empty((plan.nbuckets, cap), dtype=torch.int16, device=dev)
    counts = torch.zeros(plan.nbuckets, dtype=torch.int32, device=dev)
    log(f"plan: {plan.nbuckets} buckets, {plan.nsegments} segments, {plan.ntiles} tiles; cap {cap} pairs per bucket "
        f"({plan.nbuckets * cap * 6 / 1e9:.2f} GB payload buffers)")

    versions = [W1, W0]
    if args.rotate_snapshot:                     # step d diffs versions[d] against the other version, read-only
        pairs = [ctx.bind_pairs(plans[d], versions[1 - d].tensors, versions[d].tensors) for d in (0, 1)]
        sums_before = [chunked_sum(torch, w.flat) for w in versions]
    else:
        pairs = [ctx.bind_pairs(plans[d], S.tensors, versions[d].tensors) for d in (0, 1)]
    rolls = [ctx.bind_weights(plans[d], R.tensors) for d in (0, 1)]

    if args.index_coding:
        D, max_gap, anchors = srs.alloc_encoded(plan.nbuckets, cap, dev)
    if args.value_coding:
        venc = srs.alloc_value_stream(plan.nbuckets, cap, dev)
        V2 = torch.empty_like(V)
        vc_events = []

    def step(i, ev=None):
        d = i % 2
        if ev:
            ev[0].record()
        ctx.extract_multi(plans[d], None, None, I, V, counts, cap, pairs=pairs[d])
        if args.index_coding:
            ctx.encode_indices(I, counts, plan.nbuckets, cap, 0, D, max_gap, anchors)
        Vr = V
        if args.value_coding:
            q = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            q[0].record()
            ctx.encode_values(V, counts, plan.nbuckets, cap, venc)
            q[1].record()
            ctx.decode_values(venc, counts, plan.nbuckets, cap, V2)
            q[2].record()
            vc_events.append(q)
            Vr = V2
        if ev:
            ev[1].record()
        if args.index_coding:
            ctx.apply_multi_encoded(plans[d], None, D, I, Vr, counts, max_gap, anchors, cap, tensors=rolls[d])
        else:
            ctx.apply_multi(plans[d], None, I, Vr, counts, cap, tensors=rolls[d])
        if ev:
            ev[2].record()

    def regen(i):
        # S == W1 bitwise after a step, so the next update can be built from S into W1 in place
        nonlocal nchanged, rho
        if i > 0:
            nchanged, _ = synth.make_update(W1, S, args.seed, step=i + 1)
            rho = nchanged / N

    for i in range(args.warmup):
        if args.regen:
            regen(i)
        step(0 if args.regen else i)
    torch.cuda.synchronize()
    flags = ctx.status()
    if flags and not args.no_check:
        raise SystemExit(f"device flags {flags} after warm-up")

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        if args.regen:
            regen(args.warmup + k)
        step(0 if args.regen else args.warmup + k, events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start

    flags = ctx.status()
    last_new = W1 if args.regen else versions[(args.warmup + args.steps - 1) % 2]
    total_counts = int(counts.to(torch.int64).sum().item())
    if args.rotate_snapshot:                     # neither version may have been written
        snap_ok = sums_before == [chunked_sum(torch, w.flat) for w in versions]
    else:
        snap_ok = torch.equal(S.flat.view(torch.int16), last_new.flat.view(torch.int16))
    ok = flags == 0 and total_counts == nchanged and snap_ok \
        and torch.equal(R.flat.view(torch.int16), last_new.flat.view(torch.int16))
    if not ok and not args.no_check:
        raise SystemExit(f"bench self-check failed: flags={flags} counts={total_counts} expected={nchanged}")

    nbuckets = plan.nbuckets
    ext_ms = [e[0].elapsed_time(e[1]) for e in events]
    app_ms = [e[1].elapsed_time(e[2]) for e in events]
    ext_avg, app_avg = sum(ext_ms) / len(ext_ms), sum(app_ms) / len(app_ms)
    ms_per_step = (ext_avg + app_avg) if args.regen else wall * 1e3 / args.steps
    # read old+new; write I(4)+V(2) and, unless the caller rotates buffers, snapshot(2) per changed element
    bytes_extract = (4.0 + (6.0 if args.rotate_snapshot else 8.0) * rho) * N
    bytes_apply = 8.0 * rho * N                    # read I+V, write 2 per changed element
    value = 4.0 * N / (ms_per_step * 1e-3) / 1e9
    ach = bytes_extract / (ext_avg * 1e-3) / 1e9
    combined = (bytes_extract + bytes_apply) / (ms_per_step * 1e-3) / 1e9
    log("per-step extract ms: " + " ".join(f"{x:.2f}" for x in ext_ms))
    log(f"extract {ext_avg:.3f} ms (min {min(ext_ms):.3f}), apply {app_avg:.3f} ms (min {min(app_ms):.3f}), "
        f"step {ms_per_step:.3f} ms; extract {ach:.0f} GB/s = {100 * ach / HBM_PEAK_GBS:.1f}% of peak; "
        f"combined {combined:.0f} GB/s = {100 * combined / HBM_PEAK_GBS:.1f}%")

    if args.value_coding:
        enc_ms = sum(q[0].elapsed_time(q[1]) for q in vc_events[-args.steps:]) / args.steps
        dec_ms = sum(q[1].elapsed_time(q[2]) for q in vc_events[-args.steps:]) / args.steps
        cw = venc["chunk_words"].to(torch.int64)
        started = int((cw > 0).sum().item())
        wire = 256 * plan.nbuckets + nchanged + 4 * int(cw.sum().item()) + 64 * started
        log(f"value coding: encode {enc_ms:.3f} ms, decode {dec_ms:.3f} ms (both inside the extract figure above); "
            f"value stream {wire / 1e9:.3f} GB against {2 * nchanged / 1e9:.3f} GB raw: alpha = {wire / (2 * nchanged):.4f}")

    probe_gbs = None
    a = b = sink = old_ws = new_ws = None
    if args.probe or not (args.regen or args.tiny):     # context for the roofline: what two plain read streams reach here
        nbytes = min(2 * N, 16 << 30) // 32768 * 32768
        sink = torch.empty(srs.stream_probe_sink_words(nbytes), dtype=torch.int32, device=dev)
        a = W0.flat.view(torch.int16)[: nbytes // 2]; b = W1.flat.view(torch.int16)[: nbytes // 2]
        for _ in range(2):
            ctx.stream_probe(a, b, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            ctx.stream_probe(a, b, sink)
        e1.record(); torch.cuda.synchronize()
        probe_gbs = 2 * nbytes * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        log(f"two-stream read probe: {probe_gbs:.0f} GB/s")

    # the same workload under the rotating-snapshot contract (SRS_OPT_SNAPSHOT = 1), reported beside the
    # headline: an even number of steps, so that the rollout copy ends where it started
    rotating = None
    if not (args.regen or args.rotate_snapshot or args.second_pass or args.index_coding or args.value_coding or args.tiny):
        rotating = rotating_leg(args, torch, srs, wl, versions, R, (I, V, counts), cap, args.warmup + args.steps,
                                nchanged, rho, N)

    cpu = cpu_mt = None
    if not args.no_cpu_baseline and not args.regen:
        import oracle
        # one more (untimed) step in a known direction, then the oracle on a sample of its buckets
        i_next = args.warmup + args.steps
        old_ws = versions[(i_next + 1) % 2]      # what the snapshot holds now
        new_ws = versions[i_next % 2]
        step(i_next)
        torch.cuda.synchronize()
        groups = 1 if args.tiny else args.cpu_groups
        bpg = min(16, plan.nbuckets)
        te, ta, elems, _ = cpu_baseline_and_check(torch, np, oracle, wl, old_ws, new_ws, (I, V, counts), bpg, groups)
        cpu = {"value": round(4.0 * elems / (te + ta) / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{elems} elements ({elems / N * 100:.1f}% of the workload) in groups of {bpg} buckets spread "
                         f"over the set; oracle extract {te:.2f}s + apply {ta:.2f}s, compute only"}
        # the same oracle on all host cores at once, disjoint bucket ranges (a one-GPU machine's share is 16 cores)
        ncpu = os.cpu_count() or 1
        cores = args.cpu_cores or min(ncpu, 16)
        if not args.tiny and cores > 1:
            wall, elems_mt, used, changed_mt = cpu_all_cores(torch, np, oracle, wl, old_ws, new_ws, cores, min(6, plan.nbuckets))
            cpu_mt = {"value": round(4.0 * elems_mt / wall / 1e9, 3), "unit": "GB/s", "cores": used, "kind": "oracle",
                      "host_cpus": ncpu,
                      "sample": f"{elems_mt} elements ({elems_mt / N * 100:.1f}% of the workload): {used} threads, each the "
                                f"unmodified oracle (extract + apply) on its own run of buckets; wall {wall:.2f}s, "
                                f"{changed_mt} changed elements found"}
            log(f"oracle on {used} threads (host reports {ncpu} CPUs): {cpu_mt['value']} GB/s of dense bytes scanned "
                f"against {cpu['value']} on one")

    default_run = not (args.tiny or args.density or args.tile or args.interleave or args.refresh_group >= 0
                       or args.index_coding or args.value_coding or args.rotate_snapshot or args.second_pass or args.regen
                       or args.config != 2)
    traffic = measured_traffic(wl.name) if default_run else None
    tr_e = traffic["extract"] if traffic else None
    tr_a = traffic["apply"] if traffic else None
    ach_a = bytes_apply / (app_avg * 1e-3) / 1e9

    # the other workloads of the family, each with the library defaults (the headline's buffers are released first)
    others = None
    if default_run and not args.no_other_configs:
        for pl in plans:
            pl.close()
        ctx.close()
        plans, ctx = [], None
        # every name that still holds (a view of) the headline's buffers
        W0 = W1 = S = R = I = V = counts = versions = pairs = rolls = plan = last_new = None
        a = b = sink = old_ws = new_ws = None
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        free_b, total_b = torch.cuda.mem_get_info()
        log(f"headline buffers released: {free_b / 2**30:.0f} of {total_b / 2**30:.0f} GiB free")
        others = {}
        others.update(measure_other_config(args, torch, srs, synth, 1, [0.01], 3, dev))
        others.update(measure_other_config(args, torch, srs, synth, 3, [None], 2, dev))
        others.update(measure_other_config(args, torch, srs, synth, 4, [0.001, 0.01, 0.1], 3, dev))

    out = {
        "metric": "extract+apply dense GB/s scanned",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16",
        "data": "synthetic",
        "config": {"workload": wl.name, "elements": N, "buckets": nbuckets, "bucket_elems": wl.bucket_elems,
                   "changed_fraction": round(rho, 6), "payload_cap": cap, "tile_elems": args.tile or 32768,
                   "index_coding": bool(args.index_coding),
                   "snapshot": "rotate" if args.rotate_snapshot else "refresh-second-pass" if args.second_pass
                               else "refresh-in-place"},
        "sync_ms": round(ms_per_step, 4),
        "extract_ms": round(ext_avg, 4),
        "apply_ms": round(app_avg, 4),
        "pct_hbm_peak_combined": round(100 * combined / HBM_PEAK_GBS, 2),
        "pct_hbm_peak_extract": round(100 * ach / HBM_PEAK_GBS, 2),
        "read_probe_gbs": None if probe_gbs is None else round(probe_gbs, 1),
        # dominant kernel.  achieved = algorithmic bytes (4 + 8 rho) N per launch / HIP-event time of the launch;
        # traffic = L2 <-> fabric bytes per launch from the tracked counter summary (nothing is read twice; the
        # excess is the snapshot's changed lines written whole, the cheaper way to write them)
        "roofline": {"bound": "hbm", "kernel": "extract_kernel", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                     "traffic": None if tr_e is None else tr_e[0] + tr_e[1],
                     "traffic_read": None if tr_e is None else tr_e[0],
                     "traffic_written": None if tr_e is None else tr_e[1]},
        # the scatter: algorithmic bytes 8 rho N (payload read + 2 bytes written per pair); `traffic` as above.
        # line_model_gbs prices what the memory side has to do for iid changes -- payload read + read-modify-write
        # of every 128-byte line that holds a change -- and is a model, not a measurement
        "roofline_apply": {"bound": "hbm", "kernel": "apply_kernel", "achieved": round(ach_a, 1), "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": round(ach_a / HBM_PEAK_GBS, 4),
                           "traffic": None if tr_a is None else tr_a[0] + tr_a[1],
                           "traffic_read": None if tr_a is None else tr_a[0],
                           "traffic_written": None if tr_a is None else tr_a[1],
                           "line_model_gbs": round((6.0 * rho * N + 2 * 128.0 * (N / 64.0) * (1.0 - (1.0 - rho) ** 64)) / (app_avg * 1e-3) / 1e9, 1)},
        "cpu_baseline": cpu,
        "cpu_baseline_all_cores": cpu_mt,
        "rotating_snapshot": rotating,
        "other_configs": others,
        "checked": not args.no_check,
    }
    print(json.dumps(out), flush=True)
    for pl in plans:
        pl.close()
    if ctx is not None:
        ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
