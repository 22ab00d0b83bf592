"""GPU parity of srs_tensor_indices (the per-tensor view of a list payload, Alg. 2's own index) against the oracle,
element by element, and against the definition directly: per tensor, the view lists flatnonzero(old != new)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth
from util import from_u16, payload_to_host

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def srs():
    from paper_2605_07330_amd import srs as m
    return m


def run(srs, numel, be, olds, news, cap):
    ctx = srs.Context(0)
    try:
        plan = ctx.plan(numel, be)
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        tid = torch.full((plan.nbuckets, cap), -1, dtype=torch.int32, device=DEV)
        tix = torch.full((plan.nbuckets, cap), -1, dtype=torch.int32, device=DEV)
        ctx.extract_multi(plan, [from_u16(o, DEV) for o in olds], [from_u16(w, DEV) for w in news], I, V, counts, cap)
        ctx.tensor_indices(plan, I, counts, cap, tid, tix)
        flags = ctx.status()
        plan.close()
    finally:
        ctx.close()
    return payload_to_host(I, V, counts), tid.cpu().numpy().view(np.uint32), tix.cpu().numpy(), flags


@pytest.mark.parametrize("numel,be,density", [
    ([5, 1, 1, 20, 3], 7, 0.5), ([100, 0, 50, 0, 0, 25], 64, 0.3), ([4096] * 3 + [1, 70000], 8192, 0.05),
    ([40000, 7, 40000, 9, 16385], 16384, 0.2), ([700001, 3, 1200000, 50, 999999], 1300, 0.01),   # 2231 buckets
    ([300000] + [17] * 400 + [300000], 100000, 0.1),                                              # > 128 segments in a bucket
])
def test_matches_oracle_and_definition(srs, numel, be, density):
    print(f"case tensor view numel[:5]={numel[:5]} ntensors={len(numel)} be={be}", flush=True)
    rng = np.random.default_rng(sum(numel) + be)
    olds = [rng.integers(0, 1 << 16, size=m, dtype=np.uint16) for m in numel]
    news = []
    for o in olds:
        w = o.copy()
        w[rng.random(o.size) < density] ^= np.uint16(0x0101)
        news.append(w)
    cap = be
    (I, V, counts), tid, tix, flags = run(srs, numel, be, olds, news, cap)
    assert flags == 0
    wid, wix, rc = oracle.tensor_indices(I, counts, numel, be)
    assert rc == oracle.OK
    assert np.array_equal(tid, wid) and np.array_equal(tix, wix)          # including the untouched slots
    ids = np.concatenate([tid[b, :counts[b]] for b in range(counts.size)])
    idx = np.concatenate([tix[b, :counts[b]] for b in range(counts.size)])
    for k, (o, w) in enumerate(zip(olds, news)):
        assert np.array_equal(idx[ids == k], np.flatnonzero(o != w)), f"tensor {k}"


def test_tiny_model_shape_and_capacity(srs):
    wl = synth.workload(2, tiny=True)
    A = synth.WeightSet(wl, DEV); B = synth.WeightSet(wl, DEV)
    synth.fill_base(A, 3)
    synth.make_update(B, A, 3)
    numel, be, cap = A.numels, wl.bucket_elems, 40                       # cap below some buckets' counts
    (I, V, counts), tid, tix, flags = run(srs, numel, be, A.to_numpy_u16(), B.to_numpy_u16(), cap)
    assert flags == srs.FLAG_OVERFLOW and int(counts.max()) > cap
    wid, wix, rc = oracle.tensor_indices(I, counts, numel, be)          # counts above cap are read as cap
    assert rc == oracle.OK and np.array_equal(tid, wid) and np.array_equal(tix, wix)


def test_position_outside_its_bucket_is_flagged(srs):
    numel, be, cap = [1000, 2000, 500], 1024, 64
    ctx = srs.Context(0)
    try:
        plan = ctx.plan(numel, be)
        I = torch.zeros((plan.nbuckets, cap), dtype=torch.int32, device=DEV)
        counts = torch.full((plan.nbuckets,), 2, dtype=torch.int32, device=DEV)
        I[:, 1] = 5
        I[3, 1] = 428                                                    # last bucket holds 3500 - 3*1024 = 428 elements
        tid = torch.full((plan.nbuckets, cap), -1, dtype=torch.int32, device=DEV); tix = tid.clone()
        ctx.tensor_indices(plan, I, counts, cap, tid, tix)
        assert ctx.status() == srs.FLAG_BAD_INDEX
        wid, wix, rc = oracle.tensor_indices(I.cpu().numpy(), counts.cpu().numpy().view(np.uint32), numel, be)
        assert rc == oracle.BAD_INDEX
        assert np.array_equal(tid.cpu().numpy().view(np.uint32), wid) and np.array_equal(tix.cpu().numpy(), wix)
        plan.close()
    finally:
        ctx.close()
