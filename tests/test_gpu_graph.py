"""extract + apply captured into a HIP graph: every replay must equal the eager result on fresh data.
(The library clears its ticket counters and tile status words with a kernel that is part of the stream's
work, so a replay does not depend on host-side state; scratch is sized by an eager warm-up call first.)"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth
from util import assert_payload_equal, payload_to_host

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("snapshot_mode", [0, 2])      # refreshed inside the scan / by a second pass of the same call
def test_graph_replays_match_eager_and_oracle(snapshot_mode):
    from paper_2605_07330_amd import srs
    wl = synth.workload(2, tiny=True)
    base = synth.WeightSet(wl, DEV); S = synth.WeightSet(wl, DEV); R = synth.WeightSet(wl, DEV); new = synth.WeightSet(wl, DEV)
    synth.fill_base(base, 91)
    ctx = srs.Context(0)
    try:
        ctx.set_option(srs.OPT_SNAPSHOT, snapshot_mode)
        plan = ctx.plan(base.numels, wl.bucket_elems)
        cap = wl.bucket_elems
        I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
        pairs = ctx.bind_pairs(plan, S.tensors, new.tensors)
        rolls = ctx.bind_weights(plan, R.tensors)
        # eager warm-up: sizes the scratch arrays and uploads the pointer tables
        S.copy_from(base); R.copy_from(base); synth.make_update(new, base, 91, step=1)
        ctx.extract_multi(plan, None, None, I, V, counts, cap, pairs=pairs)
        ctx.apply_multi(plan, None, I, V, counts, cap, tensors=rolls)
        assert ctx.status() == 0
        torch.cuda.synchronize()

        g = torch.cuda.CUDAGraph()
        S.copy_from(base); R.copy_from(base)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            ctx.extract_multi(plan, None, None, I, V, counts, cap, pairs=pairs)
            ctx.apply_multi(plan, None, I, V, counts, cap, tensors=rolls)
        for rep in range(2, 7):
            # the program's own eager work between replays: new inputs, cleared outputs
            S.copy_from(base); R.copy_from(base)
            nchanged, _ = synth.make_update(new, base, 91, step=rep)
            I.fill_(-1); V.fill_(-1); counts.zero_()
            torch.cuda.synchronize()
            want = oracle.extract_multi(base.to_numpy_u16(), new.to_numpy_u16(), base.numels, wl.bucket_elems)[:3]
            g.replay()
            torch.cuda.synchronize()
            assert ctx.status() == 0
            assert_payload_equal(payload_to_host(I, V, counts), want, f"replay {rep}")
            assert int(want[2].sum()) == nchanged
            assert S.equal(new) and R.equal(new), f"replay {rep}: weights"
        plan.close()
    finally:
        ctx.close()
