"""GPU parity for the value entropy coding (Sec. 3.3): srs_encode_values / srs_decode_values against the oracle,
bit for bit (code lengths, low bytes, every used stream word, chunk sizes, sub-block offsets, decoded values)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth

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


def to_dev(a, dtype):
    return torch.from_numpy(a.view(dtype).copy()).to(DEV)


def check_stream(enc_g, want, counts, cap):
    nb = len(counts)
    g = {k: v.cpu().numpy() for k, v in enc_g.items()}
    assert np.array_equal(g["lens"].view(np.uint8), want["lens"]), "code lengths"
    cw = g["chunk_words"].view(np.uint32)
    assert np.array_equal(cw, want["chunk_words"]), "chunk sizes"
    bits = g["bits"].view(np.uint32); sub = g["sub"].view(np.uint16); low = g["low"].view(np.uint8)
    for b in range(nb):
        c = min(int(counts[b]), cap)
        assert np.array_equal(low[b, :c], want["low"][b, :c]), f"low bytes of bucket {b}"
        assert np.all(low[b, c:] == 0xFF), "low bytes beyond the count were written"
        for k in range(cw.shape[1]):
            u = int(cw[b, k])
            assert np.array_equal(bits[b, k, :u], want["bits"][b, k, :u]), f"stream words of bucket {b} chunk {k}"
            nsub = (min(2048, c - k * 2048) + 63) // 64 if c > k * 2048 else 0
            assert np.array_equal(sub[b, k, :nsub], want["sub"][b, k, :nsub]), f"sub offsets of bucket {b} chunk {k}"


CASES = [
    ("normal", [5000, 0, 1, 2049, 4096, 4999], 5000),
    ("any", [3000, 3000], 3000),
    ("one-symbol", [2500, 64, 65], 2500),
    ("fibonacci", [46367], 46368),
    ("normal", [100000, 99999], 100000),
]


@pytest.mark.parametrize("kind,counts,cap", CASES)
def test_encode_and_decode_match_oracle(srs, ctx, kind, counts, cap):
    print(f"case kind={kind} counts={counts} cap={cap}", flush=True)
    rng = np.random.default_rng(cap + len(kind))
    nb = len(counts)
    counts = np.array(counts, np.uint32)
    if kind == "normal":
        x = (rng.standard_normal(nb * cap) * 0.02).astype(np.float32)
        V = (x.view(np.uint32) >> 16).astype(np.uint16).reshape(nb, cap)
    elif kind == "any":
        V = rng.integers(0, 1 << 16, size=(nb, cap), dtype=np.uint16)
    elif kind == "one-symbol":
        V = (rng.integers(0, 256, size=(nb, cap), dtype=np.uint16)) | 0x3C00
    else:
        f = [1, 1]
        while len(f) < 23:
            f.append(f[-1] + f[-2])
        hi = np.repeat(np.arange(23, dtype=np.uint16) + 40, f)[:cap]
        rng.shuffle(hi)
        V = ((hi << 8) | rng.integers(0, 256, size=hi.size, dtype=np.uint16)).reshape(1, -1)
        V = np.pad(V, ((0, 0), (0, cap - V.shape[1])))
    want = oracle.encode_values(V, counts)
    d_V = to_dev(V, np.int16); d_counts = to_dev(counts, np.int32)
    enc = srs.alloc_value_stream(nb, cap, DEV)
    ctx.encode_values(d_V, d_counts, nb, cap, enc)
    assert ctx.status() == 0
    check_stream(enc, want, counts, cap)
    V_out = torch.full((nb, cap), -1, dtype=torch.int16, device=DEV)
    ctx.decode_values(enc, d_counts, nb, cap, V_out)
    assert ctx.status() == 0
    got = V_out.cpu().numpy().view(np.uint16)
    for b in range(nb):
        c = int(counts[b])
        assert np.array_equal(got[b, :c], V[b, :c]), f"decoded values of bucket {b}"
        assert np.all(got[b, c:] == 0xFFFF)


def test_payload_of_a_workload_round_trips_through_both_codings(srs, ctx):
    """extract -> index coding + value coding -> decode -> encoded apply: the receiver ends bit-identical."""
    wl = synth.workload(2, tiny=True)
    a = synth.WeightSet(wl, DEV); b = synth.WeightSet(wl, DEV); r = synth.WeightSet(wl, DEV)
    synth.fill_base(a, 61); synth.make_update(b, a, 61); r.copy_from(a)
    plan = ctx.plan(a.numels, wl.bucket_elems)
    cap = wl.bucket_elems
    I, V, counts = srs.alloc_payload(plan.nbuckets, cap, DEV)
    ctx.extract_multi(plan, a.tensors, b.tensors, I, V, counts, cap)
    D, mg, an = srs.alloc_encoded(plan.nbuckets, cap, DEV)
    ctx.encode_indices(I, counts, plan.nbuckets, cap, 0, D, mg, an)
    enc = srs.alloc_value_stream(plan.nbuckets, cap, DEV)
    ctx.encode_values(V, counts, plan.nbuckets, cap, enc)
    V2 = torch.full_like(V, -1)
    ctx.decode_values(enc, counts, plan.nbuckets, cap, V2)
    ctx.apply_multi_encoded(plan, r.tensors, D, I, V2, counts, mg, an, cap)
    assert ctx.status() == 0
    plan.close()
    assert r.equal(b)


def test_corrupt_stream_is_flagged(srs, ctx):
    rng = np.random.default_rng(1)
    cap = 4096
    V = ((rng.integers(0, 4, size=(1, cap), dtype=np.uint16) + 0x3B) << 8) | rng.integers(0, 256, size=(1, cap), dtype=np.uint16)
    counts = np.array([cap], np.uint32)
    d_V = to_dev(V, np.int16); d_counts = to_dev(counts, np.int32)
    enc = srs.alloc_value_stream(1, cap, DEV)
    ctx.encode_values(d_V, d_counts, 1, cap, enc)
    assert ctx.status() == 0
    enc["lens"][0, 0x3B] = 0                         # a code word of the stream is no longer in the table
    V_out = torch.full((1, cap), -1, dtype=torch.int16, device=DEV)
    ctx.decode_values(enc, d_counts, 1, cap, V_out)
    assert ctx.status() == srs.FLAG_BAD_INDEX
